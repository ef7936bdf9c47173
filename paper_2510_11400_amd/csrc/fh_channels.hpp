// Where an element of a [outer][channels][inner] tensor lives, and whether its channel is
// kept verbatim beside the quantised stream (salient channels, paper Section 4.4.1) --
// shared by the forward and the backward kernels of the mixed path.
//
// A wave finds the (sample, channel, position) of its first element once, with scalar
// arithmetic; lanes then only add offsets below 2^12 and divide by comparing or by one
// multiply.  Element counts are limited to 2^31 so that all of it is 32-bit.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "fh_device.hpp"

namespace fh {

// floor(n / d) for every 32-bit n and a divisor fixed on the host (division by an
// invariant through multiplication: with s = ceil(log2 d) and
// m = floor(2^32 * (2^s - d) / d) + 1,  n / d = (t + ((n - t) >> min(s,1))) >> max(s-1,0),
// t = mulhi(m, n)).
struct ExactDiv {
    uint32_t d, m, sh1, sh2;
};
inline ExactDiv make_exact_div(uint32_t d)
{
    uint32_t s = 0;
    while (s < 32 && ((uint64_t)1 << s) < d) ++s;
    ExactDiv v;
    v.d = d;
    v.m = (uint32_t)((((uint64_t)1 << 32) * (((uint64_t)1 << s) - d)) / d + 1u);
    v.sh1 = s < 1 ? s : 1;
    v.sh2 = s > 1 ? s - 1 : 0;
    return v;
}
__device__ __forceinline__ uint32_t div_exact(uint32_t n, const ExactDiv& v)
{
    const uint32_t t = __umulhi(v.m, n);
    return (t + ((n - t) >> v.sh1)) >> v.sh2;
}

// floor(n / d) for small dividends: n < d + 4096 and n < 2^17.  magic = floor(2^32 / d) + 1
// is exact while n * d < 2^32, which covers every d below 2^15; larger divisors can only
// give 0 or 1.
struct SmallDiv {
    uint32_t d, magic;
};
inline SmallDiv make_small_div(uint32_t d)
{
    SmallDiv v;
    v.d = d;
    v.magic = d >= 2u ? (uint32_t)(((uint64_t)1 << 32) / d) + 1u : 0u;
    return v;
}
__device__ __forceinline__ uint32_t div_small(uint32_t n, const SmallDiv& v)
{
    if (v.d == 1u) return n;                                  // branches on the divisor are wave-uniform
    if (v.d >= 32768u) return n >= v.d ? 1u : 0u;
    return __umulhi(n, v.magic);
}

struct ChannelMap {
    const int16_t* slots;      // device, [channels]: raw-store row of a kept channel, anything else = normal
    void*          raw;        // device, [outer][raw_channels][inner] elements of the tensor's dtype
    uint32_t       raw_channels;
    ExactDiv       inner_exact, channels_exact;
    SmallDiv       inner, channels;
};

struct ElemPos {
    uint32_t o, c, pos;        // sample, channel, index inside the channel's run of `inner` elements
};

// position of the element `index` (wave-uniform: compiles to scalar instructions)
__device__ __forceinline__ ElemPos locate_base(const ChannelMap& cm, uint32_t index)
{
    const uint32_t run = div_exact(index, cm.inner_exact);
    ElemPos p;
    p.pos = index - run * cm.inner.d;
    p.o = div_exact(run, cm.channels_exact);
    p.c = run - p.o * cm.channels.d;
    return p;
}
// position of the element `off` (< 4096) after `p`
__device__ __forceinline__ ElemPos advance(const ChannelMap& cm, const ElemPos& p, uint32_t off)
{
    const uint32_t t = p.pos + off;
    const uint32_t runs = div_small(t, cm.inner);
    const uint32_t cc = p.c + runs;
    const uint32_t wraps = div_small(cc, cm.channels);
    ElemPos q;
    q.pos = t - runs * cm.inner.d;
    q.c = cc - wraps * cm.channels.d;
    q.o = p.o + wraps;
    return q;
}

__device__ __forceinline__ bool kept(const ChannelMap& cm, int16_t slot)
{
    return (uint32_t)(int32_t)slot < cm.raw_channels;         // negative slots wrap to huge values
}

// Bit j set iff element j of the N consecutive elements starting at p belongs to a kept
// channel.  N = 4 or 8; the first element's index is a multiple of N.
template <int N>
__device__ __forceinline__ uint32_t kept_mask(const ChannelMap& cm, const ElemPos& p)
{
    if (cm.raw_channels == 0u) return 0u;
    uint32_t mask = 0u;
    if (cm.inner.d == 1u && (cm.channels.d & (N - 1)) == 0u) {
        // one channel per element, and the N channels of a lane never wrap: one vector load
        if constexpr (N == 8) {
            const u32x4 s = *reinterpret_cast<const u32x4*>(cm.slots + p.c);
            const uint32_t w[4] = {s.x, s.y, s.z, s.w};
#pragma unroll
            for (int j = 0; j < 8; ++j)
                mask |= kept(cm, (int16_t)(w[j >> 1] >> ((j & 1) * 16))) ? 1u << j : 0u;
        } else {
            const u32x2 s = *reinterpret_cast<const u32x2*>(cm.slots + p.c);
            const uint32_t w[2] = {s.x, s.y};
#pragma unroll
            for (int j = 0; j < 4; ++j)
                mask |= kept(cm, (int16_t)(w[j >> 1] >> ((j & 1) * 16))) ? 1u << j : 0u;
        }
        return mask;
    }
    const bool straddles = p.pos + N > cm.inner.d;
    if (__builtin_amdgcn_ballot_w64(straddles) == 0ull)       // the usual case for feature maps
        return kept(cm, cm.slots[p.c]) ? (1u << N) - 1u : 0u;
#pragma unroll
    for (int j = 0; j < N; ++j) {
        const ElemPos q = advance(cm, p, j);
        mask |= kept(cm, cm.slots[q.c]) ? 1u << j : 0u;
    }
    return mask;
}

// index into the raw store of element j after p (whose channel must be kept)
__device__ __forceinline__ uint64_t raw_index(const ChannelMap& cm, const ElemPos& p, uint32_t j)
{
    const ElemPos q = advance(cm, p, j);
    const uint32_t slot = (uint32_t)(int32_t)cm.slots[q.c];
    return ((uint64_t)q.o * cm.raw_channels + slot) * cm.inner.d + q.pos;
}

}  // namespace fh
