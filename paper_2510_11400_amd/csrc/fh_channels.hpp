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
    const uint64_t* rows_in_use;  // device, or null: raw-store rows in use; 0 there = no channel of this tensor is kept
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

// Does the caller's count say that nothing is kept?  (wave-uniform: one scalar load)
__device__ __forceinline__ bool nothing_kept(const ChannelMap& cm)
{
    return cm.rows_in_use != nullptr && *cm.rows_in_use == 0u;
}

__device__ __forceinline__ bool kept(const ChannelMap& cm, int16_t slot)
{
    return (uint32_t)(int32_t)slot < cm.raw_channels;         // negative slots wrap to huge values
}

// What a lane knows about its run of N consecutive elements (N = 4 or 8; the first element's
// index is a multiple of N).
template <int N> struct KeptRun {
    ElemPos  p;                // position of the first element
    uint32_t mask;             // bit j set iff element j belongs to a kept channel
    uint32_t slotw[N / 2];     // half-word j: raw-store row of element j (meaningful where bit j is set)
};

// The runs of one lane in the ROWS rows of a wave's span (row r starts row_stride * r elements
// after wave_pos; the lane's run starts lane_off into the row).  All table loads are issued
// before any of them is needed, so a wave pays one memory latency, not one per row.
template <int ROWS, int N>
__device__ __forceinline__ void kept_runs(const ChannelMap& cm, const ElemPos& wave_pos, uint32_t lane_off,
                                          uint32_t row_stride, KeptRun<N> (&run)[ROWS])
{
#pragma unroll
    for (int r = 0; r < ROWS; ++r) {
        run[r].p = advance(cm, wave_pos, r * row_stride + lane_off);
        run[r].mask = 0u;
#pragma unroll
        for (int k = 0; k < N / 2; ++k) run[r].slotw[k] = 0xffffffffu;
    }
    if (cm.raw_channels == 0u) return;
    if (cm.inner.d == 1u && (cm.channels.d & (N - 1)) == 0u) {
        // one channel per element, and the N channels of a lane never wrap: one vector load
#pragma unroll
        for (int r = 0; r < ROWS; ++r) {
            if constexpr (N == 8) {
                const u32x4 s = *reinterpret_cast<const u32x4*>(cm.slots + run[r].p.c);
                run[r].slotw[0] = s.x; run[r].slotw[1] = s.y; run[r].slotw[2] = s.z; run[r].slotw[3] = s.w;
            } else {
                const u32x2 s = *reinterpret_cast<const u32x2*>(cm.slots + run[r].p.c);
                run[r].slotw[0] = s.x; run[r].slotw[1] = s.y;
            }
        }
#pragma unroll
        for (int r = 0; r < ROWS; ++r)
#pragma unroll
            for (int j = 0; j < N; ++j)
                run[r].mask |= kept(cm, (int16_t)(run[r].slotw[j >> 1] >> ((j & 1) * 16))) ? 1u << j : 0u;
        return;
    }
    uint32_t first[ROWS];
    bool straddles = false;
#pragma unroll
    for (int r = 0; r < ROWS; ++r) {
        first[r] = (uint16_t)cm.slots[run[r].p.c];
        straddles |= run[r].p.pos + N > cm.inner.d;
    }
#pragma unroll
    for (int r = 0; r < ROWS; ++r) {
        run[r].mask = kept(cm, (int16_t)first[r]) ? (1u << N) - 1u : 0u;
#pragma unroll
        for (int k = 0; k < N / 2; ++k) run[r].slotw[k] = first[r] * 0x10001u;
    }
    if (__builtin_amdgcn_ballot_w64(straddles) != 0ull) {     // rare for feature maps
#pragma unroll
        for (int r = 0; r < ROWS; ++r) {
            if (run[r].p.pos + N > cm.inner.d) {              // a channel ends inside this lane's run
                uint32_t m = 0u;
#pragma unroll
                for (int j = 0; j < N; ++j) {
                    const ElemPos q = advance(cm, run[r].p, j);
                    const uint32_t s = (uint16_t)cm.slots[q.c];
                    m |= kept(cm, (int16_t)s) ? 1u << j : 0u;
                    if (j & 1) run[r].slotw[j >> 1] = (run[r].slotw[j >> 1] & 0xffffu) | (s << 16);
                    else run[r].slotw[j >> 1] = (run[r].slotw[j >> 1] & 0xffff0000u) | s;
                }
                run[r].mask = m;
            }
        }
    }
}

// ---- one channel per element --------------------------------------------------------------
// With inner == 1, channels a multiple of N and at most 16384 raw-store rows, the N channels of
// a lane's run never wrap and their table entries are one vector load; what the lane needs then
// comes out of packed 16-bit arithmetic on the entry pairs, with no branch and no per-element
// compare: an entry s names a row iff 0 <= s < raw_channels, i.e. iff bit 15 of ~s & (s - raw_channels)
// is set (s - raw_channels cannot wrap: both are below 2^15 in magnitude).
typedef int16_t i16x2 __attribute__((ext_vector_type(2)));
typedef uint16_t u16x2 __attribute__((ext_vector_type(2)));

template <int N> struct KeptVector {
    uint32_t keep[N / 2];      // half-word j: 0xffff iff element j belongs to a kept channel
    uint32_t slot[N / 2];      // half-word j: that channel's raw-store row times the element size, 0 for a normal channel
    uint32_t row;              // byte offset of (the run's sample, row 0) from the row 0 of the wave's first sample
};

template <int N>
__device__ __forceinline__ bool one_channel_per_element(const ChannelMap& cm)
{
    return cm.inner.d == 1u && (cm.channels.d & (N - 1)) == 0u && cm.raw_channels - 1u < 16384u;
}

// elem_shift: log2 of the raw store's element size (1 or 2; rows < 2^14, so the scaled rows fit 16 bits)
template <int ROWS, int N>
__device__ __forceinline__ void kept_vectors(const ChannelMap& cm, const ElemPos& wave_pos, uint32_t lane_off,
                                             uint32_t row_stride, uint32_t elem_shift, KeptVector<N> (&kv)[ROWS])
{
    uint32_t w[ROWS][N / 2];
#pragma unroll
    for (int r = 0; r < ROWS; ++r) {                          // all table loads first
        const ElemPos p = advance(cm, wave_pos, r * row_stride + lane_off);
        kv[r].row = ((p.o - wave_pos.o) * cm.raw_channels) << elem_shift;
        if constexpr (N == 8) {
            const u32x4 s = *reinterpret_cast<const u32x4*>(cm.slots + p.c);
            w[r][0] = s.x; w[r][1] = s.y; w[r][2] = s.z; w[r][3] = s.w;
        } else {
            const u32x2 s = *reinterpret_cast<const u32x2*>(cm.slots + p.c);
            w[r][0] = s.x; w[r][1] = s.y;
        }
    }
    const int16_t rows = (int16_t)cm.raw_channels;
    const i16x2 limit = {rows, rows};
#pragma unroll
    for (int r = 0; r < ROWS; ++r)
#pragma unroll
        for (int k = 0; k < N / 2; ++k) {
            const i16x2 s = __builtin_bit_cast(i16x2, w[r][k]);
            const i16x2 keep = (~s & (s - limit)) >> 15;      // arithmetic shift: 0xffff or 0 per half
            kv[r].keep[k] = __builtin_bit_cast(uint32_t, keep);
            const u16x2 scaled = __builtin_bit_cast(u16x2, w[r][k] & kv[r].keep[k]) << (uint16_t)elem_shift;
            kv[r].slot[k] = __builtin_bit_cast(uint32_t, scaled);
        }
}

// byte offset, from the raw-store row of the wave's first sample, of the entry element j of the run reads or writes
// (a normal element gets row 0 of its sample, which exists: raw_channels >= 1)
template <int N>
__device__ __forceinline__ uint32_t raw_offset(const KeptVector<N>& kv, int j)
{
    return ((j & 1) ? kv.slot[j >> 1] >> 16 : kv.slot[j >> 1] & 0xffffu) + kv.row;
}

// does any lane of the wave hold a kept element in this run? (a wave-uniform answer keeps the branch scalar)
template <int N>
__device__ __forceinline__ bool any_kept(const KeptVector<N>& kv)
{
    uint32_t any = 0;
#pragma unroll
    for (int k = 0; k < N / 2; ++k) any |= kv.keep[k];
    return __builtin_amdgcn_ballot_w64(any != 0u) != 0ull;
}

// index into the raw store of element j of the run (whose bit in run.mask must be set)
template <int N>
__device__ __forceinline__ uint64_t raw_index(const ChannelMap& cm, const KeptRun<N>& run, uint32_t j)
{
    const uint32_t slot = (run.slotw[j >> 1] >> ((j & 1u) * 16u)) & 0xffffu;
    if (cm.inner.d == 1u && (cm.channels.d & (N - 1)) == 0u)  // same sample for the whole run
        return (uint64_t)run.p.o * cm.raw_channels + slot;
    const ElemPos q = advance(cm, run.p, j);
    return ((uint64_t)q.o * cm.raw_channels + slot) * cm.inner.d + q.pos;
}

}  // namespace fh
