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

#include "fh_types.hpp"

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
    SmallDiv       inner, channels, raw_div;   // raw_div: by raw_channels (1 when there are none)
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

// ---- one channel per element: the kept elements of a span, listed by raw-store row -----------
// With inner == 1 a raw-store row holds one element per sample, and the kept elements of a
// wave's span are few and scattered (a few per cent of the channels).  Instead of every lane
// testing each of its elements, the workgroup lists once which channel each raw-store row keeps
// (`rows`: LDS, uint16 per row, kNoChannel for a row that keeps none; two channels must not name
// the same row), and the lanes of a wave walk the (sample, row) pairs of the span: the element's
// position follows from the pair by one multiply-add, and the raw-store side of consecutive
// lanes is contiguous.  The wave's elements themselves pass through LDS once, where the pairs
// read or patch them.
constexpr uint32_t kListedRows = 2048;                        // raw-store rows the list has room for
constexpr uint32_t kNoChannel = 0xffffu;                      // channels are below 2^14

__device__ __forceinline__ bool rows_listed(const ChannelMap& cm)
{
    return cm.inner.d == 1u && cm.raw_channels - 1u < kListedRows;
}

// The list is built in two steps so that a kernel can put its own loads between them: the table entries a
// thread is responsible for are requested first (two channels per 4-byte load, the first kSlotRounds * 2 * THREADS
// channels), and filed once they have arrived.  An entry names a row iff, read as an unsigned 16-bit number, it is
// below raw_channels (<= 2048: negative entries read as 32768 or more).  Every thread of the workgroup calls both;
// the second ends with a barrier.
constexpr int kSlotRounds = 8;
struct SlotWords { uint32_t w[kSlotRounds]; };

template <int THREADS>
__device__ __forceinline__ void list_rows_request(const ChannelMap& cm, SlotWords& words)
{
    const uint32_t C = cm.channels.d;
    const uint32_t* table = reinterpret_cast<const uint32_t*>(cm.slots);   // 16-byte aligned
#pragma unroll
    for (int k = 0; k < kSlotRounds; ++k) {
        const uint32_t c = 2u * (threadIdx.x + k * THREADS);
        words.w[k] = 0xffffffffu;
        if (2u * k * THREADS >= C) continue;                  // workgroup-uniform
        if (c + 1u < C) words.w[k] = table[c >> 1];
        else if (c < C) words.w[k] = 0xffff0000u | (uint16_t)cm.slots[c];  // an odd channel count's last entry
    }
}

template <int THREADS>
__device__ __forceinline__ void list_rows_file(const ChannelMap& cm, const SlotWords& words, uint16_t* rows)
{
    for (uint32_t s = threadIdx.x; s < cm.raw_channels; s += THREADS) rows[s] = (uint16_t)kNoChannel;
    __syncthreads();
    const uint32_t C = cm.channels.d, R = cm.raw_channels;
#pragma unroll
    for (int k = 0; k < kSlotRounds; ++k) {
        const uint32_t c = 2u * (threadIdx.x + k * THREADS);
        if (2u * k * THREADS >= C) break;                     // workgroup-uniform
        const uint32_t lo = words.w[k] & 0xffffu, hi = words.w[k] >> 16;
        if (lo < R) rows[lo] = (uint16_t)c;
        if (hi < R) rows[hi] = (uint16_t)(c + 1u);
    }
    for (uint32_t c = 2u * kSlotRounds * THREADS + threadIdx.x; c < C; c += THREADS) {   // beyond 4096 channels
        const uint32_t s = (uint16_t)cm.slots[c];
        if (s < R) rows[s] = (uint16_t)c;
    }
    __syncthreads();
}

// The (sample, row) pairs a wave's span of `span` elements can hold: `samples` samples starting at the
// first element's, each with raw_channels rows.  pairs <= span + 2 * raw_channels <= 6144.
__device__ __forceinline__ uint32_t span_pairs(const ChannelMap& cm, const ElemPos& wave_pos, uint32_t span)
{
    const uint32_t samples = div_exact(wave_pos.c + span - 1u, cm.channels_exact) + 1u;
    return samples * cm.raw_channels;
}

// A lane's walk over the pairs lane, lane + 64, lane + 128, ...: pair i is (sample i / raw_channels of the span,
// row i % raw_channels), kept up to date by additions (64 = q * raw_channels + r, so a step adds r to the row, q -- or
// q + 1 when the row wraps -- to the sample).  `u` is the offset inside the span of the sample's channel 0, so the
// pair's element sits at offset u + (the row's channel); a row that keeps no channel (kNoChannel = 65535) and a
// sample beyond the span's last both give an offset of `span` or more -- also when u is "negative", wrapped --, so
// that one comparison decides whether the pair is a kept element of this span.  The pair's index in the raw store,
// less that of (the span's first sample, row 0), is i itself.
struct PairWalk {
    uint32_t row, u;           // per lane
    uint32_t row_step, u_step; // wave-uniform
};

__device__ __forceinline__ PairWalk pair_walk(const ChannelMap& cm, const ElemPos& wave_pos, uint32_t lane)
{
    PairWalk p;
    const uint32_t t = div_small(lane, cm.raw_div);
    p.row = lane - t * cm.raw_channels;
    p.u = t * cm.channels.d - wave_pos.c;
    const uint32_t q = div_small(64u, cm.raw_div);
    p.row_step = 64u - q * cm.raw_channels;
    p.u_step = q * cm.channels.d;
    return p;
}

// offset inside the span of the current pair's element (>= span: not a kept element of this span); `rows` as listed
__device__ __forceinline__ uint32_t pair_offset(const PairWalk& p, const uint16_t* rows) { return p.u + rows[p.row]; }

__device__ __forceinline__ void pair_advance(const ChannelMap& cm, PairWalk& p)
{
    p.row += p.row_step;
    p.u += p.u_step;
    const bool wrap = p.row >= cm.raw_channels;
    p.row = wrap ? p.row - cm.raw_channels : p.row;
    p.u = wrap ? p.u + cm.channels.d : p.u;
}

// A lane's first kPairsAhead pairs, worked out before the span's data is needed; leaves the walk at the next pair.
constexpr int kPairsAhead = 4;
__device__ __forceinline__ void first_pairs(const ChannelMap& cm, PairWalk& p, const uint16_t* rows, uint32_t pairs,
                                            uint32_t (&off)[kPairsAhead])
{
#pragma unroll
    for (int k = 0; k < kPairsAhead; ++k) {
        off[k] = 0xffffffffu;
        if (k * 64u >= pairs) continue;                       // wave-uniform
        off[k] = pair_offset(p, rows);
        pair_advance(cm, p);
    }
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
