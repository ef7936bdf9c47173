// Channel classification on gfx950: outliers by the k-sigma rule, counted per channel
// (paper Section 4.4.1: outliers are found with the empirical three-sigma rule and
// channels are sorted into salient and normal ones).  Contract and definition:
// include/fedhybrid.h.
//
// Two streaming passes over the tensor:
//   1. moments: pairwise binary64 sums of x and x*x.  The balanced tree of the
//      definition is walked in 1024-element spans (one per wave): inside a lane over its
//      consecutive elements, across the 64 lanes by xor 1, 2, 4, ... 32, across the rows of
//      the span, and then across spans by the same routine applied to the partial sums
//      (1024 partials per wave) until one pair is left.  Binary64 addition is commutative,
//      so a butterfly exchange forms exactly the tree's nodes; partial sums of different
//      rows and of the two moments are spread over the lanes (reduce-scatter) so that
//      each exchange level handles half of what the level before did.
//   2. count: d = (double)x - mean, outlier iff d*d > threshold; outliers are rare, so
//      each lane keeps a bit mask of its 16 elements and only set bits pay for the
//      channel index (division by invariant integers through multiply-high) and an LDS
//      histogram increment; the histogram is flushed with one global atomic per
//      non-zero bin and workgroup.
#include "../../include/fedhybrid.h"

#include "fh_batch.hpp"
#include "fh_channels.hpp"
#include "fh_device.hpp"

#include <limits.h>

#include <mutex>

namespace fh {
namespace {

constexpr int kSpan = 1024;              // elements (or partial sums) per wave
constexpr int kThreads = 256;
constexpr int kWavesPerBlock = kThreads / kWave;
constexpr int kMaxChannels = 16384;

typedef double f64x2 __attribute__((ext_vector_type(2)));

// ---- lane exchanges of a double ------------------------------------------------------
template <int CTRL>
__device__ __forceinline__ double dpp_f64(double v)
{
    const uint64_t u = __builtin_bit_cast(uint64_t, v);
    const uint32_t lo = (uint32_t)__builtin_amdgcn_mov_dpp((int)(uint32_t)u, CTRL, 0xF, 0xF, true);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_mov_dpp((int)(uint32_t)(u >> 32), CTRL, 0xF, 0xF, true);
    return __builtin_bit_cast(double, ((uint64_t)hi << 32) | lo);
}
// ds_swizzle in bit-mask mode: lane l reads lane (l & 0x1f) ^ XOR inside its half
template <int XOR>
__device__ __forceinline__ double swizzle_f64(double v)
{
    constexpr int pattern = (XOR << 10) | 0x1F;
    const uint64_t u = __builtin_bit_cast(uint64_t, v);
    const uint32_t lo = (uint32_t)__builtin_amdgcn_ds_swizzle((int)(uint32_t)u, pattern);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_ds_swizzle((int)(uint32_t)(u >> 32), pattern);
    return __builtin_bit_cast(double, ((uint64_t)hi << 32) | lo);
}
template <int XOR>
__device__ __forceinline__ double from_lane_xor(double v)
{
    if constexpr (XOR == 1) return dpp_f64<0xB1>(v);        // quad_perm [1,0,3,2]
    else if constexpr (XOR == 2) return dpp_f64<0x4E>(v);   // quad_perm [2,3,0,1]
    else return swizzle_f64<XOR>(v);                          // 4, 8, 16
}
// v[l] + v[l ^ 32]: permlane32_swap of two copies returns {lo half, lo half} and
// {hi half, hi half}; their sum is the same in both halves.
__device__ __forceinline__ double add_across_halves(double v)
{
    const uint64_t u = __builtin_bit_cast(uint64_t, v);
    uint32_t a0 = (uint32_t)u, a1 = (uint32_t)(u >> 32), b0 = a0, b1 = a1;
    asm volatile("" : "+v"(b0), "+v"(b1));
    const u32x2 r0 = __builtin_amdgcn_permlane32_swap(a0, b0, false, false);
    const u32x2 r1 = __builtin_amdgcn_permlane32_swap(a1, b1, false, false);
    const uint32_t f0 = r0.x, s0 = r0.y, f1 = r1.x, s1 = r1.y;
    const double first = __builtin_bit_cast(double, ((uint64_t)f1 << 32) | f0);
    const double second = __builtin_bit_cast(double, ((uint64_t)s1 << 32) | s0);
    return first + second;
}

// ---- the span tree ---------------------------------------------------------------------
// In: for each of ROWS rows, the lane's own subtree sums a[r] (of x) and b[r] (of x*x);
// a row is 64 lanes in element order.  Out (all lanes): the span's two sums.
// Exchange levels, in the tree's order:
//   xor 1   keep the rows whose low bit equals the lane's bit 0        (ROWS == 4 only)
//   xor 2   keep the row whose high bit equals the lane's bit 1 (ROWS == 4), or the row
//           whose index equals bit 0 moved here (ROWS == 2: done at xor 1)
//   next    keep one of the two moments
//   rest    plain butterflies
// followed by the levels that join the rows.
template <int ROWS>
__device__ __forceinline__ void span_tree(const double (&a)[ROWS], const double (&b)[ROWS], uint32_t lane,
                                          double& s1, double& s2)
{
    static_assert(ROWS == 2 || ROWS == 4, "rows per span");
    const bool b0 = lane & 1u, b1 = lane & 2u, b2 = lane & 4u;
    double t;          // after the scatter levels: one (row, moment) total per lane
    if constexpr (ROWS == 4) {
        // xor 1: rows {b0, b0 + 2} of both moments stay
        double ka[2], kb[2];
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            ka[j] = (b0 ? a[2 * j + 1] : a[2 * j]) + from_lane_xor<1>(b0 ? a[2 * j] : a[2 * j + 1]);
            kb[j] = (b0 ? b[2 * j + 1] : b[2 * j]) + from_lane_xor<1>(b0 ? b[2 * j] : b[2 * j + 1]);
        }
        // xor 2: row 2 * b1 + b0 stays
        const double ma = (b1 ? ka[1] : ka[0]) + from_lane_xor<2>(b1 ? ka[0] : ka[1]);
        const double mb = (b1 ? kb[1] : kb[0]) + from_lane_xor<2>(b1 ? kb[0] : kb[1]);
        // xor 4: moment b2 stays
        t = (b2 ? mb : ma) + from_lane_xor<4>(b2 ? ma : mb);
        t = t + from_lane_xor<8>(t);
        t = t + from_lane_xor<16>(t);
        t = add_across_halves(t);
        // rows: (0 + 1), (2 + 3), then their sum; the row index sits in lane bits 0 and 1
        t = t + from_lane_xor<1>(t);
        t = t + from_lane_xor<2>(t);
        // lanes with bit 2 clear hold the sum of x, the others the sum of x*x
        const double other = from_lane_xor<4>(t);
        s1 = b2 ? other : t;
        s2 = b2 ? t : other;
    } else {
        // xor 1: row b0 of both moments stays
        const double ma = (b0 ? a[1] : a[0]) + from_lane_xor<1>(b0 ? a[0] : a[1]);
        const double mb = (b0 ? b[1] : b[0]) + from_lane_xor<1>(b0 ? b[0] : b[1]);
        // xor 2: moment b1 stays
        t = (b1 ? mb : ma) + from_lane_xor<2>(b1 ? ma : mb);
        t = t + from_lane_xor<4>(t);
        t = t + from_lane_xor<8>(t);
        t = t + from_lane_xor<16>(t);
        t = add_across_halves(t);
        t = t + from_lane_xor<1>(t);                          // row 0 + row 1
        const double other = from_lane_xor<2>(t);
        s1 = b1 ? other : t;
        s2 = b1 ? t : other;
    }
}

// ---- per-kernel descriptors (fh_batch.hpp: up to kBatch tensors per launch) ----------------
struct MomentsItem { const void* x; int64_t numel; f64x2* partial; };
struct ReduceItem  { const f64x2* in; int64_t count; f64x2* out; };
struct FinishItem  {
    const f64x2* in; int64_t count; int64_t numel; double k_sigma;
    double* stats; uint32_t* counts; uint8_t* mask; int32_t channels;
};
struct MaskItem    { const uint32_t* counts; uint8_t* mask; int64_t min_outliers; int32_t channels; };

// ---- pass 1a: spans of the tensor ------------------------------------------------------
template <typename InT> struct Span;
template <> struct Span<float> {            // 4 rows of 256, 4 consecutive elements per lane
    static constexpr int ROWS = 4, EPL = 4;
    __device__ static __forceinline__ void load(const float* p, float (&x)[EPL]) {
        const f32x4 v = stream_load(reinterpret_cast<const f32x4*>(p));
        x[0] = v.x; x[1] = v.y; x[2] = v.z; x[3] = v.w;
    }
    __device__ static __forceinline__ void widen(const u32x4& w, float (&x)[EPL]) {
        const f32x4 v = __builtin_bit_cast(f32x4, w);
        x[0] = v.x; x[1] = v.y; x[2] = v.z; x[3] = v.w;
    }
    __device__ static __forceinline__ float one(const float* p) { return *p; }
};
template <> struct Span<uint16_t> {         // 2 rows of 512, 8 consecutive elements per lane
    static constexpr int ROWS = 2, EPL = 8;
    __device__ static __forceinline__ void load(const uint16_t* p, float (&x)[EPL]) {
        const u32x4 v = stream_load(reinterpret_cast<const u32x4*>(p));
        x[0] = bf16_lo(v.x); x[1] = bf16_hi(v.x); x[2] = bf16_lo(v.y); x[3] = bf16_hi(v.y);
        x[4] = bf16_lo(v.z); x[5] = bf16_hi(v.z); x[6] = bf16_lo(v.w); x[7] = bf16_hi(v.w);
    }
    __device__ static __forceinline__ void widen(const u32x4& v, float (&x)[EPL]) {
        x[0] = bf16_lo(v.x); x[1] = bf16_hi(v.x); x[2] = bf16_lo(v.y); x[3] = bf16_hi(v.y);
        x[4] = bf16_lo(v.z); x[5] = bf16_hi(v.z); x[6] = bf16_lo(v.w); x[7] = bf16_hi(v.w);
    }
    __device__ static __forceinline__ float one(const uint16_t* p) {
        return __builtin_bit_cast(float, (uint32_t)*p << 16);
    }
};

// balanced tree over N consecutive values (N a power of two)
template <int N>
__device__ __forceinline__ double local_tree(const double (&v)[N])
{
    double w[N];
#pragma unroll
    for (int i = 0; i < N; ++i) w[i] = v[i];
#pragma unroll
    for (int n = N; n > 1; n /= 2)
#pragma unroll
        for (int i = 0; i < n / 2; ++i) w[i] = w[2 * i] + w[2 * i + 1];
    return w[0];
}

template <typename InT>
__global__ __launch_bounds__(kThreads) void moments_kernel(const Batch<MomentsItem> args)
{
    constexpr int ROWS = Span<InT>::ROWS, EPL = Span<InT>::EPL, ROW = kWave * EPL;
    uint32_t block;
    const MomentsItem& it = args.item[batch_item(args, blockIdx.x, block)];
    const InT* x = static_cast<const InT*>(it.x);
    const int64_t numel = it.numel;
    f64x2* partial = it.partial;
    const uint32_t lane = threadIdx.x & (kWave - 1);
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t span = (int64_t)block * kWavesPerBlock + wave;
    const int64_t base = span * kSpan;
    if (base >= numel) return;                                // wave-uniform
    const InT* xs = x + base;
    double a[ROWS], b[ROWS];
    const bool interior = base + kSpan <= numel;
#pragma unroll
    for (int r = 0; r < ROWS; ++r) {
        float v[EPL];
        const uint32_t e0 = r * ROW + lane * EPL;
        if (interior) {
            Span<InT>::load(xs + e0, v);
        } else {
#pragma unroll
            for (int j = 0; j < EPL; ++j) v[j] = (base + e0 + j < numel) ? Span<InT>::one(xs + e0 + j) : 0.0f;
        }
        double d[EPL], q[EPL];
#pragma unroll
        for (int j = 0; j < EPL; ++j) { d[j] = (double)v[j]; q[j] = d[j] * d[j]; }   // the square is exact
        a[r] = local_tree<EPL>(d);
        b[r] = local_tree<EPL>(q);
    }
    double s1, s2;
    span_tree<ROWS>(a, b, lane, s1, s2);
    if (lane == 0) partial[span] = f64x2{s1, s2};
}

// ---- pass 1b: spans of partial sums (4 rows of 256 pairs, 4 consecutive pairs per lane) --
__global__ __launch_bounds__(kThreads) void reduce_partials_kernel(const Batch<ReduceItem> args)
{
    constexpr int ROWS = 4, EPL = 4, ROW = kWave * EPL;
    uint32_t block;
    const ReduceItem& it = args.item[batch_item(args, blockIdx.x, block)];
    const f64x2* in = it.in;
    const int64_t count = it.count;
    f64x2* out = it.out;
    const uint32_t lane = threadIdx.x & (kWave - 1);
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t span = (int64_t)block * kWavesPerBlock + wave;
    const int64_t base = span * kSpan;
    if (base >= count) return;
    double a[ROWS], b[ROWS];
#pragma unroll
    for (int r = 0; r < ROWS; ++r) {
        double d[EPL], q[EPL];
#pragma unroll
        for (int j = 0; j < EPL; ++j) {
            const int64_t i = base + r * ROW + lane * EPL + j;
            const f64x2 p = i < count ? in[i] : f64x2{0.0, 0.0};
            d[j] = p.x; q[j] = p.y;
        }
        a[r] = local_tree<EPL>(d);
        b[r] = local_tree<EPL>(q);
    }
    double s1, s2;
    span_tree<ROWS>(a, b, lane, s1, s2);
    if (lane == 0) out[span] = f64x2{s1, s2};
}

// ---- pass 1c: last level of the tree (at most 1024 partial sums), then mean, variance and
//      threshold; clears the counters and the mask ----------------------------------------------
struct FinishBatch { FinishItem item[kBatch]; };           // one workgroup per tensor
__global__ __launch_bounds__(kThreads) void finish_moments_kernel(const FinishBatch args)
{
    const FinishItem& it = args.item[blockIdx.x];
    const f64x2* in = it.in;
    const int64_t count = it.count, numel = it.numel;
    const double k_sigma = it.k_sigma;
    double* stats = it.stats;
    uint32_t* counts = it.counts;
    uint8_t* mask = it.mask;
    const int channels = it.channels;
    for (int c = threadIdx.x; c < channels; c += kThreads) { counts[c] = 0u; mask[c] = 0; }
    if (threadIdx.x >= kWave) return;                         // the tree is one wave's work
    constexpr int ROWS = 4, EPL = 4, ROW = kWave * EPL;
    const uint32_t lane = threadIdx.x;
    double a[ROWS], b[ROWS];
#pragma unroll
    for (int r = 0; r < ROWS; ++r) {
        double d[EPL], q[EPL];
#pragma unroll
        for (int j = 0; j < EPL; ++j) {
            const int64_t i = r * ROW + lane * EPL + j;
            const f64x2 p = i < count ? in[i] : f64x2{0.0, 0.0};
            d[j] = p.x; q[j] = p.y;
        }
        a[r] = local_tree<EPL>(d);
        b[r] = local_tree<EPL>(q);
    }
    double s1, s2;
    span_tree<ROWS>(a, b, lane, s1, s2);
    if (lane == 0) {
        double mean = 0.0, variance = 0.0;
        if (numel > 0) {
            const double n = (double)numel;
            mean = (s1 + 0.0) / n;                            // a total of -0.0 counts as +0.0; IEEE division
            const double mean_sq = mean * mean;
            variance = s2 / n - mean_sq;
            if (!(variance > 0.0)) variance = 0.0;
        }
        stats[0] = mean;
        stats[1] = variance;
        stats[2] = (k_sigma * k_sigma) * variance;
        stats[3] = (double)numel;
    }
}

// ---- pass 2: outliers per channel ----------------------------------------------------------
// Channel of an outlier: division by `inner` and `channels` through the small-dividend
// divider of fh_channels.hpp (dividends stay below divisor + 2 * 1024 here).
struct CountArgs {
    const void* x;
    int64_t numel;
    const double* stats;
    uint32_t* counts;
    SmallDiv inner, channels;
    int32_t spans_per_wave;                                   // consecutive spans one wave walks
};

// AHEAD: a launch in which some wave walks more than one span.
constexpr int kAhead = 3;                         // spans requested before the one that is looked at
template <typename InT, bool AHEAD>
__global__ __launch_bounds__(kThreads) void count_outliers_kernel(const Batch<CountArgs> batch)
{
    constexpr int ROWS = Span<InT>::ROWS, EPL = Span<InT>::EPL, ROW = kWave * EPL;
    extern __shared__ uint32_t hist[];
    uint32_t block;
    const CountArgs& args = batch.item[batch_item(batch, blockIdx.x, block)];
    const uint32_t C = args.channels.d;
    for (uint32_t c = threadIdx.x; c < C; c += kThreads) hist[c] = 0u;
    __syncthreads();

    const uint32_t lane = threadIdx.x & (kWave - 1);
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const double mean = args.stats[0], threshold = args.stats[2];
    const InT* x = static_cast<const InT*>(args.x);
    const int64_t numel = args.numel;
    // this wave's spans: first_span, first_span + 1, ...
    const int64_t first_span = ((int64_t)block * kWavesPerBlock + wave) * args.spans_per_wave;
    int64_t base = first_span * kSpan;
    // position of the span's first element: rem = index inside the channel run, chan = channel
    uint32_t rem = 0, chan = 0;
    if (base < numel) {
        const uint64_t run = (uint64_t)base / args.inner.d;   // once per wave
        rem = (uint32_t)((uint64_t)base - run * args.inner.d);
        chan = (uint32_t)(run % C);
    }
    // The rows of the spans ahead are requested before this one's are looked at: a wave walks its spans one after
    // the other, and with one span in flight per wave the device does not hold enough bytes in flight to cover the
    // memory latency (measured on bf16 [tokens][hidden] tensors with 6 to 16 spans per wave: 32 -> 28 us per 80 MB
    // with one span ahead; a single such tensor is 1.5 waves per SIMD, and with three spans ahead its pass takes
    // as long as the first pass over it).  The ring of kAhead + 1 spans has constant indices: the walk is
    // unrolled by that many.
    constexpr int RING = AHEAD ? kAhead + 1 : 1;
    u32x4 ring[RING][ROWS];
    const auto request = [&](int64_t at, u32x4 (&w)[ROWS]) {  // whole spans only: the last one of a tensor is read element by element
        if (at + kSpan <= numel) {
#pragma unroll
            for (int r = 0; r < ROWS; ++r) w[r] = stream_load(reinterpret_cast<const u32x4*>(x + at + r * ROW + lane * EPL));
        }
    };
    const int spans = args.spans_per_wave;
    if (AHEAD) {
#pragma unroll
        for (int k = 0; k < kAhead; ++k)
            if (k < spans && base + (int64_t)k * kSpan < numel) request(base + (int64_t)k * kSpan, ring[k]);
    }
    // one span: the outliers of its rows into the histogram, then (rem, chan) and base move on by a span
    const auto look = [&](const u32x4 (&now)[ROWS], bool interior) {
        const InT* xs = x + base;
        uint32_t bits = 0u;                                   // bit r * EPL + j: that element is an outlier
#pragma unroll
        for (int r = 0; r < ROWS; ++r) {
            float v[EPL];
            const uint32_t e0 = r * ROW + lane * EPL;
            if (interior) {
                Span<InT>::widen(now[r], v);
            } else {
#pragma unroll
                for (int j = 0; j < EPL; ++j)
                    v[j] = (base + e0 + j < numel) ? Span<InT>::one(xs + e0 + j) : __builtin_bit_cast(float, 0x7fc00000u);
            }
#pragma unroll
            for (int j = 0; j < EPL; ++j) {
                const double d = (double)v[j] - mean;
                if (d * d > threshold) bits |= 1u << (r * EPL + j);          // false for the NaN filler
            }
        }
        while (bits) {                                        // rare: about k-sigma tail mass * 16 per lane
            const uint32_t k2 = (uint32_t)__builtin_ctz(bits);
            bits &= bits - 1u;
            const uint32_t off = (k2 / EPL) * ROW + lane * EPL + (k2 % EPL);   // element offset inside the span
            const uint32_t runs = div_small(rem + off, args.inner);           // channel runs crossed from `chan`
            const uint32_t cc = chan + runs;
            const uint32_t c = cc - div_small(cc, args.channels) * C;
            atomicAdd(&hist[c], 1u);
        }
        const uint32_t t = rem + kSpan;
        const uint32_t runs = div_small(t, args.inner);
        rem = t - runs * args.inner.d;
        const uint32_t cc = chan + runs;
        chan = cc - div_small(cc, args.channels) * C;
        base += kSpan;
    };
    for (int s0 = 0; s0 < spans && base < numel; s0 += RING) {
        // A round whose spans, and the spans requested during it, are all whole and all this wave's runs without
        // a test around any load: only then can the waits be for the oldest request alone and not for all of them.
        if (AHEAD && s0 + RING + kAhead <= spans && base + (int64_t)(RING + kAhead) * kSpan <= numel) {
#pragma unroll
            for (int k = 0; k < RING; ++k) {
                u32x4 (&ahead)[ROWS] = ring[(k + kAhead) % RING];
#pragma unroll
                for (int r = 0; r < ROWS; ++r)
                    ahead[r] = stream_load(reinterpret_cast<const u32x4*>(x + base + (int64_t)kAhead * kSpan + r * ROW + lane * EPL));
                look(ring[k], true);
            }
            continue;
        }
#pragma unroll
        for (int k = 0; k < RING; ++k) {
            const int s = s0 + k;
            if (s >= spans || base >= numel) break;
            if (AHEAD && s + kAhead < spans && base + (int64_t)kAhead * kSpan < numel)
                request(base + (int64_t)kAhead * kSpan, ring[(k + kAhead) % RING]);
            if (!AHEAD) request(base, ring[k]);
            look(ring[k], base + kSpan <= numel);
        }
    }
    __syncthreads();
    for (uint32_t c = threadIdx.x; c < C; c += kThreads) {
        const uint32_t v = hist[c];
        if (v) atomicAdd(&args.counts[c], v);
    }
}

__global__ __launch_bounds__(kThreads) void mask_kernel(const Batch<MaskItem> args)
{
    uint32_t block;
    const MaskItem& it = args.item[batch_item(args, blockIdx.x, block)];
    const int c = block * kThreads + threadIdx.x;
    if (c < it.channels) it.mask[c] = (int64_t)it.counts[c] >= it.min_outliers ? 1 : 0;
}

int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

}  // namespace
}  // namespace fh

extern "C" {

size_t fh_classify_workspace_bytes(int64_t numel)
{
    // one {sum x, sum x*x} pair per 1024-element span, then per 1024 of those, ... down to one
    if (numel <= 0) return 16;
    size_t pairs = 0;
    int64_t m = fh::ceil_div(numel, fh::kSpan);
    for (;;) {
        pairs += (size_t)m;
        if (m == 1) break;
        m = fh::ceil_div(m, fh::kSpan);
    }
    return pairs * 16;
}

}  // extern "C"

// ---- partial sums in a buffer of the library's own -------------------------------------------
// For callers that cannot allocate (HIP graph capture, serving loops, harnesses that forbid it):
// the workspace of the partial-sum tree as a device array that is part of the code object.  Each
// GPU the library runs on holds its own copy at its own address until the process ends; every
// call on a GPU shares it, so calls that overlap on one GPU race.  Nothing in it has to start
// at zero: every level of the tree is written in full before it is read.
constexpr size_t kScratchBytes = (size_t)4 << 20;           // serves up to 2^28 - 2^18 elements
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

namespace {

using namespace fh;

// The device address of `scratch` on the current device.  In host code the array's name is only
// a handle for hipGetSymbolAddress, never an address a kernel may be given; the address is
// asked for once per device, with that device current, and kept.
constexpr int kMaxDevices = 64;
std::mutex g_scratch_lock;
void* g_scratch_ptr[kMaxDevices] = {};

fh_status scratch_of_current_device(void** out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return FH_ERR_LAUNCH;
    std::lock_guard<std::mutex> hold(g_scratch_lock);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return FH_ERR_LAUNCH;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return FH_OK;
}

fh_status check_item(const fh_classify_item& it, int64_t* numel_out)
{
    if (it.x_dtype != FH_F32 && it.x_dtype != FH_BF16) return FH_ERR_BAD_DTYPE;
    if (it.reserved != 0) return FH_ERR_BAD_PARAM;
    if (it.outer < 0 || it.inner < 1 || it.channels < 1 || it.channels > kMaxChannels) return FH_ERR_BAD_SHAPE;
    if (it.inner > (int64_t)1 << 31 || it.outer > (int64_t)1 << 40) return FH_ERR_BAD_SHAPE;
    if (!(it.k_sigma > 0.0) || it.min_outliers < 1) return FH_ERR_BAD_PARAM;
    const double total = (double)it.outer * (double)it.channels * (double)it.inner;
    if (total > (double)((int64_t)1 << 40)) return FH_ERR_BAD_NUMEL;
    const int64_t numel = it.outer * it.channels * it.inner;
    if (!it.workspace || !it.stats || !it.counts || !it.mask || (numel > 0 && !it.x)) return FH_ERR_NULL;
    auto misaligned = [](const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) != 0; };
    if (misaligned(it.x, 16) || misaligned(it.workspace, 16) || misaligned(it.stats, 8) || misaligned(it.counts, 4))
        return FH_ERR_ALIGNMENT;
    if (it.workspace_cap < fh_classify_workspace_bytes(numel)) return FH_ERR_BUFFER_TOO_SMALL;
    *numel_out = numel;
    return FH_OK;
}

// One run of up to kBatch tensors of one dtype: five kinds of launches, each covering all of them.
fh_status run_classify(const fh_classify_item* items, const int64_t* numels, int n, hipStream_t s)
{
    const dim3 block(kThreads);
    const int dtype = items[0].x_dtype;
    f64x2* level[kBatch];
    int64_t m[kBatch];

    Batch<MomentsItem> mb;
    reset(mb);
    for (int i = 0; i < n; ++i) {
        level[i] = static_cast<f64x2*>(items[i].workspace);
        m[i] = numels[i] > 0 ? ceil_div(numels[i], kSpan) : 0;
        if (numels[i] > 0 && !push(mb, MomentsItem{items[i].x, numels[i], level[i]}, ceil_div(m[i], kWavesPerBlock)))
            return FH_ERR_BAD_NUMEL;
    }
    if (mb.count > 0) {
        seal(mb);
        const dim3 grid(mb.block_start[mb.count]);
        if (dtype == FH_F32) hipLaunchKernelGGL(moments_kernel<float>, grid, block, 0, s, mb);
        else hipLaunchKernelGGL(moments_kernel<uint16_t>, grid, block, 0, s, mb);
    }
    for (;;) {                                                // tree levels above the first, where needed
        Batch<ReduceItem> rb;
        reset(rb);
        for (int i = 0; i < n; ++i) {
            if (m[i] <= kSpan) continue;                      // the last <= 1024 partials are the finish kernel's
            const int64_t next = ceil_div(m[i], kSpan);
            f64x2* out = level[i] + m[i];
            push(rb, ReduceItem{level[i], m[i], out}, ceil_div(next, kWavesPerBlock));
            level[i] = out;
            m[i] = next;
        }
        if (rb.count == 0) break;
        seal(rb);
        hipLaunchKernelGGL(reduce_partials_kernel, dim3(rb.block_start[rb.count]), block, 0, s, rb);
    }
    FinishBatch fb;
    for (int i = 0; i < n; ++i)
        fb.item[i] = FinishItem{level[i], m[i], numels[i], items[i].k_sigma, static_cast<double*>(items[i].stats),
                                static_cast<uint32_t*>(items[i].counts), static_cast<uint8_t*>(items[i].mask),
                                (int32_t)items[i].channels};
    for (int i = n; i < kBatch; ++i) fb.item[i] = fb.item[0];
    hipLaunchKernelGGL(finish_moments_kernel, dim3(n), block, 0, s, fb);

    Batch<CountArgs> cb;
    Batch<MaskItem> kb;
    reset(cb);
    reset(kb);
    size_t lds = 0;
    for (int i = 0; i < n; ++i) {
        if (numels[i] == 0) continue;                         // no outliers: the cleared mask stands
        CountArgs a;
        a.x = items[i].x;
        a.numel = numels[i];
        a.stats = static_cast<const double*>(items[i].stats);
        a.counts = static_cast<uint32_t*>(items[i].counts);
        a.inner = make_small_div((uint32_t)items[i].inner);
        a.channels = make_small_div((uint32_t)items[i].channels);
        // a workgroup clears `channels` histogram bins and adds the non-zero ones to the tensor's counters with
        // atomics that meet those of every other workgroup on a few cache lines: give it enough elements to make
        // that cheap, but no more (short workgroups measured faster on feature maps; 128 elements per bin and
        // wave on [tokens][hidden] tensors, where the outliers of ordinary activations touch most bins)
        const int64_t ch = items[i].channels;
        a.spans_per_wave = (int32_t)(ch <= 512 ? 1 : ch / 128 < 16 ? ch / 128 : 16);
        const int64_t per_block = (int64_t)a.spans_per_wave * kWavesPerBlock * kSpan;
        if (!push(cb, a, ceil_div(numels[i], per_block))) return FH_ERR_BAD_NUMEL;
        push(kb, MaskItem{a.counts, static_cast<uint8_t*>(items[i].mask), items[i].min_outliers, (int32_t)ch},
             ceil_div(ch, kThreads));
        if ((size_t)ch * sizeof(uint32_t) > lds) lds = (size_t)ch * sizeof(uint32_t);
    }
    if (cb.count > 0) {
        seal(cb);
        seal(kb);
        const dim3 grid(cb.block_start[cb.count]);
        bool ahead = false;
        for (int k = 0; k < cb.count; ++k) ahead = ahead || cb.item[k].spans_per_wave > 1;
        if (dtype == FH_F32) {
            if (ahead) hipLaunchKernelGGL((count_outliers_kernel<float, true>), grid, block, lds, s, cb);
            else hipLaunchKernelGGL((count_outliers_kernel<float, false>), grid, block, lds, s, cb);
        } else {
            if (ahead) hipLaunchKernelGGL((count_outliers_kernel<uint16_t, true>), grid, block, lds, s, cb);
            else hipLaunchKernelGGL((count_outliers_kernel<uint16_t, false>), grid, block, lds, s, cb);
        }
        hipLaunchKernelGGL(mask_kernel, dim3(kb.block_start[kb.count]), block, 0, s, kb);
    }
    return hipGetLastError() == hipSuccess ? FH_OK : FH_ERR_LAUNCH;
}

}  // namespace

extern "C" {

int32_t fh_classify_batch_capacity(void) { return fh::kBatch; }

fh_status fh_classify_channels_batch(const fh_classify_item* items, int32_t count, void* stream)
{
    if (count < 0) return FH_ERR_BAD_COUNT;
    if (count > 0 && !items) return FH_ERR_NULL;
    // all items are checked before the first launch
    for (int32_t i = 0; i < count; ++i) {
        int64_t numel;
        const fh_status st = check_item(items[i], &numel);
        if (st != FH_OK) return st;
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    int32_t i = 0;
    while (i < count) {                                       // runs of one dtype, at most kBatch long
        int64_t numels[fh::kBatch];
        int n = 0;
        while (i + n < count && n < fh::kBatch && items[i + n].x_dtype == items[i].x_dtype) {
            check_item(items[i + n], &numels[n]);
            ++n;
        }
        const fh_status st = run_classify(items + i, numels, n, s);
        if (st != FH_OK) return st;
        i += n;
    }
    return FH_OK;
}

fh_status fh_classify_channels(const void* x, fh_dtype x_dtype, int64_t outer, int64_t channels, int64_t inner,
                               double k_sigma, int64_t min_outliers,
                               void* workspace, size_t workspace_cap,
                               void* stats, void* counts, void* mask, void* stream)
{
    fh_classify_item it;
    it.x = x; it.x_dtype = x_dtype; it.reserved = 0;
    it.outer = outer; it.channels = channels; it.inner = inner;
    it.k_sigma = k_sigma; it.min_outliers = min_outliers;
    it.workspace = workspace; it.workspace_cap = workspace_cap;
    it.stats = stats; it.counts = counts; it.mask = mask;
    return fh_classify_channels_batch(&it, 1, stream);
}

size_t fh_classify_static_scratch_bytes(void) { return kScratchBytes; }

fh_status fh_classify_channels_static(const void* x, fh_dtype x_dtype, int64_t outer, int64_t channels, int64_t inner,
                                      double k_sigma, int64_t min_outliers,
                                      void* stats, void* counts, void* mask, void* stream)
{
    // the size check comes first: a tensor the static buffer cannot serve is refused before
    // anything else is looked at, and before the buffer's address is asked for
    if (outer >= 0 && channels >= 1 && inner >= 1) {
        const double total = (double)outer * (double)channels * (double)inner;
        if (total > (double)((int64_t)1 << 40)) return FH_ERR_BAD_NUMEL;
        if (fh_classify_workspace_bytes(outer * channels * inner) > kScratchBytes) return FH_ERR_SCRATCH_LIMIT;
    }
    void* ws = nullptr;
    const fh_status st = scratch_of_current_device(&ws);
    if (st != FH_OK) return st;
    return fh_classify_channels(x, x_dtype, outer, channels, inner, k_sigma, min_outliers, ws, kScratchBytes,
                                stats, counts, mask, stream);
}

}  // extern "C"
