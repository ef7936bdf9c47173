// Forward side of the group quantiser on gfx950: one pass over the activation.
//
// A wave owns a span of consecutive elements (1024 fp32 or 2048 bf16 = 4 KiB of input),
// viewed as 4 rows; a lane owns one 128-bit load of every row (4 fp32 or 8 bf16
// consecutive elements), so each load instruction of a wave reads 1 KiB contiguously.
// The statistics of the four rows are reduce-scattered over the lanes of each quad, so
// every lane finishes ONE row's min/max, does one division, and the quantiser reads
// `mn` / `inv` of row r straight from the quad lane that holds them (DPP operand
// broadcast).  Codes and meta leave through a per-wave LDS staging area as contiguous
// stores.  The last, partial tile of a tensor takes a plain guarded path with 8
// elements per lane; both paths produce the same bytes because nothing in the
// definition depends on which lane does what.
//
// Follows the paper's Section 4.4.1 (normal channels: linear-scale quantisation;
// zeros must be preserved) with the parameters the paper leaves open taken from the
// caller (group size, bits, rounding, seed).
//
// The MIXED variants additionally route the channels the caller marks as kept (salient
// channels, same section) around the quantiser: their elements are copied to a raw store,
// turned into NaN -- which v_min_f32 / v_max_f32 ignore -- before the statistics, and get
// code 0.
#include <type_traits>

#include "fh_channels.hpp"
#include "fh_device.hpp"
#include "fh_kernels.hpp"

namespace fh {

namespace {

constexpr int kCBlock = 256;                       // threads per workgroup
constexpr int kWaves = kCBlock / kWave;
constexpr int kEPL = 8;                            // elements per lane in the guarded (edge) layout
constexpr int kRow = kWave * kEPL;                 // ... whose rows are 512 elements

template <typename InT> struct Layout {
    static constexpr int EPL = 16 / (int)sizeof(InT);          // elements per lane and row: one 128-bit load
    static constexpr int ROW = kWave * EPL;                    // 256 fp32 or 512 bf16
    static constexpr int SPAN = 4 * ROW;                       // elements per wave
    static constexpr int TILE = kWaves * SPAN;                 // elements per workgroup
    static constexpr int EDGE_ROWS = SPAN / kRow;              // rows of the guarded layout per span
};

// Per-wave LDS staging area: the codes of the wave's span in element order (at most one
// byte per element) followed by its groups' {scale, zero} pairs (at most span / 64).
// Each wave only touches its own area, so no workgroup barrier is involved.  It is
// written and read back through different widths, hence the may_alias types.
typedef uint8_t __attribute__((may_alias)) stage_u8;
typedef uint16_t __attribute__((may_alias)) stage_u16;
typedef uint32_t __attribute__((may_alias)) stage_u32;
typedef u32x2 __attribute__((may_alias)) stage_u32x2;
typedef u32x4 __attribute__((may_alias)) stage_u32x4;
typedef f32x2 __attribute__((may_alias)) stage_f32x2;
constexpr int kStageCodeBytes = 2048;              // the larger (bf16) span at 8 bits
constexpr int kStageMetaBytes = (2048 / 64) * 8;
constexpr int kStageDwords = (kStageCodeBytes + kStageMetaBytes) / 4;

template <int G> struct Log2;
template <> struct Log2<64>  { static constexpr int v = 6; };
template <> struct Log2<128> { static constexpr int v = 7; };
template <> struct Log2<256> { static constexpr int v = 8; };

// ---- quantise + pack ---------------------------------------------------------------
// Each element first becomes a 32-bit word with its code in one known byte and zeros
// in the code's unused upper bits; v_perm_b32 then gathers those bytes.
//
// nearest:    r = q + 2^23 rounds q to an integer with ties to even (the sum lies in
//             [2^23, 2^24), where the float spacing is 1), and leaves it in the low
//             mantissa bits: byte 0 of r is rint(q).
// stochastic: with Q = q * 2^16 (exact) and C = ceil(Q),
//                 floor(q) + [h / 2^16 < q - floor(q)]  ==  (C + 65535 - h) >> 16
//             because h < frac(q) * 2^16  <=>  h < ceil(frac(q) * 2^16)  <=>  the low
//             16 bits of C plus (65535 - h) carry.  The sum is below 2^24, so byte 2
//             is the code.  -C comes from v_cvt_flr_i32_f32(-Q); 65535 - h is a
//             half-word of the complemented random word, picked by SDWA in the subtract.
template <bool STOCH> struct CodeByte { static constexpr uint32_t pos = STOCH ? 2u : 0u; };

template <int HALF>
__device__ __forceinline__ uint32_t halfword_minus(uint32_t not_word, int neg_c)
{
    uint32_t d;
    if constexpr (HALF == 0)
        asm volatile("v_sub_u32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:WORD_0 src1_sel:DWORD"
                     : "=v"(d) : "v"(not_word), "v"(neg_c));
    else
        asm volatile("v_sub_u32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:WORD_1 src1_sel:DWORD"
                     : "=v"(d) : "v"(not_word), "v"(neg_c));
    return d;
}

// The element word of one value: q is (x - mn) * inv, not yet clamped; `not_word` is the
// complemented Philox word whose half HALF belongs to this element.
template <int B, bool STOCH, int HALF>
__device__ __forceinline__ uint32_t element_word(float q, uint32_t not_word)
{
    constexpr float Lf = (float)((1 << B) - 1);
    const float c = __builtin_amdgcn_fmed3f(q, 0.0f, Lf);     // clamp to [0, L]
    if constexpr (STOCH) {
        const float Q = c * 65536.0f;                         // exact
        int neg_c;
        asm volatile("v_cvt_flr_i32_f32_e64 %0, -%1" : "=v"(neg_c) : "v"(Q));   // -ceil(Q)
        return halfword_minus<HALF>(not_word, neg_c);
    } else {
        return __builtin_bit_cast(uint32_t, c + 0x1p23f);
    }
}

// [code(a), code(b), 0, 0] from the code bytes of two element words.
template <uint32_t POS>
__device__ __forceinline__ uint32_t pair_bytes(uint32_t a, uint32_t b)
{
    return __builtin_amdgcn_perm(b, a, 0x0c0c0000u | ((4u + POS) << 8) | POS);
}
// [code(a), code(b), code(c), code(d)]
template <uint32_t POS>
__device__ __forceinline__ uint32_t quad_bytes(uint32_t a, uint32_t b, uint32_t c, uint32_t d)
{
    return __builtin_amdgcn_perm(pair_bytes<POS>(c, d), pair_bytes<POS>(a, b), 0x05040100u);
}

// 8 consecutive codes -> 8, 4 or 2 packed bytes (w1 is used at 8 bits only)
template <int B, uint32_t POS>
__device__ __forceinline__ void pack8(const uint32_t (&e)[8], uint32_t& w0, uint32_t& w1)
{
    if constexpr (B == 8) {
        w0 = quad_bytes<POS>(e[0], e[1], e[2], e[3]);
        w1 = quad_bytes<POS>(e[4], e[5], e[6], e[7]);
    } else if constexpr (B == 4) {                            // byte k = code(2k) | code(2k+1) << 4
        const uint32_t even = quad_bytes<POS>(e[0], e[2], e[4], e[6]);
        const uint32_t odd = quad_bytes<POS>(e[1], e[3], e[5], e[7]);
        w0 = (odd << 4) | even;
        w1 = 0u;
    } else {                                                  // byte k = codes 4k .. 4k+3, two bits each
        const uint32_t c0 = pair_bytes<POS>(e[0], e[4]), c1 = pair_bytes<POS>(e[1], e[5]);
        const uint32_t c2 = pair_bytes<POS>(e[2], e[6]), c3 = pair_bytes<POS>(e[3], e[7]);
        w0 = (c3 << 6) | ((c2 << 4) | ((c1 << 2) | c0));
        w1 = 0u;
    }
}
// 4 consecutive codes -> 4, 2 or 1 packed bytes
template <int B, uint32_t POS>
__device__ __forceinline__ uint32_t pack4(const uint32_t (&e)[4])
{
    if constexpr (B == 8) {
        return quad_bytes<POS>(e[0], e[1], e[2], e[3]);
    } else if constexpr (B == 4) {
        return (pair_bytes<POS>(e[1], e[3]) << 4) | pair_bytes<POS>(e[0], e[2]);
    } else {
        // four 2-bit codes, one per byte, times (2^24 + 2^18 + 2^12 + 2^6): the shifted copies
        // fall into disjoint bit fields and the top byte collects c0 | c1<<2 | c2<<4 | c3<<6
        return (quad_bytes<POS>(e[0], e[1], e[2], e[3]) * 0x01041040u) >> 24;
    }
}

// ---- cross-lane pieces of the 4-row layout -------------------------------------------
// DPP reads of a register sit two wait states after the VALU write of it (a hazard the
// compiler cannot see inside an asm block); each block opens and closes with s_nop 1.
#define FH_DPP_TAIL " row_mask:0xf bank_mask:0xf\n\t"

// min/max of `keep` with the partner lane's `send` (partner chosen by CTRL)
#define FH_DEFINE_EXCHANGE(NAME, CTRL)                                                            \
    __device__ __forceinline__ void NAME(float& kmin, float smin, float& kmax, float smax)        \
    {                                                                                             \
        asm volatile("s_nop 1\n\t"                                                                \
                     "v_min_f32_dpp %0, %2, %0 " CTRL FH_DPP_TAIL                                 \
                     "v_max_f32_dpp %1, %3, %1 " CTRL FH_DPP_TAIL "s_nop 1"                       \
                     : "+v"(kmin), "+v"(kmax) : "v"(smin), "v"(smax));                            \
    }
FH_DEFINE_EXCHANGE(exchange_xor1, "quad_perm:[1,0,3,2]")
FH_DEFINE_EXCHANGE(exchange_xor2, "quad_perm:[2,3,0,1]")
#undef FH_DEFINE_EXCHANGE

// All-reduce over the lanes of a run that share lane mod 4.
// RUN == 8: the partner is the lane 4 away inside each run of 8.  Lanes 0-3 and 8-11 of
//   a 16-lane row (DPP banks 0 and 2) read 4 lanes up, then banks 1 and 3 read 4 lanes
//   down; min/max are idempotent, so the second step may see the first one's result.
// RUN == 16: two rotations of the row.
template <int RUN>
__device__ __forceinline__ void allreduce_mod4(float& mn, float& mx)
{
    static_assert(RUN == 8 || RUN == 16, "inside one DPP row");
    if constexpr (RUN == 8) {
        asm volatile("s_nop 1\n\t"
                     "v_min_f32_dpp %0, %0, %0 row_shl:4 row_mask:0xf bank_mask:0x5\n\t"
                     "v_max_f32_dpp %1, %1, %1 row_shl:4 row_mask:0xf bank_mask:0x5\n\t"
                     "s_nop 0\n\t"
                     "v_min_f32_dpp %0, %0, %0 row_shr:4 row_mask:0xf bank_mask:0xa\n\t"
                     "v_max_f32_dpp %1, %1, %1 row_shr:4 row_mask:0xf bank_mask:0xa\n\t"
                     "s_nop 1"
                     : "+v"(mn), "+v"(mx));
    } else {
        asm volatile("s_nop 1\n\t"
                     "v_min_f32_dpp %0, %0, %0 row_ror:4" FH_DPP_TAIL
                     "v_max_f32_dpp %1, %1, %1 row_ror:4" FH_DPP_TAIL
                     "s_nop 0\n\t"
                     "v_min_f32_dpp %0, %0, %0 row_ror:8" FH_DPP_TAIL
                     "v_max_f32_dpp %1, %1, %1 row_ror:8" FH_DPP_TAIL "s_nop 1"
                     : "+v"(mn), "+v"(mx));
    }
}

// The value of a lane in a quad of the other parity of the same run, same lane mod 4.
template <int RUN>
__device__ __forceinline__ float from_other_quad(float v)
{
    if constexpr (RUN == 8) {
        float r;
        asm volatile("s_nop 1\n\t"
                     "v_mov_b32_dpp %0, %1 row_shl:4 row_mask:0xf bank_mask:0x5\n\t"
                     "v_mov_b32_dpp %0, %1 row_shr:4 row_mask:0xf bank_mask:0xa\n\t"
                     "s_nop 1"
                     : "=&v"(r) : "v"(v));
        return r;
    } else {
        return __builtin_bit_cast(float,
            __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), 0x124, 0xF, 0xF, true));   // row_ror:4
    }
}

// q[j] = (x[j] - mn_row) * inv_row with mn_row / inv_row read from quad lane HOLDER
template <int HOLDER>
__device__ __forceinline__ void scaled_offsets(float x0, float x1, float x2, float x3,
                                               float mn_held, float inv_held, float* q)
{
#define FH_Q4(SEL)                                                                                 \
    asm volatile("s_nop 1\n\t"                                                                     \
                 "v_subrev_f32_dpp %0, %8, %4 " SEL FH_DPP_TAIL                                    \
                 "v_subrev_f32_dpp %1, %8, %5 " SEL FH_DPP_TAIL                                    \
                 "v_subrev_f32_dpp %2, %8, %6 " SEL FH_DPP_TAIL                                    \
                 "v_subrev_f32_dpp %3, %8, %7 " SEL FH_DPP_TAIL                                    \
                 "v_mul_f32_dpp %0, %9, %0 " SEL FH_DPP_TAIL                                       \
                 "v_mul_f32_dpp %1, %9, %1 " SEL FH_DPP_TAIL                                       \
                 "v_mul_f32_dpp %2, %9, %2 " SEL FH_DPP_TAIL                                       \
                 "v_mul_f32_dpp %3, %9, %3 " SEL FH_DPP_TAIL                                       \
                 : "=&v"(q[0]), "=&v"(q[1]), "=&v"(q[2]), "=&v"(q[3])                              \
                 : "v"(x0), "v"(x1), "v"(x2), "v"(x3), "v"(mn_held), "v"(inv_held))
    if constexpr (HOLDER == 0) FH_Q4("quad_perm:[0,0,0,0]");
    else if constexpr (HOLDER == 1) FH_Q4("quad_perm:[1,1,1,1]");
    else if constexpr (HOLDER == 2) FH_Q4("quad_perm:[2,2,2,2]");
    else FH_Q4("quad_perm:[3,3,3,3]");
#undef FH_Q4
}
#undef FH_DPP_TAIL

__device__ __forceinline__ uint32_t from_pair_lane_u32(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0xB1, 0xF, 0xF, true);   // quad_perm [1,0,3,2]
}

template <typename InT> struct Loader;

template <> struct Loader<float> {
    __device__ static __forceinline__ void row(const float* p, float (&x)[4]) {
        const f32x4 v = stream_load(reinterpret_cast<const f32x4*>(p));
        x[0] = v.x; x[1] = v.y; x[2] = v.z; x[3] = v.w;
    }
    __device__ static __forceinline__ void widen(const u32x4& a, float (&x)[4]) {
        const f32x4 v = __builtin_bit_cast(f32x4, a);         // (a bit cast of one element of a vector reads element 0)
        x[0] = v.x; x[1] = v.y; x[2] = v.z; x[3] = v.w;
    }
    __device__ static __forceinline__ float one(const float* base, uint32_t i) { return base[i]; }
};

template <> struct Loader<uint16_t> {   // bf16 bit patterns; widening is exact
    __device__ static __forceinline__ void widen(const u32x4& a, float (&x)[8]) {
        x[0] = bf16_lo(a.x); x[1] = bf16_hi(a.x); x[2] = bf16_lo(a.y); x[3] = bf16_hi(a.y);
        x[4] = bf16_lo(a.z); x[5] = bf16_hi(a.z); x[6] = bf16_lo(a.w); x[7] = bf16_hi(a.w);
    }
    __device__ static __forceinline__ void row(const uint16_t* p, float (&x)[8]) {
        widen(stream_load(reinterpret_cast<const u32x4*>(p)), x);
    }
    __device__ static __forceinline__ float one(const uint16_t* base, uint32_t i) {
        return __builtin_bit_cast(float, (uint32_t)base[i] << 16);
    }
};

template <int N>
__device__ __forceinline__ void local_minmax(const float (&x)[N], float& mn, float& mx)
{
    mn = vmin3(x[0], x[1], x[2]);  mx = vmax3(x[0], x[1], x[2]);
    if constexpr (N == 4) {
        mn = vmin(mn, x[3]);  mx = vmax(mx, x[3]);
    } else {
        mn = vmin3(mn, x[3], x[4]);  mx = vmax3(mx, x[3], x[4]);
        mn = vmin3(mn, x[5], x[6]);  mx = vmax3(mx, x[5], x[6]);
        mn = vmin(mn, x[7]);         mx = vmax(mx, x[7]);
    }
}

// ---- kept channels (MIXED) ---------------------------------------------------------------
template <typename InT> struct RawElem;
template <> struct RawElem<float> {
    __device__ static __forceinline__ void put(void* raw, uint64_t i, float v) {
        static_cast<uint32_t*>(raw)[i] = __builtin_bit_cast(uint32_t, v);
    }
};
template <> struct RawElem<uint16_t> {
    __device__ static __forceinline__ void put(void* raw, uint64_t i, float v) {
        static_cast<uint16_t*>(raw)[i] = (uint16_t)(__builtin_bit_cast(uint32_t, v) >> 16);   // the original bits
    }
};

// Copy the kept elements of a lane's run to the raw store and hide them from the statistics:
// a kept element becomes a quiet NaN, which v_min_f32 / v_max_f32 pass over and which the
// quantiser's clamp (v_med3_f32: the minimum of the other two operands for a NaN) turns into code 0.
template <typename InT, int N>
__device__ __forceinline__ void divert_kept(const ChannelMap& cm, const KeptRun<N>& run, float (&x)[N])
{
#pragma unroll
    for (int j = 0; j < N; ++j) {
        if (run.mask & (1u << j)) {
            RawElem<InT>::put(cm.raw, raw_index<N>(cm, run, j), x[j]);
            x[j] = __builtin_bit_cast(float, 0x7fc00000u);
        }
    }
}

// One channel per element (fh_channels.hpp): the span's ROWS * 64 * 16 bytes are parked in the wave's
// staging area (free until the codes are staged), the lanes walk the span's (sample, row) pairs,
// copy each kept element from there to the raw store -- consecutive lanes, consecutive rows -- and
// leave a quiet NaN in its place; then every lane takes its elements back.  (The alternatives
// measured: every lane testing its own elements and storing the kept ones with one predicated
// 2- or 4-byte store each; the same with the kept elements compacted through LDS first.)
template <typename InT, int ROWS>
__device__ __forceinline__ void divert_listed(const ChannelMap& cm, const ElemPos& wave_pos, const uint16_t* rows,
                                              uint8_t* area, uint32_t lane, u32x4 (&w)[ROWS])
{
    typedef typename std::conditional<sizeof(InT) == 4, uint32_t, uint16_t>::type __attribute__((may_alias)) Elem;
    constexpr uint32_t SPAN = ROWS * kWave * 16 / sizeof(InT);
    constexpr Elem kQuietNaN = sizeof(InT) == 4 ? (Elem)0x7fc00000u : (Elem)0x7fc0u;
    // which pairs are this lane's, while the span's loads are still on their way
    const uint32_t pairs = span_pairs(cm, wave_pos, SPAN);
    PairWalk walk = pair_walk(cm, wave_pos, lane);
    uint32_t off[kPairsAhead];
    first_pairs(cm, walk, rows, pairs, off);
    stage_u32x4* in = reinterpret_cast<stage_u32x4*>(area);
#pragma unroll
    for (int r = 0; r < ROWS; ++r) in[r * kWave + lane] = w[r];
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");    // LDS operations of one wave complete in order
    Elem* elems = reinterpret_cast<Elem*>(area);
    Elem* raw = static_cast<Elem*>(cm.raw) + (uint64_t)wave_pos.o * cm.raw_channels + lane;
    Elem v[kPairsAhead];
#pragma unroll
    for (int k = 0; k < kPairsAhead; ++k) v[k] = off[k] < SPAN ? elems[off[k]] : (Elem)0;
#pragma unroll
    for (int k = 0; k < kPairsAhead; ++k) {
        if (off[k] < SPAN) {
            raw[k * kWave] = v[k];                            // the original bits
            elems[off[k]] = kQuietNaN;
        }
    }
    for (uint32_t i = kPairsAhead * kWave; i < pairs; i += kWave) {            // wave-uniform trip count
        const uint32_t o = pair_offset(walk, rows);
        pair_advance(cm, walk);
        if (o < SPAN) {
            raw[i] = elems[o];
            elems[o] = kQuietNaN;
        }
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
#pragma unroll
    for (int r = 0; r < ROWS; ++r) w[r] = in[r * kWave + lane];
}

// ---- interior spans: the 4-row layout --------------------------------------------------
//   * the four rows' min/max are reduce-scattered over each quad (lane xor 1 keeps two
//     rows, lane xor 2 keeps one), then all-reduced over the quads of the group by
//     exchanges that preserve lane mod 4 (row shifts / rotations, permlane swaps for
//     groups wider than 16 lanes), so each lane ends up holding the finished statistics
//     of ONE row: row = 2*(lane&1) + ((lane>>1)&1);
//   * scale and inverse of that row come from one division per lane, even quads
//     computing range/L and odd quads L/range, traded between neighbouring quads;
//   * the first quad of every group publishes the four rows' meta;
//   * fp32 (4 elements per lane and row): a Philox block (8 elements) spans a lane pair;
//     the even lane computes the blocks of rows 0 and 2, the odd lane those of rows 1
//     and 3, and they trade the halves.  bf16 (8 per lane and row): a block per lane and row.
template <typename InT, int G, int B, bool STOCH, bool MIXED>
__device__ __forceinline__ void compress_span(const CompressItem& it, int64_t wave_base, const InT* xw,
                                              uint8_t* pw, float* mw, uint32_t lane,
                                              uint8_t* stage_codes, float* stage_meta,
                                              const ChannelMap* cm, const ElemPos& wave_pos, const uint16_t* rows,
                                              u32x4 (&w)[4])
{
    using L = Layout<InT>;
    constexpr int ROWS = 4, EPL = L::EPL, ROW = L::ROW;
    constexpr int LPG = G / EPL;                              // lanes per group: 8 .. 64
    constexpr int RUN = LPG < 16 ? LPG : 16;                  // ... of which inside one DPP row
    constexpr int ROW_CODE_BYTES = ROW * B / 8;
    constexpr float Lf = (float)((1 << B) - 1);
    constexpr uint32_t POS = CodeByte<STOCH>::pos;
    static_assert(LPG >= 8 && LPG <= 64, "a group is 8 to 64 lanes");
    const bool b0 = lane & 1u, b1 = lane & 2u;

    float x[ROWS][EPL];
    if (MIXED && rows != nullptr) {                           // wave-uniform: one channel per element; `w` holds the span
        divert_listed<InT, ROWS>(*cm, wave_pos, rows, stage_codes, lane, w);
#pragma unroll
        for (int r = 0; r < ROWS; ++r) Loader<InT>::widen(w[r], x[r]);
    } else {
#pragma unroll
        for (int r = 0; r < ROWS; ++r) Loader<InT>::row(xw + r * ROW + lane * EPL, x[r]);
        if constexpr (MIXED) {
            KeptRun<EPL> run[ROWS];
            kept_runs<ROWS, EPL>(*cm, wave_pos, lane * EPL, ROW, run);
#pragma unroll
            for (int r = 0; r < ROWS; ++r)
                if (run[r].mask) divert_kept<InT, EPL>(*cm, run[r], x[r]);
        }
    }

    float mn[ROWS], mx[ROWS];
#pragma unroll
    for (int r = 0; r < ROWS; ++r) local_minmax<EPL>(x[r], mn[r], mx[r]);
    // reduce-scatter over the quad: odd lanes take rows 2,3, even lanes rows 0,1 ...
    float ka = b0 ? mn[2] : mn[0], kb = b0 ? mn[3] : mn[1];
    float Ka = b0 ? mx[2] : mx[0], Kb = b0 ? mx[3] : mx[1];
    exchange_xor1(ka, b0 ? mn[0] : mn[2], Ka, b0 ? mx[0] : mx[2]);
    exchange_xor1(kb, b0 ? mn[1] : mn[3], Kb, b0 ? mx[1] : mx[3]);
    // ... then lanes with bit 1 set take the second of their two rows
    float lo = b1 ? kb : ka, hi = b1 ? Kb : Ka;
    exchange_xor2(lo, b1 ? ka : kb, hi, b1 ? Ka : Kb);
    // finished over the quad; now over the quads of the group
    allreduce_mod4<RUN>(lo, hi);
    if constexpr (LPG >= 32) {
        float a, b;
        self_swap<16>(lo, a, b);  lo = vmin(a, b);
        self_swap<16>(hi, a, b);  hi = vmax(a, b);
    }
    if constexpr (LPG >= 64) {
        float a, b;
        self_swap<32>(lo, a, b);  lo = vmin(a, b);
        self_swap<32>(hi, a, b);  hi = vmax(a, b);
    }
    // this lane now holds min/max of row `held` for its group
    const uint32_t held = (b0 ? 2u : 0u) + (b1 ? 1u : 0u);

    // one division per lane: even quads range / L, odd quads L / range
    const float range = hi - lo;
    const bool degenerate = !(range >= 0x1p-100f);            // also a group without normal elements (NaN)
    const bool odd_quad = lane & 4u;
    const float mine = (odd_quad ? Lf : range) / (odd_quad ? range : Lf);      // IEEE-correct division
    const float other = from_other_quad<RUN>(mine);
    const float scale = degenerate ? 0.0f : (odd_quad ? other : mine);
    const float inv = degenerate ? 0.0f : (odd_quad ? mine : other);

    // the first quad of every group publishes the meta of the four rows (-0.0 -> +0.0)
    float zero = lo + 0.0f;
    if constexpr (MIXED) zero = lo == lo ? zero : 0.0f;       // no normal element: {0, 0}
    if ((lane & (LPG - 1)) < 4u)
        *reinterpret_cast<stage_f32x2*>(stage_meta + 2 * (held * (ROW / G) + lane / LPG)) = f32x2{scale, zero};

    // complemented random words of this lane's elements, per row; a span starts on a
    // multiple of its block count, so the additions below never carry out of the low word
    uint32_t nr[ROWS][EPL / 2] = {};
    if constexpr (STOCH) {
        const uint64_t blk = (uint64_t)wave_base >> 3;
        const uint32_t ctr_hi = (uint32_t)(blk >> 32);
        const uint32_t t_lo = (uint32_t)it.tensor_id, t_hi = (uint32_t)(it.tensor_id >> 32);
        const uint32_t k_lo = (uint32_t)it.seed, k_hi = (uint32_t)(it.seed >> 32);
        if constexpr (EPL == 8) {
#pragma unroll
            for (int r = 0; r < ROWS; ++r) {
                const u32x4 w = philox4x32_10((uint32_t)blk + r * (ROW / 8) + lane, ctr_hi, t_lo, t_hi, k_lo, k_hi);
                nr[r][0] = ~w.x; nr[r][1] = ~w.y; nr[r][2] = ~w.z; nr[r][3] = ~w.w;
            }
        } else {
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const uint32_t ctr_lo = (uint32_t)blk + (2u * j + (b0 ? 1u : 0u)) * (ROW / 8) + (lane >> 1);
                const u32x4 w = philox4x32_10(ctr_lo, ctr_hi, t_lo, t_hi, k_lo, k_hi);
                const uint32_t n0 = ~w.x, n1 = ~w.y, n2 = ~w.z, n3 = ~w.w;
                // even lane: owns words 0,1 of both rows' blocks; odd lane: words 2,3
                const uint32_t r0 = from_pair_lane_u32(b0 ? n0 : n2);
                const uint32_t r1 = from_pair_lane_u32(b0 ? n1 : n3);
                nr[2 * j][0] = b0 ? r0 : n0;      nr[2 * j][1] = b0 ? r1 : n1;       // row 2j: the even lane's block
                nr[2 * j + 1][0] = b0 ? n2 : r0;  nr[2 * j + 1][1] = b0 ? n3 : r1;   // row 2j+1: the odd lane's block
            }
        }
    }

#pragma unroll
    for (int r = 0; r < ROWS; ++r) {
        float q[EPL];
        // rows 0,1,2,3 are held by quad lanes 0,2,1,3
#pragma unroll
        for (int h = 0; h < EPL; h += 4) {
            if (r == 0) scaled_offsets<0>(x[r][h], x[r][h + 1], x[r][h + 2], x[r][h + 3], lo, inv, q + h);
            else if (r == 1) scaled_offsets<2>(x[r][h], x[r][h + 1], x[r][h + 2], x[r][h + 3], lo, inv, q + h);
            else if (r == 2) scaled_offsets<1>(x[r][h], x[r][h + 1], x[r][h + 2], x[r][h + 3], lo, inv, q + h);
            else scaled_offsets<3>(x[r][h], x[r][h + 1], x[r][h + 2], x[r][h + 3], lo, inv, q + h);
        }
        uint32_t e[EPL];
#pragma unroll
        for (int j = 0; j < EPL; j += 2) {
            e[j] = element_word<B, STOCH, 0>(q[j], nr[r][j >> 1]);
            e[j + 1] = element_word<B, STOCH, 1>(q[j + 1], nr[r][j >> 1]);
        }
        // codes go to the staging area in element order
        uint8_t* sc = stage_codes + r * ROW_CODE_BYTES + lane * (EPL * B / 8);
        if constexpr (EPL == 8) {
            uint32_t w0, w1;
            pack8<B, POS>(e, w0, w1);
            if constexpr (B == 8) *reinterpret_cast<stage_u32x2*>(sc) = u32x2{w0, w1};
            else if constexpr (B == 4) *reinterpret_cast<stage_u32*>(sc) = w0;
            else *reinterpret_cast<stage_u16*>(sc) = (uint16_t)w0;
        } else {
            const uint32_t w = pack4<B, POS>(e);
            if constexpr (B == 8) *reinterpret_cast<stage_u32*>(sc) = w;
            else if constexpr (B == 4) *reinterpret_cast<stage_u16*>(sc) = (uint16_t)w;
            else *reinterpret_cast<stage_u8*>(sc) = (uint8_t)w;
        }
    }

    // The span's codes leave as contiguous runs: each store instruction writes 16, 8 or 4
    // bytes per lane in lane order.  LDS operations of one wave complete in order, so the
    // reads see the writes above; the fence only orders the compiler.
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    constexpr int SPAN_CODE_BYTES = ROWS * ROW_CODE_BYTES;    // 256 .. 2048
    if constexpr (SPAN_CODE_BYTES >= 1024) {
#pragma unroll
        for (int k = 0; k < SPAN_CODE_BYTES / 1024; ++k) {
            const u32x4 c = *reinterpret_cast<const stage_u32x4*>(stage_codes + k * 1024 + lane * 16);
            code_store(reinterpret_cast<u32x4*>(pw + k * 1024 + lane * 16), c);
        }
    } else if constexpr (SPAN_CODE_BYTES == 512) {
        const u32x2 c = *reinterpret_cast<const stage_u32x2*>(stage_codes + lane * 8);
        code_store(reinterpret_cast<u32x2*>(pw + lane * 8), c);
    } else {
        const uint32_t c = *reinterpret_cast<const stage_u32*>(stage_codes + lane * 4);
        code_store(reinterpret_cast<uint32_t*>(pw + lane * 4), c);
    }
    // likewise the span's meta pairs: one 8-byte store from each of the first lanes
    constexpr uint32_t kGroups = L::SPAN / G;                 // 4 .. 32
    if (lane < kGroups)
        *reinterpret_cast<f32x2*>(mw + 2 * lane) = *reinterpret_cast<const stage_f32x2*>(stage_meta + 2 * lane);
}

// ---- the guarded layout (last tile of a tensor): 8 elements per lane -----------------------
// scale = range / L and inv = L / range with ONE division per lane: even lanes divide
// range by L, odd lanes L by range, and neighbours (always in the same group, so they
// hold the same range) trade results.
template <int B>
__device__ __forceinline__ void scale_and_inverse(float range, bool odd_lane, float& scale, float& inv)
{
    constexpr float Lf = (float)((1 << B) - 1);
    const bool degenerate = range < 0x1p-100f;
    const float num = odd_lane ? Lf : range;
    const float den = odd_lane ? range : Lf;
    const float mine = num / den;                             // IEEE-correct division
    const float other = from_pair_lane(mine);
    scale = degenerate ? 0.0f : (odd_lane ? other : mine);
    inv = degenerate ? 0.0f : (odd_lane ? mine : other);
}

template <int B>
__device__ __forceinline__ void store_codes(uint8_t* dst, uint32_t w0, uint32_t w1)
{
    if constexpr (B == 8) {
        code_store(reinterpret_cast<u32x2*>(dst), u32x2{w0, w1});
    } else if constexpr (B == 4) {
        code_store(reinterpret_cast<uint32_t*>(dst), w0);
    } else {
        code_store(reinterpret_cast<uint16_t*>(dst), (uint16_t)w0);
    }
}

// The tensor ends inside this wave's span.  All 64 lanes stay active through the
// reductions; missing elements enter them as +inf / -inf and get code 0.
template <typename InT, int G, int B, bool STOCH, bool MIXED>
__device__ __forceinline__ void compress_edge(const CompressItem& it, int64_t wave_base, int64_t extent,
                                              const InT* xw, uint8_t* pw, float* mw, uint32_t lane,
                                              const ChannelMap* cm, const ElemPos& wave_pos)
{
    constexpr int LPG = G / kEPL;                             // lanes per group
    constexpr int LOGG = Log2<G>::v;
    constexpr uint32_t POS = CodeByte<STOCH>::pos;
    const bool odd_lane = lane & 1u;
    const int64_t numel = it.numel;
    for (int r = 0; r < Layout<InT>::EDGE_ROWS; ++r) {
        const int64_t row_base = wave_base + r * kRow;
        if (row_base >= extent) break;                        // wave-uniform
        const uint32_t e0 = r * kRow + lane * kEPL;           // element offset from wave_base
        const int64_t i0 = row_base + lane * kEPL;
        const int64_t left = numel - i0;
        const int valid = left >= kEPL ? kEPL : (left > 0 ? (int)left : 0);
        float x[kEPL];
#pragma unroll
        for (int j = 0; j < kEPL; ++j) x[j] = j < valid ? Loader<InT>::one(xw, e0 + j) : 0.0f;
        uint32_t keptm = 0u;
        if constexpr (MIXED) {
            KeptRun<kEPL> run[1];
            kept_runs<1, kEPL>(*cm, wave_pos, e0, 0, run);
            run[0].mask &= (1u << valid) - 1u;
            keptm = run[0].mask;
            if (keptm) divert_kept<InT, kEPL>(*cm, run[0], x);
        }
        float mn = 0.0f, mx = 0.0f;
#pragma unroll
        for (int j = 0; j < kEPL; ++j) {
            const bool ok = j < valid;
            const float lo = ok ? x[j] : __builtin_inff();
            const float hi = ok ? x[j] : -__builtin_inff();
            mn = j == 0 ? lo : vmin(mn, lo);
            mx = j == 0 ? hi : vmax(mx, hi);
        }
        group_minmax<LPG>(mn, mx);
        if (!(mn <= mx)) { mn = 0.0f; mx = 0.0f; }            // a run with no (normal) element at all
        float scale, inv;
        scale_and_inverse<B>(mx - mn, odd_lane, scale, inv);
        // a group exists iff its first element does
        if ((lane & (LPG - 1)) == 0 && i0 < numel)
            *reinterpret_cast<f32x2*>(mw + 2 * (e0 >> LOGG)) = f32x2{scale, mn + 0.0f};   // -0.0 -> +0.0
        // a row starts on a multiple of 512 elements = 64 Philox blocks, so adding the lane
        // never carries out of the low counter word
        uint32_t nr[4] = {0u, 0u, 0u, 0u};
        if constexpr (STOCH) {
            const uint64_t blk = (uint64_t)row_base >> 3;
            const u32x4 w = philox4x32_10((uint32_t)blk + lane, (uint32_t)(blk >> 32),
                                          (uint32_t)it.tensor_id, (uint32_t)(it.tensor_id >> 32),
                                          (uint32_t)it.seed, (uint32_t)(it.seed >> 32));
            nr[0] = ~w.x; nr[1] = ~w.y; nr[2] = ~w.z; nr[3] = ~w.w;
        }
        uint32_t e[kEPL];
#pragma unroll
        for (int j = 0; j < kEPL; j += 2) {
            const float t0 = x[j] - mn, t1 = x[j + 1] - mn;
            e[j] = element_word<B, STOCH, 0>(t0 * inv, nr[j >> 1]);
            e[j + 1] = element_word<B, STOCH, 1>(t1 * inv, nr[j >> 1]);
        }
#pragma unroll
        for (int j = 0; j < kEPL; ++j) e[j] = (j < valid && !(keptm & (1u << j))) ? e[j] : 0u;
        uint32_t w0, w1;
        pack8<B, POS>(e, w0, w1);
        // chunks are size-aligned and the padded length is a multiple of 16, so a chunk is
        // either wholly inside the buffer or wholly outside
        const uint64_t off = (uint64_t)i0 * B / 8;
        if (off < it.packed_padded) store_codes<B>(pw + (e0 * B >> 3), w0, w1);
    }
}

// `listed` (MIXED only): LDS for the list of raw-store rows, built here -- by every thread of the workgroup, which
// all call this with the same arguments -- when the tensor has one channel per element.
template <typename InT, int G, int B, bool STOCH, bool MIXED = false>
__device__ __forceinline__ void compress_tile(const CompressItem& it, uint32_t tile, uint32_t* stage,
                                              const ChannelMap* cm = nullptr, uint16_t* listed = nullptr,
                                              uint32_t stage_dwords = kStageDwords)
{
    using L = Layout<InT>;
    const uint32_t lane = threadIdx.x & (kWave - 1);
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t numel = it.numel;
    // everything derived from wave_base is wave-uniform and lives in scalar registers;
    // lanes add 32-bit offsets
    const int64_t wave_base = (int64_t)tile * L::TILE + (int64_t)wave * L::SPAN;
    const int64_t padded_elems = (int64_t)(it.packed_padded * 8u / (unsigned)B);
    const int64_t extent = numel > padded_elems ? numel : padded_elems;
    const bool interior = wave_base + L::SPAN <= numel;
    const InT* xw = static_cast<const InT*>(it.x) + wave_base;
    const uint16_t* rows = nullptr;
    u32x4 w[4] = {};
    if constexpr (MIXED) {
        if (rows_listed(*cm)) {
            // the table entries first, then the span (so that waiting for the former does not wait for the latter),
            // and the list is filed while the span is on its way
            SlotWords words;
            list_rows_request<kCBlock>(*cm, words);
            // (the filing is written out on both paths: behind their join the compiler could not tell how many loads
            // are outstanding and would wait for the span before the table entries may be used)
            if (interior) {
#pragma unroll
                for (int r = 0; r < 4; ++r) w[r] = stream_load(reinterpret_cast<const u32x4*>(xw + r * L::ROW + lane * L::EPL));
                list_rows_file<kCBlock>(*cm, words, listed);
            } else {
                list_rows_file<kCBlock>(*cm, words, listed);
            }
            rows = listed;
        }
    }
    if (wave_base >= extent) return;

    uint8_t* pw = it.packed + ((uint64_t)wave_base * B >> 3);
    float* mw = it.meta + 2 * (wave_base >> Log2<G>::v);
    ElemPos wave_pos = {0u, 0u, 0u};
    if constexpr (MIXED) wave_pos = locate_base(*cm, (uint32_t)wave_base);
    if (interior) {
        uint8_t* stage_codes = reinterpret_cast<uint8_t*>(stage + wave * stage_dwords);
        float* stage_meta = reinterpret_cast<float*>(stage_codes + kStageCodeBytes);
        compress_span<InT, G, B, STOCH, MIXED>(it, wave_base, xw, pw, mw, lane, stage_codes, stage_meta, cm, wave_pos, rows, w);
    } else {
        compress_edge<InT, G, B, STOCH, MIXED>(it, wave_base, extent, xw, pw, mw, lane, cm, wave_pos);
    }
}

template <typename InT, int G>
__global__ __launch_bounds__(kCBlock) void compress_kernel(const CompressBatch args)
{
    const uint32_t bid = blockIdx.x;
    int lo = 0, hi = args.count;                              // last item with tile_start <= bid
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (args.tile_start[mid] <= bid) lo = mid; else hi = mid;
    }
    const CompressItem& it = args.item[lo];
    const uint32_t tile = bid - args.tile_start[lo];
    __shared__ __attribute__((aligned(16))) uint32_t stage[kWaves * kStageDwords];
    switch (it.bits * 2 + it.stochastic) {
        case 4:  compress_tile<InT, G, 2, false>(it, tile, stage); break;
        case 5:  compress_tile<InT, G, 2, true >(it, tile, stage); break;
        case 8:  compress_tile<InT, G, 4, false>(it, tile, stage); break;
        case 9:  compress_tile<InT, G, 4, true >(it, tile, stage); break;
        case 16: compress_tile<InT, G, 8, false>(it, tile, stage); break;
        case 17: compress_tile<InT, G, 8, true >(it, tile, stage); break;
        default: break;
    }
}

// Tensors whose kept channels go to the raw store.  A wave's staging area also parks the span's
// input while its kept elements are taken out (4 KiB: 2048 bf16 or 1024 fp32 elements).
constexpr int kMixedStageDwords = 1024;
static_assert(kMixedStageDwords >= kStageDwords && kMixedStageDwords * 4 == Layout<float>::SPAN * 4 &&
              kMixedStageDwords * 4 == Layout<uint16_t>::SPAN * 2, "a span of either dtype is 4 KiB");

template <typename InT, int G>
__global__ __launch_bounds__(kCBlock) void compress_mixed_kernel(const Batch<MixedCompressJob> batch)
{
    __shared__ __attribute__((aligned(16))) uint32_t stage[kWaves * kMixedStageDwords];
    __shared__ uint16_t listed[kListedRows];
    uint32_t tile;
    const MixedCompressJob& job = batch.item[batch_item(batch, blockIdx.x, tile)];
    const CompressItem& it = job.it;
    const ChannelMap& cm = job.cm;
    if (nothing_kept(cm)) {                                   // the classification found no salient channel: the plain code
        switch (it.bits * 2 + it.stochastic) {
            case 4:  compress_tile<InT, G, 2, false>(it, tile, stage); break;
            case 5:  compress_tile<InT, G, 2, true >(it, tile, stage); break;
            case 8:  compress_tile<InT, G, 4, false>(it, tile, stage); break;
            case 9:  compress_tile<InT, G, 4, true >(it, tile, stage); break;
            case 16: compress_tile<InT, G, 8, false>(it, tile, stage); break;
            case 17: compress_tile<InT, G, 8, true >(it, tile, stage); break;
            default: break;
        }
        return;
    }
    switch (it.bits * 2 + it.stochastic) {
        case 4:  compress_tile<InT, G, 2, false, true>(it, tile, stage, &cm, listed, kMixedStageDwords); break;
        case 5:  compress_tile<InT, G, 2, true , true>(it, tile, stage, &cm, listed, kMixedStageDwords); break;
        case 8:  compress_tile<InT, G, 4, false, true>(it, tile, stage, &cm, listed, kMixedStageDwords); break;
        case 9:  compress_tile<InT, G, 4, true , true>(it, tile, stage, &cm, listed, kMixedStageDwords); break;
        case 16: compress_tile<InT, G, 8, false, true>(it, tile, stage, &cm, listed, kMixedStageDwords); break;
        case 17: compress_tile<InT, G, 8, true , true>(it, tile, stage, &cm, listed, kMixedStageDwords); break;
        default: break;
    }
}

}  // namespace

int compress_tile_elems(int dtype, int) { return dtype == 0 ? Layout<float>::TILE : Layout<uint16_t>::TILE; }

hipError_t launch_compress(const CompressBatch& b, int dtype, int group_size, hipStream_t s)
{
    const uint32_t tiles = b.tile_start[b.count];
    if (tiles == 0) return hipSuccess;
    const dim3 grid(tiles), block(kCBlock);
#define FH_LAUNCH(T, GS) hipLaunchKernelGGL((compress_kernel<T, GS>), grid, block, 0, s, b)
    if (dtype == 0) {
        if (group_size == 64) FH_LAUNCH(float, 64);
        else if (group_size == 128) FH_LAUNCH(float, 128);
        else FH_LAUNCH(float, 256);
    } else {
        if (group_size == 64) FH_LAUNCH(uint16_t, 64);
        else if (group_size == 128) FH_LAUNCH(uint16_t, 128);
        else FH_LAUNCH(uint16_t, 256);
    }
#undef FH_LAUNCH
    return hipGetLastError();
}

hipError_t launch_compress_mixed(const Batch<MixedCompressJob>& b, int dtype, int group_size, hipStream_t s)
{
    const uint32_t tiles = b.block_start[b.count];
    if (tiles == 0) return hipSuccess;
    const dim3 grid(tiles), block(kCBlock);
#define FH_LAUNCH(T, GS) hipLaunchKernelGGL((compress_mixed_kernel<T, GS>), grid, block, 0, s, b)
    if (dtype == 0) {
        if (group_size == 64) FH_LAUNCH(float, 64);
        else if (group_size == 128) FH_LAUNCH(float, 128);
        else FH_LAUNCH(float, 256);
    } else {
        if (group_size == 64) FH_LAUNCH(uint16_t, 64);
        else if (group_size == 128) FH_LAUNCH(uint16_t, 128);
        else FH_LAUNCH(uint16_t, 256);
    }
#undef FH_LAUNCH
    return hipGetLastError();
}

}  // namespace fh
