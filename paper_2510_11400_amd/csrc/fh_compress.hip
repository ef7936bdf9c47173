// Forward side of the group quantiser on gfx950: one pass over the activation.
//
// Each lane owns 8 consecutive elements (two 128-bit loads for fp32, one for bf16),
// which is also exactly one Philox block, so stochastic rounding needs no cross-lane
// traffic for its random bits.  A group of G elements is a run of G/8 lanes; its
// min/max come from DPP / permlane exchanges, its scale from two IEEE divisions per
// lane-run, and each lane packs its own 8 codes into 8, 4 or 2 bytes that land in
// memory in lane order, so every load and store of a wave is one contiguous span.
//
// Follows the paper's Section 4.4.1 (normal channels: linear-scale quantisation;
// zeros must be preserved) with the parameters the paper leaves open taken from the
// caller (group size, bits, rounding, seed).
#include "fh_device.hpp"
#include "fh_kernels.hpp"

namespace fh {

namespace {

#ifndef FH_COMPRESS_BLOCK
#define FH_COMPRESS_BLOCK 256
#endif
constexpr int kCBlock = FH_COMPRESS_BLOCK;   // threads per workgroup
constexpr int kEPL = 8;                  // elements per lane
constexpr int kRow = kWave * kEPL;       // elements one wave covers per row: 512
#ifndef FH_COMPRESS_ROWS
#define FH_COMPRESS_ROWS 2
#endif
constexpr int kRowsPerWave = FH_COMPRESS_ROWS;   // rows whose loads are issued before any is consumed
constexpr int kWaveSpan = kRowsPerWave * kRow;
constexpr int kTile = (kCBlock / kWave) * kWaveSpan;   // 4096 elements per workgroup

// Per-wave LDS staging area: the codes of the wave's span in element order (at most one
// byte per element) followed by its groups' {scale, zero} pairs (at most span/64).
// Each wave only touches its own area, so no workgroup barrier is involved.
#ifndef FH_COMPRESS_LDS
#define FH_COMPRESS_LDS 1
#endif
// the staging area is written and read back through different widths
typedef uint16_t __attribute__((may_alias)) stage_u16;
typedef uint32_t __attribute__((may_alias)) stage_u32;
typedef u32x2 __attribute__((may_alias)) stage_u32x2;
typedef u32x4 __attribute__((may_alias)) stage_u32x4;
typedef f32x2 __attribute__((may_alias)) stage_f32x2;
constexpr int kStageCodeBytes = kWaveSpan;
constexpr int kStageMetaBytes = (kWaveSpan / 64) * 8;
constexpr int kStageDwords = (kStageCodeBytes + kStageMetaBytes) / 4;
static_assert(kRowsPerWave == 2 || !FH_COMPRESS_LDS, "the staged store assumes two rows per wave");

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

// Quantise the 8 values of one lane and pack their codes.  `valid` = number of leading
// elements that exist (8 except in the last lanes of a tensor); the others get code 0.
// (ctr_lo, ctr_hi) is the Philox block index of these 8 elements.
template <int B, bool STOCH, bool FULL>
__device__ __forceinline__ void quantise8(const float (&x)[kEPL], float mn, float inv, int valid,
                                          uint32_t ctr_lo, uint32_t ctr_hi, uint64_t seed, uint64_t tensor_id,
                                          uint32_t& w0, uint32_t& w1)
{
    constexpr float Lf = (float)((1 << B) - 1);
    constexpr uint32_t POS = CodeByte<STOCH>::pos;
    uint32_t e[kEPL];
    uint32_t nrnd[4] = {0u, 0u, 0u, 0u};
    if constexpr (STOCH) {
        const u32x4 rnd = philox4x32_10(ctr_lo, ctr_hi, (uint32_t)tensor_id, (uint32_t)(tensor_id >> 32),
                                        (uint32_t)seed, (uint32_t)(seed >> 32));
        nrnd[0] = ~rnd.x; nrnd[1] = ~rnd.y; nrnd[2] = ~rnd.z; nrnd[3] = ~rnd.w;
    }
#pragma unroll
    for (int j = 0; j < kEPL; ++j) {
        const float t = x[j] - mn;
        float q = t * inv;
        q = __builtin_amdgcn_fmed3f(q, 0.0f, Lf);            // clamp to [0, L]
        if constexpr (STOCH) {
            const float Q = q * 65536.0f;                     // exact
            int neg_c;
            asm volatile("v_cvt_flr_i32_f32_e64 %0, -%1" : "=v"(neg_c) : "v"(Q));   // -ceil(Q)
            e[j] = (j & 1) ? halfword_minus<1>(nrnd[j >> 1], neg_c) : halfword_minus<0>(nrnd[j >> 1], neg_c);
        } else {
            e[j] = __builtin_bit_cast(uint32_t, q + 0x1p23f);
        }
        if constexpr (!FULL) e[j] = (j < valid) ? e[j] : 0u;
    }
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

template <typename InT> struct Loader;

template <> struct Loader<float> {
    __device__ static __forceinline__ void full(const float* base, uint32_t i0, float (&x)[kEPL]) {
        const f32x4* p = reinterpret_cast<const f32x4*>(base + i0);
        const f32x4 a = stream_load(p), b = stream_load(p + 1);
        x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w;
        x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
    }
    __device__ static __forceinline__ float one(const float* base, uint32_t i) {
        return base[i];
    }
};

template <> struct Loader<uint16_t> {   // bf16 bit patterns; widening is exact
    __device__ static __forceinline__ void full(const uint16_t* base, uint32_t i0, float (&x)[kEPL]) {
        const u32x4 a = stream_load(reinterpret_cast<const u32x4*>(base + i0));
        x[0] = bf16_lo(a.x); x[1] = bf16_hi(a.x); x[2] = bf16_lo(a.y); x[3] = bf16_hi(a.y);
        x[4] = bf16_lo(a.z); x[5] = bf16_hi(a.z); x[6] = bf16_lo(a.w); x[7] = bf16_hi(a.w);
    }
    __device__ static __forceinline__ float one(const uint16_t* base, uint32_t i) {
        return __builtin_bit_cast(float, (uint32_t)base[i] << 16);
    }
};

// ---- fp32 interior spans: fully coalesced variant -----------------------------------
// With 4-byte elements the 8-per-lane layout makes a lane read 32 consecutive bytes,
// i.e. each wave load touches every other 16 bytes of its span, and that measures
// 6-8 % below lane-contiguous 16-byte loads on MI355X.  Interior fp32 spans therefore
// use a second layout over the same 1024 elements: 4 rows of 256, lane l owning the 4
// elements at 4*l of every row, so each load instruction reads 1 KiB contiguously.
// The price is cross-lane bookkeeping, organised so that it costs no more ALU work
// than the other layout:
//   * the four rows' min/max are reduce-scattered over each quad (lane xor 1 keeps two
//     rows, lane xor 2 keeps one), all-reduced across quads with row rotations that
//     preserve lane mod 4 (plus permlane swaps for groups wider than 16 lanes), so each
//     lane ends up holding the finished statistics of ONE row: row = 2*(lane&1) + ((lane>>1)&1);
//   * scale and inverse of that row come from one division per lane, even quads
//     computing range/L and odd quads L/range, traded by a rotation of 4;
//   * the subtract and multiply of the quantiser read `mn` and `inv` of row r straight
//     from the quad lane that holds them (DPP quad_perm broadcast on the operand);
//   * a Philox block (8 elements) spans a lane pair: the even lane computes the blocks of
//     rows 0 and 2, the odd lane those of rows 1 and 3, and they trade the halves.
// Results are identical to the other layout because nothing in the definition depends
// on which lane does what.
#ifndef FH_COMPRESS_F32_COALESCED
#define FH_COMPRESS_F32_COALESCED 1
#endif
typedef uint8_t __attribute__((may_alias)) stage_u8;

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

// all-reduce over the four lanes of a 16-lane row that share lane mod 4
__device__ __forceinline__ void allreduce_mod4(float& mn, float& mx)
{
    asm volatile("s_nop 1\n\t"
                 "v_min_f32_dpp %0, %0, %0 row_ror:4" FH_DPP_TAIL
                 "v_max_f32_dpp %1, %1, %1 row_ror:4" FH_DPP_TAIL
                 "s_nop 0\n\t"
                 "v_min_f32_dpp %0, %0, %0 row_ror:8" FH_DPP_TAIL
                 "v_max_f32_dpp %1, %1, %1 row_ror:8" FH_DPP_TAIL "s_nop 1"
                 : "+v"(mn), "+v"(mx));
}

// q[j] = (x[j] - mn_row) * inv_row with mn_row / inv_row read from quad lane HOLDER
template <int HOLDER>
__device__ __forceinline__ void scaled_offsets(const f32x4 x, float mn_held, float inv_held, float (&q)[4])
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
                 : "v"(x.x), "v"(x.y), "v"(x.z), "v"(x.w), "v"(mn_held), "v"(inv_held))
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

template <int G, int B, bool STOCH>
__device__ __forceinline__ void compress_span_f32(const CompressItem& it, int64_t wave_base, const float* xw,
                                                  uint8_t* pw, float* mw, uint32_t lane,
                                                  uint8_t* stage_codes, float* stage_meta)
{
    constexpr int ROWS = 4, ROW = 256;
    static_assert(ROWS * ROW == kWaveSpan, "same span as the other layout");
    constexpr int LPG = G / 4;                                // lanes per group: 16, 32 or 64
    constexpr float Lf = (float)((1 << B) - 1);
    constexpr uint32_t POS = CodeByte<STOCH>::pos;
    const bool b0 = lane & 1u, b1 = lane & 2u;

    f32x4 x[ROWS];
#pragma unroll
    for (int r = 0; r < ROWS; ++r)
        x[r] = stream_load(reinterpret_cast<const f32x4*>(xw + r * ROW) + lane);

    float mn[ROWS], mx[ROWS];
#pragma unroll
    for (int r = 0; r < ROWS; ++r) {
        mn[r] = vmin(vmin3(x[r].x, x[r].y, x[r].z), x[r].w);
        mx[r] = vmax(vmax3(x[r].x, x[r].y, x[r].z), x[r].w);
    }
    // reduce-scatter over the quad: odd lanes take rows 2,3, even lanes rows 0,1 ...
    float ka = b0 ? mn[2] : mn[0], kb = b0 ? mn[3] : mn[1];
    float Ka = b0 ? mx[2] : mx[0], Kb = b0 ? mx[3] : mx[1];
    exchange_xor1(ka, b0 ? mn[0] : mn[2], Ka, b0 ? mx[0] : mx[2]);
    exchange_xor1(kb, b0 ? mn[1] : mn[3], Kb, b0 ? mx[1] : mx[3]);
    // ... then lanes with bit 1 set take the second of their two rows
    float lo = b1 ? kb : ka, hi = b1 ? Kb : Ka;
    exchange_xor2(lo, b1 ? ka : kb, hi, b1 ? Ka : Kb);
    // finished over the quad; now over the quads of the group
    allreduce_mod4(lo, hi);
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
    const bool degenerate = range < 0x1p-100f;
    const bool odd_quad = lane & 4u;
    const float mine = (odd_quad ? Lf : range) / (odd_quad ? range : Lf);      // IEEE-correct division
    const float other = __builtin_bit_cast(float,
        __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, mine), 0x124, 0xF, 0xF, true));   // row_ror:4
    const float scale = degenerate ? 0.0f : (odd_quad ? other : mine);
    const float inv = degenerate ? 0.0f : (odd_quad ? mine : other);

    // the first quad of every group publishes the meta of the four rows
    if ((lane & (LPG - 1)) < 4u)
        *reinterpret_cast<stage_f32x2*>(stage_meta + 2 * (held * (ROW / G) + lane / LPG)) = f32x2{scale, lo + 0.0f};

    // random bits: this lane's blocks are those of rows b0 and b0 + 2; a span starts on a
    // multiple of 128 blocks, so the additions below never carry out of the low word
    uint32_t nr[ROWS][2] = {};
    if constexpr (STOCH) {
        const uint64_t blk = (uint64_t)wave_base >> 3;
        const uint32_t ctr_hi = (uint32_t)(blk >> 32);
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const uint32_t ctr_lo = (uint32_t)blk + (2u * j + (b0 ? 1u : 0u)) * (ROW / 8) + (lane >> 1);
            const u32x4 w = philox4x32_10(ctr_lo, ctr_hi, (uint32_t)it.tensor_id, (uint32_t)(it.tensor_id >> 32),
                                          (uint32_t)it.seed, (uint32_t)(it.seed >> 32));
            const uint32_t n0 = ~w.x, n1 = ~w.y, n2 = ~w.z, n3 = ~w.w;
            // even lane: owns words 0,1 of both rows' blocks; odd lane: words 2,3
            const uint32_t r0 = from_pair_lane_u32(b0 ? n0 : n2);
            const uint32_t r1 = from_pair_lane_u32(b0 ? n1 : n3);
            nr[2 * j][0] = b0 ? r0 : n0;      nr[2 * j][1] = b0 ? r1 : n1;       // row 2j: block of the even lane
            nr[2 * j + 1][0] = b0 ? n2 : r0;  nr[2 * j + 1][1] = b0 ? n3 : r1;   // row 2j+1: block of the odd lane
        }
    }

#pragma unroll
    for (int r = 0; r < ROWS; ++r) {
        float q[4];
        // rows 0,1,2,3 are held by quad lanes 0,2,1,3
        if (r == 0) scaled_offsets<0>(x[r], lo, inv, q);
        else if (r == 1) scaled_offsets<2>(x[r], lo, inv, q);
        else if (r == 2) scaled_offsets<1>(x[r], lo, inv, q);
        else scaled_offsets<3>(x[r], lo, inv, q);
        uint32_t e[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float c = __builtin_amdgcn_fmed3f(q[j], 0.0f, Lf);
            if constexpr (STOCH) {
                const float Q = c * 65536.0f;
                int neg_c;
                asm volatile("v_cvt_flr_i32_f32_e64 %0, -%1" : "=v"(neg_c) : "v"(Q));
                e[j] = (j & 1) ? halfword_minus<1>(nr[r][j >> 1], neg_c) : halfword_minus<0>(nr[r][j >> 1], neg_c);
            } else {
                e[j] = __builtin_bit_cast(uint32_t, c + 0x1p23f);
            }
        }
        if constexpr (B == 8) {
            *reinterpret_cast<stage_u32*>(stage_codes + r * ROW + lane * 4) = quad_bytes<POS>(e[0], e[1], e[2], e[3]);
        } else if constexpr (B == 4) {
            const uint32_t w = (pair_bytes<POS>(e[1], e[3]) << 4) | pair_bytes<POS>(e[0], e[2]);
            *reinterpret_cast<stage_u16*>(stage_codes + r * (ROW / 2) + lane * 2) = (uint16_t)w;
        } else {
            // four 2-bit codes, one per byte, times (2^24 + 2^18 + 2^12 + 2^6): the shifted copies
            // fall into disjoint bit fields and the top byte collects c0 | c1<<2 | c2<<4 | c3<<6
            const uint32_t w = quad_bytes<POS>(e[0], e[1], e[2], e[3]) * 0x01041040u;
            *reinterpret_cast<stage_u8*>(stage_codes + r * (ROW / 4) + lane) = (uint8_t)(w >> 24);
        }
    }

    // the span's codes and meta leave as one contiguous store each (see compress_tile)
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    if constexpr (B == 8) {
        const u32x4 c = *reinterpret_cast<const stage_u32x4*>(stage_codes + lane * 16);
        code_store(reinterpret_cast<u32x4*>(pw + lane * 16), c);
    } else if constexpr (B == 4) {
        const u32x2 c = *reinterpret_cast<const stage_u32x2*>(stage_codes + lane * 8);
        code_store(reinterpret_cast<u32x2*>(pw + lane * 8), c);
    } else {
        const uint32_t c = *reinterpret_cast<const stage_u32*>(stage_codes + lane * 4);
        code_store(reinterpret_cast<uint32_t*>(pw + lane * 4), c);
    }
    constexpr uint32_t kGroups = kWaveSpan / G;
    if (lane < kGroups)
        *reinterpret_cast<f32x2*>(mw + 2 * lane) = *reinterpret_cast<const stage_f32x2*>(stage_meta + 2 * lane);
}

template <typename InT, int G, int B, bool STOCH>
__device__ __forceinline__ void compress_tile(const CompressItem& it, uint32_t tile, uint32_t* stage)
{
    constexpr int LPG = G / kEPL;                             // lanes per group
    constexpr int LOGG = Log2<G>::v;
    const uint32_t lane = threadIdx.x & (kWave - 1);
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const bool odd_lane = lane & 1u;
    const int64_t numel = it.numel;
    // everything derived from wave_base is wave-uniform and lives in scalar registers;
    // lanes add 32-bit offsets
    const int64_t wave_base = (int64_t)tile * kTile + (int64_t)wave * kWaveSpan;
    const int64_t padded_elems = (int64_t)(it.packed_padded * 8u / (unsigned)B);
    const int64_t extent = numel > padded_elems ? numel : padded_elems;
    if (wave_base >= extent) return;

    const InT* xw = static_cast<const InT*>(it.x) + wave_base;
    uint8_t* pw = it.packed + ((uint64_t)wave_base * B >> 3);
    float* mw = it.meta + 2 * (wave_base >> LOGG);
    const uint32_t lane_elem = lane * kEPL;                   // first element of the lane inside a row
    uint8_t* stage_codes = reinterpret_cast<uint8_t*>(stage + wave * kStageDwords);
    float* stage_meta = reinterpret_cast<float*>(stage_codes + kStageCodeBytes);

    if (wave_base + kWaveSpan <= numel) {
#if FH_COMPRESS_F32_COALESCED && FH_COMPRESS_LDS
        if constexpr (sizeof(InT) == 4) {
            compress_span_f32<G, B, STOCH>(it, wave_base, xw, pw, mw, lane, stage_codes, stage_meta);
            return;
        }
#endif
        // ---- interior: every element exists, every access is a full vector ----
        float x[kRowsPerWave][kEPL];
#pragma unroll
        for (int r = 0; r < kRowsPerWave; ++r)
            Loader<InT>::full(xw, r * kRow + lane_elem, x[r]);
#pragma unroll
        for (int r = 0; r < kRowsPerWave; ++r) {
            const uint32_t e0 = r * kRow + lane_elem;         // element offset from wave_base
            float mn = vmin3(x[r][0], x[r][1], x[r][2]), mx = vmax3(x[r][0], x[r][1], x[r][2]);
            mn = vmin3(mn, x[r][3], x[r][4]);  mx = vmax3(mx, x[r][3], x[r][4]);
            mn = vmin3(mn, x[r][5], x[r][6]);  mx = vmax3(mx, x[r][5], x[r][6]);
            mn = vmin(mn, x[r][7]);            mx = vmax(mx, x[r][7]);
            group_minmax<LPG>(mn, mx);
            float scale, inv;
            scale_and_inverse<B>(mx - mn, odd_lane, scale, inv);
#if FH_COMPRESS_LDS
            if ((lane & (LPG - 1)) == 0)
                *reinterpret_cast<stage_f32x2*>(stage_meta + 2 * (e0 >> LOGG)) = f32x2{scale, mn + 0.0f};   // -0.0 -> +0.0
#else
            if ((lane & (LPG - 1)) == 0)
                *reinterpret_cast<f32x2*>(mw + 2 * (e0 >> LOGG)) = f32x2{scale, mn + 0.0f};   // -0.0 -> +0.0
#endif
            // a row starts on a multiple of 512 elements = 64 Philox blocks, so adding the
            // lane never carries out of the low counter word
            const uint64_t blk = (uint64_t)(wave_base + r * kRow) >> 3;
            uint32_t w0, w1;
            quantise8<B, STOCH, true>(x[r], mn, inv, kEPL, (uint32_t)blk + lane, (uint32_t)(blk >> 32),
                                      it.seed, it.tensor_id, w0, w1);
#if FH_COMPRESS_LDS
            // codes go to the staging area in element order ...
            uint8_t* sc = stage_codes + (e0 * B >> 3);
            if constexpr (B == 8) *reinterpret_cast<stage_u32x2*>(sc) = u32x2{w0, w1};
            else if constexpr (B == 4) *reinterpret_cast<stage_u32*>(sc) = w0;
            else *reinterpret_cast<stage_u16*>(sc) = (uint16_t)w0;
#else
            store_codes<B>(pw + (e0 * B >> 3), w0, w1);
#endif
        }
#if FH_COMPRESS_LDS
        // ... and leave as ONE store per wave: lane l takes the 2*B bytes at l*2*B, so the
        // wave writes its 256 / 512 / 1024 code bytes as one contiguous run.  LDS
        // operations of one wave complete in order, so the reads see the writes above.
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");    // compiler ordering only: no instruction
        if constexpr (B == 8) {
            const u32x4 c = *reinterpret_cast<const stage_u32x4*>(stage_codes + lane * 16);
            code_store(reinterpret_cast<u32x4*>(pw + lane * 16), c);
        } else if constexpr (B == 4) {
            const u32x2 c = *reinterpret_cast<const stage_u32x2*>(stage_codes + lane * 8);
            code_store(reinterpret_cast<u32x2*>(pw + lane * 8), c);
        } else {
            const uint32_t c = *reinterpret_cast<const stage_u32*>(stage_codes + lane * 4);
            code_store(reinterpret_cast<uint32_t*>(pw + lane * 4), c);
        }
        // likewise the span's kWaveSpan / G meta pairs: one 8-byte store from each of the first lanes
        constexpr uint32_t kGroups = kWaveSpan / G;
        if (lane < kGroups)
            *reinterpret_cast<f32x2*>(mw + 2 * lane) = *reinterpret_cast<const stage_f32x2*>(stage_meta + 2 * lane);
#endif
        return;
    }

    // ---- edge: the tensor ends inside this wave's span.  All 64 lanes stay active
    //      through the reductions; missing elements enter them as +inf / -inf. ----
    for (int r = 0; r < kRowsPerWave; ++r) {
        const int64_t row_base = wave_base + r * kRow;
        if (row_base >= extent) break;                        // wave-uniform
        const uint32_t e0 = r * kRow + lane_elem;
        const int64_t i0 = row_base + lane_elem;
        const int64_t left = numel - i0;
        const int valid = left >= kEPL ? kEPL : (left > 0 ? (int)left : 0);
        float x[kEPL];
        float mn = 0.0f, mx = 0.0f;
#pragma unroll
        for (int j = 0; j < kEPL; ++j) {
            const bool ok = j < valid;
            x[j] = ok ? Loader<InT>::one(xw, e0 + j) : 0.0f;
            const float lo = ok ? x[j] : __builtin_inff();
            const float hi = ok ? x[j] : -__builtin_inff();
            mn = j == 0 ? lo : vmin(mn, lo);
            mx = j == 0 ? hi : vmax(mx, hi);
        }
        group_minmax<LPG>(mn, mx);
        if (mn > mx) { mn = 0.0f; mx = 0.0f; }                // a run with no element at all
        float scale, inv;
        scale_and_inverse<B>(mx - mn, odd_lane, scale, inv);
        // a group exists iff its first element does
        if ((lane & (LPG - 1)) == 0 && i0 < numel)
            *reinterpret_cast<f32x2*>(mw + 2 * (e0 >> LOGG)) = f32x2{scale, mn + 0.0f};
        const uint64_t blk = (uint64_t)row_base >> 3;
        uint32_t w0, w1;
        quantise8<B, STOCH, false>(x, mn, inv, valid, (uint32_t)blk + lane, (uint32_t)(blk >> 32),
                                   it.seed, it.tensor_id, w0, w1);
        // chunks are size-aligned and the padded length is a multiple of 16, so a chunk is
        // either wholly inside the buffer or wholly outside
        const uint64_t off = (uint64_t)i0 * B / 8;
        if (off < it.packed_padded) store_codes<B>(pw + (e0 * B >> 3), w0, w1);
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
    __shared__ __attribute__((aligned(16))) uint32_t stage[(kCBlock / kWave) * kStageDwords];
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

}  // namespace

int compress_tile_elems(int, int) { return kTile; }

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

}  // namespace fh
