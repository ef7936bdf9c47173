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

constexpr int kEPL = 8;                  // elements per lane
constexpr int kRow = kWave * kEPL;       // elements one wave covers per row: 512
#ifndef FH_COMPRESS_ROWS
#define FH_COMPRESS_ROWS 2
#endif
constexpr int kRowsPerWave = FH_COMPRESS_ROWS;   // rows whose loads are issued before any is consumed
constexpr int kWaveSpan = kRowsPerWave * kRow;
constexpr int kTile = (kBlock / kWave) * kWaveSpan;   // 4096 elements per workgroup

template <int G> struct Log2;
template <> struct Log2<64>  { static constexpr int v = 6; };
template <> struct Log2<128> { static constexpr int v = 7; };
template <> struct Log2<256> { static constexpr int v = 8; };

// Quantise and pack the 8 values of one lane.  `valid` = number of leading elements
// that exist (8 except in the last lanes of a tensor); codes of the others are 0.
template <int B, bool STOCH>
__device__ __forceinline__ void quantise8(const float (&x)[kEPL], float mn, float inv, int valid,
                                          int64_t i0, uint64_t seed, uint64_t tensor_id,
                                          uint32_t& w0, uint32_t& w1)
{
    constexpr float Lf = (float)((1 << B) - 1);
    uint32_t code[kEPL];
    u32x4 rnd = {0u, 0u, 0u, 0u};
    if constexpr (STOCH) {
        const uint64_t blk = (uint64_t)i0 >> 3;
        rnd = philox4x32_10((uint32_t)blk, (uint32_t)(blk >> 32),
                            (uint32_t)tensor_id, (uint32_t)(tensor_id >> 32),
                            (uint32_t)seed, (uint32_t)(seed >> 32));
    }
#pragma unroll
    for (int j = 0; j < kEPL; ++j) {
        const float t = x[j] - mn;
        float q = t * inv;
        q = __builtin_amdgcn_fmed3f(q, 0.0f, Lf);            // clamp to [0, L]
        uint32_t c;
        if constexpr (STOCH) {
            const float k = __builtin_floorf(q);
            const float f = q - k;                            // exact
            const uint32_t word = rnd[j >> 1];
            const uint32_t h = (j & 1) ? (word >> 16) : (word & 0xFFFFu);
            const float u = (float)h * 0x1p-16f;
            c = (uint32_t)k + (u < f ? 1u : 0u);
        } else {
            c = (uint32_t)__builtin_rintf(q);                 // v_rndne_f32: ties to even
        }
        code[j] = (j < valid) ? c : 0u;
    }
    if constexpr (B == 8) {
        w0 = code[0] | (code[1] << 8) | (code[2] << 16) | (code[3] << 24);
        w1 = code[4] | (code[5] << 8) | (code[6] << 16) | (code[7] << 24);
    } else if constexpr (B == 4) {
        w0 = code[0] | (code[1] << 4) | (code[2] << 8) | (code[3] << 12) |
             (code[4] << 16) | (code[5] << 20) | (code[6] << 24) | (code[7] << 28);
        w1 = 0u;
    } else {
        w0 = code[0] | (code[1] << 2) | (code[2] << 4) | (code[3] << 6) |
             (code[4] << 8) | (code[5] << 10) | (code[6] << 12) | (code[7] << 14);
        w1 = 0u;
    }
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
    __device__ static __forceinline__ void full(const void* base, int64_t i0, float (&x)[kEPL]) {
        const f32x4* p = reinterpret_cast<const f32x4*>(static_cast<const float*>(base) + i0);
        const f32x4 a = stream_load(p), b = stream_load(p + 1);
        x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w;
        x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
    }
    __device__ static __forceinline__ float one(const void* base, int64_t i) {
        return static_cast<const float*>(base)[i];
    }
};

template <> struct Loader<uint16_t> {   // bf16 bit patterns; widening is exact
    __device__ static __forceinline__ void full(const void* base, int64_t i0, float (&x)[kEPL]) {
        const u32x4 a = stream_load(reinterpret_cast<const u32x4*>(static_cast<const uint16_t*>(base) + i0));
        x[0] = bf16_lo(a.x); x[1] = bf16_hi(a.x); x[2] = bf16_lo(a.y); x[3] = bf16_hi(a.y);
        x[4] = bf16_lo(a.z); x[5] = bf16_hi(a.z); x[6] = bf16_lo(a.w); x[7] = bf16_hi(a.w);
    }
    __device__ static __forceinline__ float one(const void* base, int64_t i) {
        return __builtin_bit_cast(float, (uint32_t)static_cast<const uint16_t*>(base)[i] << 16);
    }
};

template <typename InT, int G, int B, bool STOCH>
__device__ __forceinline__ void compress_tile(const CompressItem& it, uint32_t tile)
{
    constexpr int LPG = G / kEPL;                             // lanes per group
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t numel = it.numel;
    const int64_t wave_base = (int64_t)tile * kTile + (int64_t)wave * kWaveSpan;
    const int64_t padded_elems = (int64_t)(it.packed_padded * 8u / (unsigned)B);
    const int64_t extent = numel > padded_elems ? numel : padded_elems;
    if (wave_base >= extent) return;

    if (wave_base + kWaveSpan <= numel) {
        // ---- interior: every element exists, every access is a full vector ----
        float x[kRowsPerWave][kEPL];
#pragma unroll
        for (int r = 0; r < kRowsPerWave; ++r)
            Loader<InT>::full(it.x, wave_base + r * kRow + lane * kEPL, x[r]);
#pragma unroll
        for (int r = 0; r < kRowsPerWave; ++r) {
            const int64_t i0 = wave_base + r * kRow + lane * kEPL;
            float mn = vmin3(x[r][0], x[r][1], x[r][2]), mx = vmax3(x[r][0], x[r][1], x[r][2]);
            mn = vmin3(mn, x[r][3], x[r][4]);  mx = vmax3(mx, x[r][3], x[r][4]);
            mn = vmin3(mn, x[r][5], x[r][6]);  mx = vmax3(mx, x[r][5], x[r][6]);
            mn = vmin(mn, x[r][7]);            mx = vmax(mx, x[r][7]);
            group_minmax<LPG>(mn, mx);
            float scale, zero, inv;
            {
                constexpr float Lf = (float)((1 << B) - 1);
                const float range = mx - mn;
                const bool degenerate = range < 0x1p-100f;
                zero = mn + 0.0f;                             // -0.0 -> +0.0
                scale = degenerate ? 0.0f : range / Lf;       // IEEE-correct divisions
                inv = degenerate ? 0.0f : Lf / range;
            }
            if ((lane & (LPG - 1)) == 0)
                *reinterpret_cast<f32x2*>(it.meta + 2 * (i0 >> Log2<G>::v)) = f32x2{scale, zero};
            uint32_t w0, w1;
            quantise8<B, STOCH>(x[r], mn, inv, kEPL, i0, it.seed, it.tensor_id, w0, w1);
            store_codes<B>(it.packed + (uint64_t)i0 * B / 8, w0, w1);
        }
        return;
    }

    // ---- edge: the tensor ends inside this wave's span.  All 64 lanes stay active
    //      through the reductions; missing elements enter them as +inf / -inf. ----
    for (int r = 0; r < kRowsPerWave; ++r) {
        const int64_t row_base = wave_base + r * kRow;
        if (row_base >= extent) break;                        // wave-uniform
        const int64_t i0 = row_base + lane * kEPL;
        const int64_t left = numel - i0;
        const int valid = left >= kEPL ? kEPL : (left > 0 ? (int)left : 0);
        float x[kEPL];
        float mn = 0.0f, mx = 0.0f;
#pragma unroll
        for (int j = 0; j < kEPL; ++j) {
            const bool ok = j < valid;
            x[j] = ok ? Loader<InT>::one(it.x, i0 + j) : 0.0f;
            const float lo = ok ? x[j] : __builtin_inff();
            const float hi = ok ? x[j] : -__builtin_inff();
            mn = j == 0 ? lo : vmin(mn, lo);
            mx = j == 0 ? hi : vmax(mx, hi);
        }
        group_minmax<LPG>(mn, mx);
        if (mn > mx) { mn = 0.0f; mx = 0.0f; }                // a run with no element at all
        constexpr float Lf = (float)((1 << B) - 1);
        const float range = mx - mn;
        const bool degenerate = range < 0x1p-100f;
        const float zero = mn + 0.0f;
        const float scale = degenerate ? 0.0f : range / Lf;
        const float inv = degenerate ? 0.0f : Lf / range;
        // a group exists iff its first element does
        if ((lane & (LPG - 1)) == 0 && i0 < numel)
            *reinterpret_cast<f32x2*>(it.meta + 2 * (i0 >> Log2<G>::v)) = f32x2{scale, zero};
        uint32_t w0, w1;
        quantise8<B, STOCH>(x, mn, inv, valid, i0, it.seed, it.tensor_id, w0, w1);
        // chunks are size-aligned and the padded length is a multiple of 16, so a chunk is
        // either wholly inside the buffer or wholly outside
        const uint64_t off = (uint64_t)i0 * B / 8;
        if (off < it.packed_padded) store_codes<B>(it.packed + off, w0, w1);
    }
}

template <typename InT, int G>
__global__ __launch_bounds__(kBlock) void compress_kernel(const CompressBatch args)
{
    const uint32_t bid = blockIdx.x;
    int lo = 0, hi = args.count;                              // last item with tile_start <= bid
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (args.tile_start[mid] <= bid) lo = mid; else hi = mid;
    }
    const CompressItem& it = args.item[lo];
    const uint32_t tile = bid - args.tile_start[lo];
    switch (it.bits * 2 + it.stochastic) {
        case 4:  compress_tile<InT, G, 2, false>(it, tile); break;
        case 5:  compress_tile<InT, G, 2, true >(it, tile); break;
        case 8:  compress_tile<InT, G, 4, false>(it, tile); break;
        case 9:  compress_tile<InT, G, 4, true >(it, tile); break;
        case 16: compress_tile<InT, G, 8, false>(it, tile); break;
        case 17: compress_tile<InT, G, 8, true >(it, tile); break;
        default: break;
    }
}

}  // namespace

int compress_tile_elems(int, int) { return kTile; }

hipError_t launch_compress(const CompressBatch& b, int dtype, int group_size, hipStream_t s)
{
    const uint32_t tiles = b.tile_start[b.count];
    if (tiles == 0) return hipSuccess;
    const dim3 grid(tiles), block(kBlock);
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
