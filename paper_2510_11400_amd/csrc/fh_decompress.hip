// Backward side of the group quantiser on gfx950: unpack + fused dequantise.
//
// The output side carries almost all the bytes, so the lane layout is chosen for it:
// each lane produces exactly one 128-bit store (4 fp32 or 8 bf16 consecutive
// elements) and a wave's store is one contiguous span.  The codes a lane needs are
// 8..64 bits of the packed stream; lanes read the aligned 32-bit word that holds
// them (neighbouring lanes share a word when bits < 8, which the memory pipeline
// serves as one access) and shift their part out.  scale/zero come from an 8-byte
// load that all lanes of a group share.
//
// Reconstruction follows the paper's Section 4.4.1 (floating-point values are rebuilt
// from the quantisation codes): x^ = fma(code, scale, zero), one rounding.
//
// The MIXED variants take the elements of kept (salient) channels from the raw store
// instead.
#include <type_traits>

#include "fh_channels.hpp"
#include "fh_device.hpp"
#include "fh_kernels.hpp"

namespace fh {

namespace {

constexpr int kDBlock = 256;                       // threads per workgroup

// EPL: elements per lane and row (one 128-bit store).  ROWS: rows of a wave, whose loads are all
// issued before the first store -- measured with the codes coming from HBM: 2 rows (2 KiB out per
// wave) for fp32 output (1 row costs 30 %, 4 rows 7 %), 4 rows (4 KiB) for bf16 output (2 rows cost 9 %).
template <typename OutT> struct OutTraits;
template <> struct OutTraits<float>    { static constexpr int EPL = 4; static constexpr int ROWS = 2; };
template <> struct OutTraits<uint16_t> { static constexpr int EPL = 8; static constexpr int ROWS = 4; };

template <typename OutT> constexpr int tile_elems()
{
    return (kDBlock / kWave) * OutTraits<OutT>::ROWS * kWave * OutTraits<OutT>::EPL;
}

template <int G> struct Log2;
template <> struct Log2<64>  { static constexpr int v = 6; };
template <> struct Log2<128> { static constexpr int v = 7; };
template <> struct Log2<256> { static constexpr int v = 8; };

// The EPL*B code bits of the lane whose first element is i0, right-aligned in c0 (and
// c1 for the 64-bit case).
template <int EPL, int B>
__device__ __forceinline__ void load_codes(const uint8_t* packed, int64_t i0, uint32_t& c0, uint32_t& c1)
{
    constexpr int NBITS = EPL * B;
    const uint64_t off = (uint64_t)i0 * B / 8;                // byte offset, multiple of NBITS/8
    c1 = 0u;
    if constexpr (NBITS == 64) {
        const u32x2 w = code_load(reinterpret_cast<const u32x2*>(packed + off));
        c0 = w.x; c1 = w.y;
    } else if constexpr (NBITS == 32) {
        c0 = code_load(reinterpret_cast<const uint32_t*>(packed + off));
    } else {                                                  // 16 or 8 bits inside an aligned word
        const uint32_t w = code_load(reinterpret_cast<const uint32_t*>(packed + (off & ~(uint64_t)3)));
        c0 = (w >> (((uint32_t)off & 3u) * 8u)) & ((1u << NBITS) - 1u);
    }
}

template <int B>
__device__ __forceinline__ float dequant(uint32_t bitsword, int j, float scale, float zero)
{
    const uint32_t code = (bitsword >> (j * B)) & ((1u << B) - 1u);
    return __builtin_fmaf((float)code, scale, zero);          // single rounding
}

// Restore the EPL elements of one lane from its code bits and its group's meta.
template <int EPL, int B>
__device__ __forceinline__ void restore(uint32_t c0, uint32_t c1, f32x2 m, float (&v)[EPL])
{
    constexpr int PER_WORD = 32 / B;                          // codes per 32-bit word
#pragma unroll
    for (int j = 0; j < EPL; ++j)
        v[j] = dequant<B>((j < PER_WORD) ? c0 : c1, j % PER_WORD, m.x, m.y);
}

__device__ __forceinline__ u32x4 pack_bf16x8(const float (&v)[8])
{
    u32x4 o;
    o.x = bf16_bits(v[0]) | (bf16_bits(v[1]) << 16);
    o.y = bf16_bits(v[2]) | (bf16_bits(v[3]) << 16);
    o.z = bf16_bits(v[4]) | (bf16_bits(v[5]) << 16);
    o.w = bf16_bits(v[6]) | (bf16_bits(v[7]) << 16);
    return o;
}

// ---- kept channels (MIXED) ---------------------------------------------------------------
// Replace the kept elements of a lane's run by their raw values (widened to fp32 when the raw
// store is bf16; rounding to a bf16 output happens with the rest of the lane's elements).
template <int N>
__device__ __forceinline__ void fetch_kept(const ChannelMap& cm, int raw_dtype, const KeptRun<N>& run, float (&v)[N])
{
#pragma unroll
    for (int j = 0; j < N; ++j) {
        if (run.mask & (1u << j)) {
            const uint64_t i = raw_index<N>(cm, run, j);
            const uint32_t bits = raw_dtype == 0 ? static_cast<const uint32_t*>(cm.raw)[i]
                                                 : (uint32_t) static_cast<const uint16_t*>(cm.raw)[i] << 16;
            v[j] = __builtin_bit_cast(float, bits);
        }
    }
}

// The same in two steps: the loads alone (the raw values as fp32 bit patterns) ...
template <int N>
__device__ __forceinline__ void request_kept(const ChannelMap& cm, int raw_dtype, const KeptRun<N>& run, uint32_t (&bits)[N])
{
    if (raw_dtype == 0) {
#pragma unroll
        for (int j = 0; j < N; ++j)
            if (run.mask & (1u << j)) bits[j] = static_cast<const uint32_t*>(cm.raw)[raw_index<N>(cm, run, j)];
    } else {
#pragma unroll
        for (int j = 0; j < N; ++j)
            if (run.mask & (1u << j)) bits[j] = (uint32_t) static_cast<const uint16_t*>(cm.raw)[raw_index<N>(cm, run, j)] << 16;
    }
}

// One channel per element (fh_channels.hpp): the wave's restored span is parked in LDS in the output's
// dtype, the lanes walk the span's (sample, row) pairs and overwrite the kept elements with the
// raw store's values -- consecutive lanes, consecutive rows --, then every lane takes its 16 bytes
// per row back and stores them.  A lane's first raw-store entries are requested together with the
// codes, before the list of rows exists, so that their latency overlaps that of the codes.  (The alternative measured: every lane
// loading a raw entry for each of its elements and merging by masks.)
typedef uint16_t __attribute__((may_alias)) park_u16;
typedef uint32_t __attribute__((may_alias)) park_u32;
typedef u32x4 __attribute__((may_alias)) park_u32x4;

template <typename OutT>
__device__ __forceinline__ OutT raw_as(const void* raw, uint64_t i, int raw_dtype)
{
    if constexpr (sizeof(OutT) == 4) {
        return raw_dtype == 0 ? static_cast<const uint32_t*>(raw)[i] : (uint32_t) static_cast<const uint16_t*>(raw)[i] << 16;
    } else {
        return raw_dtype == 0 ? (OutT)bf16_bits(static_cast<const float*>(raw)[i]) : static_cast<const uint16_t*>(raw)[i];
    }
}

template <typename OutT, int G, int B, bool MIXED = false>
__device__ __forceinline__ void decompress_tile(const DecompressItem& it, uint32_t tile,
                                                const ChannelMap* cm = nullptr, int raw_dtype = 0,
                                                uint16_t* listed = nullptr, uint8_t* park = nullptr)
{
    constexpr int EPL = OutTraits<OutT>::EPL;
    constexpr int kRowsPerWave = OutTraits<OutT>::ROWS;
    constexpr int ROW = kWave * EPL;
    constexpr int WAVE_SPAN = kRowsPerWave * ROW;
    constexpr int TILE = (kDBlock / kWave) * WAVE_SPAN;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t numel = it.numel;
    const int64_t wave_base = (int64_t)tile * TILE + (int64_t)wave * WAVE_SPAN;
    const bool interior = wave_base + WAVE_SPAN <= numel;
    uint32_t c0[kRowsPerWave] = {}, c1[kRowsPerWave] = {};
    f32x2 m[kRowsPerWave] = {};
    const auto load_span = [&]() {                            // interior spans: all loads first
#pragma unroll
        for (int r = 0; r < kRowsPerWave; ++r) {
            const int64_t i0 = wave_base + r * ROW + lane * EPL;
            load_codes<EPL, B>(it.packed, i0, c0[r], c1[r]);
            m[r] = code_load(reinterpret_cast<const f32x2*>(it.meta + 2 * (i0 >> Log2<G>::v)));
        }
    };
    const uint16_t* rows = nullptr;
    using RawBits = typename std::conditional<sizeof(OutT) == 4, uint32_t, uint16_t>::type;
    RawBits ahead[kPairsAhead] = {};                          // MIXED: a lane's first raw-store entries, in the output's dtype
    if constexpr (MIXED) {
        if (rows_listed(*cm)) {                               // the same for every thread of the workgroup, which all get here
            // the table entries first, then the span's codes (so that waiting for the former does not wait for the
            // latter), and the list is filed while the codes are on their way
            SlotWords words;
            list_rows_request<kDBlock>(*cm, words);
            if (interior) {
                load_span();
                // ... and the raw store's entries of the span's samples, all rows of them: which of them are kept
                // elements of this span is known only once the list is there, but where they lie is not a
                // question -- consecutive lanes, consecutive entries -- so they are on their way together with the codes
                const ElemPos at = locate_base(*cm, (uint32_t)wave_base);
                const uint64_t raw0 = (uint64_t)at.o * cm->raw_channels;
                const uint32_t pairs = span_pairs(*cm, at, WAVE_SPAN);
#pragma unroll
                for (int k = 0; k < kPairsAhead; ++k) {
                    const uint32_t i = k * kWave + lane;
                    ahead[k] = i < pairs ? raw_as<RawBits>(cm->raw, raw0 + i, raw_dtype) : (RawBits)0;
                }
                // (the filing is written out on both paths: behind their join the compiler could not tell how many
                // loads are outstanding and would wait for the codes before the table entries may be used)
                list_rows_file<kDBlock>(*cm, words, listed);
            } else {
                list_rows_file<kDBlock>(*cm, words, listed);
            }
            rows = listed;
        }
    }
    if (wave_base >= numel) return;
    ElemPos wave_pos = {0u, 0u, 0u};
    if constexpr (MIXED) wave_pos = locate_base(*cm, (uint32_t)wave_base);

    if (interior) {
        // ---- interior: all loads first, then one 128-bit store per lane and row ----
        if (!(MIXED && rows != nullptr)) load_span();
        if constexpr (MIXED) {
            if (rows != nullptr) {                            // wave-uniform: one channel per element
                using Bits = typename std::conditional<sizeof(OutT) == 4, uint32_t, uint16_t>::type;
                typedef Bits __attribute__((may_alias)) Parked;
                const uint64_t raw0 = (uint64_t)wave_pos.o * cm->raw_channels;
                const uint32_t pairs = span_pairs(*cm, wave_pos, WAVE_SPAN);
                PairWalk walk = pair_walk(*cm, wave_pos, lane);
                uint32_t off[kPairsAhead];
                first_pairs(*cm, walk, rows, pairs, off);
                park_u32x4* mine = reinterpret_cast<park_u32x4*>(park + wave * (WAVE_SPAN * sizeof(OutT)));
#pragma unroll
                for (int r = 0; r < kRowsPerWave; ++r) {
                    float v[EPL];
                    restore<EPL, B>(c0[r], c1[r], m[r], v);
                    if constexpr (EPL == 4) {
                        mine[r * kWave + lane] = u32x4{__builtin_bit_cast(uint32_t, v[0]), __builtin_bit_cast(uint32_t, v[1]),
                                                       __builtin_bit_cast(uint32_t, v[2]), __builtin_bit_cast(uint32_t, v[3])};
                    } else {
                        mine[r * kWave + lane] = pack_bf16x8(v);
                    }
                }
                __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");   // LDS operations of one wave complete in order
                Parked* elems = reinterpret_cast<Parked*>(mine);
#pragma unroll
                for (int k = 0; k < kPairsAhead; ++k)
                    if (off[k] < (uint32_t)WAVE_SPAN) elems[off[k]] = ahead[k];
                for (uint32_t i = kPairsAhead * kWave; i < pairs; i += kWave) {            // wave-uniform trip count
                    const uint32_t o = pair_offset(walk, rows);
                    pair_advance(*cm, walk);
                    if (o < (uint32_t)WAVE_SPAN) elems[o] = raw_as<Bits>(cm->raw, raw0 + i + lane, raw_dtype);
                }
                __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
#pragma unroll
                for (int r = 0; r < kRowsPerWave; ++r) {
                    const int64_t i0 = wave_base + r * ROW + lane * EPL;
                    const u32x4 o = mine[r * kWave + lane];
                    stream_store(reinterpret_cast<u32x4*>(static_cast<OutT*>(it.out) + i0), o);
                }
                return;
            }
        }
        KeptRun<EPL> run[kRowsPerWave];
        uint32_t kept[kRowsPerWave][EPL] = {};                // MIXED: the raw store's bits of the lane's kept elements
        if constexpr (MIXED) {
            // which elements are kept does not depend on the codes: their raw values are requested now, with the codes
            // on their way, and not row by row after the codes have come (a wave with a kept run paid a second memory
            // latency per row)
            kept_runs<kRowsPerWave, EPL>(*cm, wave_pos, lane * EPL, ROW, run);
#pragma unroll
            for (int r = 0; r < kRowsPerWave; ++r)
                if (run[r].mask) request_kept<EPL>(*cm, raw_dtype, run[r], kept[r]);
        }
#pragma unroll
        for (int r = 0; r < kRowsPerWave; ++r) {
            const int64_t i0 = wave_base + r * ROW + lane * EPL;
            float v[EPL];
            restore<EPL, B>(c0[r], c1[r], m[r], v);
            if constexpr (MIXED) {
#pragma unroll
                for (int j = 0; j < EPL; ++j)
                    if (run[r].mask & (1u << j)) v[j] = __builtin_bit_cast(float, kept[r][j]);
            }
            if constexpr (EPL == 4) {
                stream_store(reinterpret_cast<f32x4*>(static_cast<float*>(it.out) + i0), f32x4{v[0], v[1], v[2], v[3]});
            } else {
                stream_store(reinterpret_cast<u32x4*>(static_cast<uint16_t*>(it.out) + i0), pack_bf16x8(v));
            }
        }
        return;
    }

    // ---- edge: the tensor ends inside this wave's span ----
    for (int r = 0; r < kRowsPerWave; ++r) {
        const int64_t i0 = wave_base + r * ROW + lane * EPL;
        if (i0 >= numel) continue;
        // a lane whose first element exists reads inside the padded code stream and inside
        // the meta array (its group exists)
        uint32_t c0, c1;
        load_codes<EPL, B>(it.packed, i0, c0, c1);
        const f32x2 m = *reinterpret_cast<const f32x2*>(it.meta + 2 * (i0 >> Log2<G>::v));
        float v[EPL];
        restore<EPL, B>(c0, c1, m, v);
        if constexpr (MIXED) {
            const int64_t left = numel - i0;
            const uint32_t valid = left >= EPL ? (1u << EPL) - 1u : (1u << (int)left) - 1u;
            KeptRun<EPL> run[1];
            kept_runs<1, EPL>(*cm, wave_pos, r * ROW + lane * EPL, 0, run);
            run[0].mask &= valid;
            if (run[0].mask) fetch_kept<EPL>(*cm, raw_dtype, run[0], v);
        }
        if constexpr (EPL == 4) {
            float* dst = static_cast<float*>(it.out) + i0;
            if (i0 + EPL <= numel) {
                *reinterpret_cast<f32x4*>(dst) = f32x4{v[0], v[1], v[2], v[3]};
            } else {
#pragma unroll
                for (int j = 0; j < EPL; ++j) if (i0 + j < numel) dst[j] = v[j];
            }
        } else {
            uint16_t* dst = static_cast<uint16_t*>(it.out) + i0;
            if (i0 + EPL <= numel) {
                *reinterpret_cast<u32x4*>(dst) = pack_bf16x8(v);
            } else {
#pragma unroll
                for (int j = 0; j < EPL; ++j) if (i0 + j < numel) dst[j] = (uint16_t)bf16_bits(v[j]);
            }
        }
    }
}

template <typename OutT, int G>
__global__ __launch_bounds__(kDBlock) void decompress_kernel(const DecompressBatch args)
{
    // Tiles are taken from the end of the set backwards: the backward pass needs the
    // tensors in the reverse of the order the forward pass saved them, and the codes
    // written last are the ones most likely still held by the memory-side cache.
    const uint32_t bid = gridDim.x - 1u - blockIdx.x;
    const int lo = find_item(args.tile_start, bid);
    const DecompressItem it = args.item[lo];                  // by value: one batch of scalar loads
    const uint32_t tile = bid - args.tile_start[lo];
    switch (it.bits) {
        case 2: decompress_tile<OutT, G, 2>(it, tile); break;
        case 4: decompress_tile<OutT, G, 4>(it, tile); break;
        case 8: decompress_tile<OutT, G, 8>(it, tile); break;
        default: break;
    }
}

// Tensors whose kept channels come from the raw store.
template <typename OutT, int G>
__global__ __launch_bounds__(kDBlock) void decompress_mixed_kernel(const Batch<MixedDecompressJob> batch)
{
    uint32_t tile;
    const MixedDecompressJob& job = batch.item[batch_item(batch, gridDim.x - 1u - blockIdx.x, tile)];
    const DecompressItem& it = job.it;
    const ChannelMap& cm = job.cm;
    const int raw_dtype = job.raw_dtype;
    __shared__ __attribute__((aligned(16))) uint8_t park[tile_elems<OutT>() * sizeof(OutT)];
    __shared__ uint16_t listed[kListedRows];
    if (nothing_kept(cm)) {                                   // no channel of this tensor was kept: the plain code
        switch (it.bits) {
            case 2: decompress_tile<OutT, G, 2>(it, tile); break;
            case 4: decompress_tile<OutT, G, 4>(it, tile); break;
            case 8: decompress_tile<OutT, G, 8>(it, tile); break;
            default: break;
        }
        return;
    }
    switch (it.bits) {
        case 2: decompress_tile<OutT, G, 2, true>(it, tile, &cm, raw_dtype, listed, park); break;
        case 4: decompress_tile<OutT, G, 4, true>(it, tile, &cm, raw_dtype, listed, park); break;
        case 8: decompress_tile<OutT, G, 8, true>(it, tile, &cm, raw_dtype, listed, park); break;
        default: break;
    }
}

}  // namespace

int decompress_tile_elems(int out_dtype, int)
{
    return out_dtype == 0 ? tile_elems<float>() : tile_elems<uint16_t>();
}

hipError_t launch_decompress(const DecompressBatch& b, int out_dtype, int group_size, hipStream_t s)
{
    const uint32_t tiles = b.tile_start[b.count];
    if (tiles == 0) return hipSuccess;
    const dim3 grid(tiles), block(kDBlock);
#define FH_LAUNCH(T, GS) hipLaunchKernelGGL((decompress_kernel<T, GS>), grid, block, 0, s, b)
    if (out_dtype == 0) {
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

hipError_t launch_decompress_mixed(const Batch<MixedDecompressJob>& b, int out_dtype, int group_size, hipStream_t s)
{
    const uint32_t tiles = b.block_start[b.count];
    if (tiles == 0) return hipSuccess;
    const dim3 grid(tiles), block(kDBlock);
#define FH_LAUNCH(T, GS) hipLaunchKernelGGL((decompress_mixed_kernel<T, GS>), grid, block, 0, s, b)
    if (out_dtype == 0) {
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
