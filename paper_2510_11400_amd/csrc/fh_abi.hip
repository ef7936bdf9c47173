// C ABI of the activation compressor: host-side argument checks, size helpers and
// the grouping of tensors into launches.  Declarations and the full contract are in
// include/fedhybrid.h.
#include "../../include/fedhybrid.h"

#include "fh_kernels.hpp"

#include <limits.h>

namespace {

using namespace fh;

bool aligned(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

size_t elem_size(int dtype) { return dtype == FH_F32 ? 4u : 2u; }

fh_status check_params(const fh_params* p, bool need_round)
{
    if (!p) return FH_ERR_NULL;
    if (p->group_size != 64 && p->group_size != 128 && p->group_size != 256) return FH_ERR_BAD_GROUP;
    if (p->bits != 2 && p->bits != 4 && p->bits != 8) return FH_ERR_BAD_BITS;
    if (need_round && p->rounding != FH_ROUND_NEAREST && p->rounding != FH_ROUND_STOCHASTIC)
        return FH_ERR_BAD_ROUND;
    if (p->reserved != 0) return FH_ERR_BAD_PARAM;
    return FH_OK;
}

fh_status check_dtype(int d) { return (d == FH_F32 || d == FH_BF16) ? FH_OK : FH_ERR_BAD_DTYPE; }

// numel must be indexable: tile counts are 32-bit and byte offsets 64-bit.
fh_status check_numel(int64_t numel)
{
    if (numel < 0 || numel > (int64_t)1 << 40) return FH_ERR_BAD_NUMEL;
    return FH_OK;
}

fh_status check_compress_item(const fh_item& it)
{
    fh_status s;
    if ((s = check_params(&it.params, true)) != FH_OK) return s;
    if ((s = check_dtype(it.x_dtype)) != FH_OK) return s;
    if ((s = check_numel(it.numel)) != FH_OK) return s;
    if (it.numel == 0) return FH_OK;
    if (!it.x || !it.packed || !it.meta) return FH_ERR_NULL;
    if (!aligned(it.x, 16) || !aligned(it.packed, 16) || !aligned(it.meta, 8)) return FH_ERR_ALIGNMENT;
    if (it.packed_cap < fh_packed_bytes(it.numel, it.params.bits)) return FH_ERR_BUFFER_TOO_SMALL;
    if (it.meta_cap < fh_meta_bytes(it.numel, it.params.group_size)) return FH_ERR_BUFFER_TOO_SMALL;
    return FH_OK;
}

fh_status check_decompress_item(const fh_item& it)
{
    fh_status s;
    if ((s = check_params(&it.params, false)) != FH_OK) return s;
    if ((s = check_dtype(it.out_dtype)) != FH_OK) return s;
    if ((s = check_numel(it.numel)) != FH_OK) return s;
    if (it.numel == 0) return FH_OK;
    if (!it.packed || !it.meta || !it.out) return FH_ERR_NULL;
    if (!aligned(it.packed, 16) || !aligned(it.out, 16) || !aligned(it.meta, 8)) return FH_ERR_ALIGNMENT;
    if (it.packed_cap < fh_packed_bytes(it.numel, it.params.bits)) return FH_ERR_BUFFER_TOO_SMALL;
    if (it.meta_cap < fh_meta_bytes(it.numel, it.params.group_size)) return FH_ERR_BUFFER_TOO_SMALL;
    if (it.out_cap < (size_t)it.numel * elem_size(it.out_dtype)) return FH_ERR_BUFFER_TOO_SMALL;
    return FH_OK;
}

uint32_t tiles_for(int64_t elems, int tile) { return (uint32_t)((elems + tile - 1) / tile); }

// Launch runs of consecutive items that share (dtype, group size), at most kMaxItems
// per launch and fewer than 2^31 tiles per launch.
fh_status run_compress(const fh_item* items, int32_t count, hipStream_t stream)
{
    int32_t i = 0;
    while (i < count) {
        while (i < count && items[i].numel == 0) ++i;
        if (i >= count) break;
        const int dtype = items[i].x_dtype, G = items[i].params.group_size;
        const int tile = compress_tile_elems(dtype, G);
        CompressBatch b;
        b.count = 0;
        b.tile_start[0] = 0;
        while (i < count && b.count < kMaxItems) {
            const fh_item& it = items[i];
            if (it.numel == 0) { ++i; continue; }
            if (it.x_dtype != dtype || it.params.group_size != G) break;
            const uint32_t t = tiles_for(it.numel, tile);
            if ((uint64_t)b.tile_start[b.count] + t > (uint64_t)INT_MAX) {
                if (b.count == 0) return FH_ERR_BAD_NUMEL;
                break;
            }
            CompressItem& d = b.item[b.count];
            d.x = it.x;
            d.packed = static_cast<uint8_t*>(it.packed);
            d.meta = static_cast<float*>(it.meta);
            d.numel = it.numel;
            d.packed_padded = fh_packed_bytes(it.numel, it.params.bits);
            d.seed = it.params.seed;
            d.tensor_id = it.params.tensor_id;
            d.bits = it.params.bits;
            d.stochastic = it.params.rounding == FH_ROUND_STOCHASTIC ? 1 : 0;
            b.tile_start[b.count + 1] = b.tile_start[b.count] + t;
            ++b.count;
            ++i;
        }
        for (int k = b.count + 1; k <= kMaxItems; ++k) b.tile_start[k] = b.tile_start[b.count];
        if (launch_compress(b, dtype, G, stream) != hipSuccess) return FH_ERR_LAUNCH;
    }
    return FH_OK;
}

fh_status run_decompress(const fh_item* items, int32_t count, hipStream_t stream)
{
    int32_t i = 0;
    while (i < count) {
        while (i < count && items[i].numel == 0) ++i;
        if (i >= count) break;
        const int dtype = items[i].out_dtype, G = items[i].params.group_size;
        const int tile = decompress_tile_elems(dtype, G);
        DecompressBatch b;
        b.count = 0;
        b.tile_start[0] = 0;
        while (i < count && b.count < kMaxItems) {
            const fh_item& it = items[i];
            if (it.numel == 0) { ++i; continue; }
            if (it.out_dtype != dtype || it.params.group_size != G) break;
            const uint32_t t = tiles_for(it.numel, tile);
            if ((uint64_t)b.tile_start[b.count] + t > (uint64_t)INT_MAX) {
                if (b.count == 0) return FH_ERR_BAD_NUMEL;
                break;
            }
            DecompressItem& d = b.item[b.count];
            d.packed = static_cast<const uint8_t*>(it.packed);
            d.meta = static_cast<const float*>(it.meta);
            d.out = it.out;
            d.numel = it.numel;
            d.bits = it.params.bits;
            d.pad = 0;
            b.tile_start[b.count + 1] = b.tile_start[b.count] + t;
            ++b.count;
            ++i;
        }
        for (int k = b.count + 1; k <= kMaxItems; ++k) b.tile_start[k] = b.tile_start[b.count];
        if (launch_decompress(b, dtype, G, stream) != hipSuccess) return FH_ERR_LAUNCH;
    }
    return FH_OK;
}

template <typename Check>
fh_status check_all(const fh_item* items, int32_t count, Check check)
{
    if (count < 0) return FH_ERR_BAD_COUNT;
    if (count > 0 && !items) return FH_ERR_NULL;
    for (int32_t i = 0; i < count; ++i) {
        const fh_status s = check(items[i]);
        if (s != FH_OK) return s;
    }
    return FH_OK;
}

}  // namespace

extern "C" {

size_t fh_packed_bytes(int64_t numel, int32_t bits)
{
    if (numel <= 0 || (bits != 2 && bits != 4 && bits != 8)) return 0;
    const uint64_t raw = ((uint64_t)numel * (uint64_t)bits + 7u) >> 3;
    return (size_t)((raw + 15u) & ~(uint64_t)15u);
}

size_t fh_meta_bytes(int64_t numel, int32_t group_size)
{
    if (numel <= 0 || group_size <= 0) return 0;
    return (size_t)(8u * (((uint64_t)numel + (uint64_t)group_size - 1u) / (uint64_t)group_size));
}

int32_t fh_batch_capacity(void) { return kMaxItems; }

fh_status fh_compress_batch(const fh_item* items, int32_t count, void* stream)
{
    const fh_status s = check_all(items, count, check_compress_item);
    if (s != FH_OK) return s;
    return run_compress(items, count, static_cast<hipStream_t>(stream));
}

fh_status fh_decompress_batch(const fh_item* items, int32_t count, void* stream)
{
    const fh_status s = check_all(items, count, check_decompress_item);
    if (s != FH_OK) return s;
    return run_decompress(items, count, static_cast<hipStream_t>(stream));
}

fh_status fh_roundtrip_batch(const fh_item* items, int32_t count, void* stream)
{
    fh_status s = check_all(items, count, check_compress_item);
    if (s != FH_OK) return s;
    s = check_all(items, count, check_decompress_item);
    if (s != FH_OK) return s;
    s = run_compress(items, count, static_cast<hipStream_t>(stream));
    if (s != FH_OK) return s;
    return run_decompress(items, count, static_cast<hipStream_t>(stream));
}

fh_status fh_compress(const void* x, fh_dtype x_dtype, int64_t numel, const fh_params* params,
                      void* packed, size_t packed_cap, void* meta, size_t meta_cap, void* stream)
{
    if (!params) return FH_ERR_NULL;
    fh_item it = {};
    it.x = x; it.x_dtype = x_dtype; it.out_dtype = FH_F32; it.numel = numel;
    it.packed = packed; it.packed_cap = packed_cap; it.meta = meta; it.meta_cap = meta_cap;
    it.params = *params;
    return fh_compress_batch(&it, 1, stream);
}

fh_status fh_decompress(const void* packed, const void* meta, int64_t numel, const fh_params* params,
                        fh_dtype out_dtype, void* out, size_t out_cap, void* stream)
{
    if (!params) return FH_ERR_NULL;
    fh_item it = {};
    it.x_dtype = FH_F32; it.out_dtype = out_dtype; it.numel = numel;
    it.packed = const_cast<void*>(packed); it.packed_cap = fh_packed_bytes(numel, params->bits);
    it.meta = const_cast<void*>(meta); it.meta_cap = fh_meta_bytes(numel, params->group_size);
    it.out = out; it.out_cap = out_cap;
    it.params = *params;
    return fh_decompress_batch(&it, 1, stream);
}

fh_status fh_roundtrip(const void* x, fh_dtype x_dtype, int64_t numel, const fh_params* params,
                       void* packed, size_t packed_cap, void* meta, size_t meta_cap,
                       fh_dtype out_dtype, void* out, size_t out_cap, void* stream)
{
    if (!params) return FH_ERR_NULL;
    fh_item it = {};
    it.x = x; it.x_dtype = x_dtype; it.out_dtype = out_dtype; it.numel = numel;
    it.packed = packed; it.packed_cap = packed_cap; it.meta = meta; it.meta_cap = meta_cap;
    it.out = out; it.out_cap = out_cap;
    it.params = *params;
    return fh_roundtrip_batch(&it, 1, stream);
}

const char* fh_status_string(fh_status s)
{
    switch (s) {
        case FH_OK: return "ok";
        case FH_ERR_NULL: return "a required pointer is NULL";
        case FH_ERR_BAD_DTYPE: return "unsupported dtype (expected FH_F32 or FH_BF16)";
        case FH_ERR_BAD_GROUP: return "group_size must be 64, 128 or 256";
        case FH_ERR_BAD_BITS: return "bits must be 2, 4 or 8";
        case FH_ERR_BAD_ROUND: return "rounding must be FH_ROUND_NEAREST or FH_ROUND_STOCHASTIC";
        case FH_ERR_BAD_NUMEL: return "numel is negative or too large";
        case FH_ERR_BUFFER_TOO_SMALL: return "an output or input buffer capacity is too small";
        case FH_ERR_ALIGNMENT: return "x, packed and out must be 16-byte aligned, meta 8-byte aligned";
        case FH_ERR_LAUNCH: return "the HIP runtime refused the kernel launch";
        case FH_ERR_BAD_COUNT: return "item count is negative";
        case FH_ERR_BAD_SHAPE: return "outer / maps must be >= 0, inner / h / w >= 1, channels in 1..16384, raw_channels in 0..channels";
        case FH_ERR_BAD_PARAM: return "k_sigma must be positive, min_outliers at least 1, the pooling window 2, 4 or 8, every reserved field 0";
        case FH_ERR_SCRATCH_LIMIT: return "the tensor needs more scratch than the library's static buffer holds";
    }
    return "unknown status";
}

}  // extern "C"
