// Routing salient channels around the quantiser (paper Section 4.4.1, Channel-wise Mix
// Compression: only normal channels are quantised): the slot table that says which
// channels are kept verbatim, and the C entry points of the mixed forward / backward
// calls.  The kernels themselves are the MIXED variants in fh_compress.hip and
// fh_decompress.hip.
#include "../../include/fedhybrid.h"

#include "fh_channels.hpp"
#include "fh_kernels.hpp"

namespace fh {
namespace {

constexpr int kSlotThreads = 1024;
constexpr int kSlotPerThread = 16;                 // 1024 * 16 = the largest channel count

// slots[c] = number of salient channels before c, for salient channels while that number is
// below raw_channels; -1 for every other channel.  One workgroup: each thread owns 16
// consecutive channels, the per-thread counts are scanned through LDS.
__device__ __forceinline__ void number_slots(const uint8_t* __restrict__ mask, int channels, int raw_channels,
                                             int16_t* __restrict__ slots, uint64_t* __restrict__ used)
{
    __shared__ int scan[kSlotThreads];
    const int t = threadIdx.x;
    const int first = t * kSlotPerThread;
    int mine = 0;
    for (int k = 0; k < kSlotPerThread; ++k) {
        const int c = first + k;
        if (c < channels && mask[c] != 0) ++mine;
    }
    scan[t] = mine;
    __syncthreads();
    for (int step = 1; step < kSlotThreads; step <<= 1) {     // inclusive scan, all threads reach every barrier
        const int add = t >= step ? scan[t - step] : 0;
        __syncthreads();
        scan[t] += add;
        __syncthreads();
    }
    int rank = scan[t] - mine;                                // salient channels before this thread's first
    for (int k = 0; k < kSlotPerThread; ++k) {
        const int c = first + k;
        if (c >= channels) break;
        if (mask[c] != 0 && rank < raw_channels) slots[c] = (int16_t)rank;
        else slots[c] = (int16_t)-1;
        if (mask[c] != 0) ++rank;
    }
    if (used && t == kSlotThreads - 1) *used = (uint64_t)(scan[t] < raw_channels ? scan[t] : raw_channels);
}

struct SlotsJob {
    const uint8_t* mask;
    int16_t*       slots;
    uint64_t*      used;
    int32_t        channels, raw_channels;
};
struct SlotsBatch { SlotsJob job[kBatch]; };

// one workgroup per tensor
__global__ __launch_bounds__(kSlotThreads) void channel_slots_kernel(const SlotsBatch batch)
{
    const SlotsJob& j = batch.job[blockIdx.x];
    number_slots(j.mask, j.channels, j.raw_channels, j.slots, j.used);
}

bool aligned(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }
size_t elem_size(int dtype) { return dtype == FH_F32 ? 4u : 2u; }

constexpr int64_t kMaxMixedElems = (int64_t)1 << 31;

fh_status check_shape(int64_t outer, int64_t channels, int64_t inner, int64_t raw_channels, int64_t* numel)
{
    if (outer < 0 || channels < 1 || channels > 16384 || inner < 1) return FH_ERR_BAD_SHAPE;
    if (raw_channels < 0 || raw_channels > channels) return FH_ERR_BAD_SHAPE;
    if (inner > kMaxMixedElems) return FH_ERR_BAD_NUMEL;
    const int64_t per_sample = channels * inner;              // <= 2^45
    if (per_sample > kMaxMixedElems) return FH_ERR_BAD_NUMEL;
    if (outer > kMaxMixedElems / per_sample) return FH_ERR_BAD_NUMEL;
    *numel = outer * per_sample;
    return FH_OK;
}

fh_status check_quantiser(const fh_params* p, bool need_round)
{
    if (!p) return FH_ERR_NULL;
    if (p->group_size != 64 && p->group_size != 128 && p->group_size != 256) return FH_ERR_BAD_GROUP;
    if (p->bits != 2 && p->bits != 4 && p->bits != 8) return FH_ERR_BAD_BITS;
    if (need_round && p->rounding != FH_ROUND_NEAREST && p->rounding != FH_ROUND_STOCHASTIC) return FH_ERR_BAD_ROUND;
    if (p->reserved != 0) return FH_ERR_BAD_PARAM;
    return FH_OK;
}

ChannelMap make_map(const void* slots, void* raw, int64_t channels, int64_t inner, int64_t raw_channels,
                    const void* rows_in_use)
{
    ChannelMap cm;
    cm.rows_in_use = static_cast<const uint64_t*>(rows_in_use);
    cm.slots = static_cast<const int16_t*>(slots);
    cm.raw = raw;
    cm.raw_channels = (uint32_t)raw_channels;
    cm.inner_exact = make_exact_div((uint32_t)inner);
    cm.channels_exact = make_exact_div((uint32_t)channels);
    cm.inner = make_small_div((uint32_t)inner);
    cm.channels = make_small_div((uint32_t)channels);
    cm.raw_div = make_small_div(raw_channels > 0 ? (uint32_t)raw_channels : 1u);
    return cm;
}

}  // namespace
}  // namespace fh

extern "C" {

size_t fh_raw_bytes(int64_t outer, int64_t raw_channels, int64_t inner, fh_dtype dtype)
{
    if (outer <= 0 || raw_channels <= 0 || inner <= 0) return 0;
    if (dtype != FH_F32 && dtype != FH_BF16) return 0;
    return (size_t)outer * (size_t)raw_channels * (size_t)inner * fh::elem_size(dtype);
}

fh_status fh_channel_slots_batch(const fh_slots_item* items, int32_t count, void* stream)
{
    if (count < 0) return FH_ERR_BAD_COUNT;
    if (count > 0 && !items) return FH_ERR_NULL;
    for (int32_t i = 0; i < count; ++i) {                     // everything is checked before the first launch
        const fh_slots_item& it = items[i];
        if (it.channels < 1 || it.channels > 16384 || it.raw_channels < 0 || it.raw_channels > it.channels) return FH_ERR_BAD_SHAPE;
        if (!it.mask || !it.slots) return FH_ERR_NULL;
        if (!fh::aligned(it.slots, 16) || !fh::aligned(it.used, 8)) return FH_ERR_ALIGNMENT;
    }
    for (int32_t i = 0; i < count;) {
        fh::SlotsBatch b;
        int n = 0;
        for (; i < count && n < fh::kBatch; ++i, ++n) {
            const fh_slots_item& it = items[i];
            b.job[n] = fh::SlotsJob{static_cast<const uint8_t*>(it.mask), static_cast<int16_t*>(it.slots),
                                    static_cast<uint64_t*>(it.used), (int32_t)it.channels, (int32_t)it.raw_channels};
        }
        for (int k = n; k < fh::kBatch; ++k) b.job[k] = b.job[0];
        hipLaunchKernelGGL(fh::channel_slots_kernel, dim3(n), dim3(fh::kSlotThreads), 0, static_cast<hipStream_t>(stream), b);
    }
    if (count == 0) return FH_OK;
    return hipGetLastError() == hipSuccess ? FH_OK : FH_ERR_LAUNCH;
}

fh_status fh_channel_slots_used(const void* mask, int64_t channels, int64_t raw_channels, void* slots, void* used,
                                void* stream)
{
    fh_slots_item it;
    it.mask = mask; it.channels = channels; it.raw_channels = raw_channels; it.slots = slots; it.used = used;
    return fh_channel_slots_batch(&it, 1, stream);
}

fh_status fh_channel_slots(const void* mask, int64_t channels, int64_t raw_channels, void* slots, void* stream)
{
    return fh_channel_slots_used(mask, channels, raw_channels, slots, nullptr, stream);
}

}  // extern "C"

namespace {

using namespace fh;

fh_status check_compress(const fh_mixed_item& it, int64_t* numel)
{
    fh_status s;
    if ((s = check_quantiser(&it.params, true)) != FH_OK) return s;
    if (it.reserved != 0) return FH_ERR_BAD_PARAM;
    if (!aligned(it.rows_in_use, 8)) return FH_ERR_ALIGNMENT;
    if (it.x_dtype != FH_F32 && it.x_dtype != FH_BF16) return FH_ERR_BAD_DTYPE;
    if ((s = check_shape(it.outer, it.channels, it.inner, it.raw_channels, numel)) != FH_OK) return s;
    if (*numel == 0) return FH_OK;
    if (!it.x || !it.slots || !it.packed || !it.meta || (it.raw_channels > 0 && !it.raw)) return FH_ERR_NULL;
    if (!aligned(it.x, 16) || !aligned(it.packed, 16) || !aligned(it.meta, 8) || !aligned(it.slots, 16) ||
        !aligned(it.raw, 16))
        return FH_ERR_ALIGNMENT;
    if (it.packed_cap < fh_packed_bytes(*numel, it.params.bits)) return FH_ERR_BUFFER_TOO_SMALL;
    if (it.meta_cap < fh_meta_bytes(*numel, it.params.group_size)) return FH_ERR_BUFFER_TOO_SMALL;
    if (it.raw_cap < fh_raw_bytes(it.outer, it.raw_channels, it.inner, (fh_dtype)it.x_dtype)) return FH_ERR_BUFFER_TOO_SMALL;
    return FH_OK;
}

fh_status check_decompress(const fh_mixed_item& it, int64_t* numel)
{
    fh_status s;
    if ((s = check_quantiser(&it.params, false)) != FH_OK) return s;
    if (it.reserved != 0) return FH_ERR_BAD_PARAM;
    if (!aligned(it.rows_in_use, 8)) return FH_ERR_ALIGNMENT;
    if (it.raw_dtype != FH_F32 && it.raw_dtype != FH_BF16) return FH_ERR_BAD_DTYPE;
    if (it.out_dtype != FH_F32 && it.out_dtype != FH_BF16) return FH_ERR_BAD_DTYPE;
    if ((s = check_shape(it.outer, it.channels, it.inner, it.raw_channels, numel)) != FH_OK) return s;
    if (*numel == 0) return FH_OK;
    if (!it.packed || !it.meta || !it.slots || !it.out || (it.raw_channels > 0 && !it.raw)) return FH_ERR_NULL;
    if (!aligned(it.packed, 16) || !aligned(it.out, 16) || !aligned(it.meta, 8) || !aligned(it.slots, 16) ||
        !aligned(it.raw, 16))
        return FH_ERR_ALIGNMENT;
    if (it.packed_cap < fh_packed_bytes(*numel, it.params.bits)) return FH_ERR_BUFFER_TOO_SMALL;
    if (it.meta_cap < fh_meta_bytes(*numel, it.params.group_size)) return FH_ERR_BUFFER_TOO_SMALL;
    if (it.raw_cap < fh_raw_bytes(it.outer, it.raw_channels, it.inner, (fh_dtype)it.raw_dtype)) return FH_ERR_BUFFER_TOO_SMALL;
    if (it.out_cap < (size_t)*numel * elem_size(it.out_dtype)) return FH_ERR_BUFFER_TOO_SMALL;
    return FH_OK;
}

}  // namespace

extern "C" {

int32_t fh_mixed_batch_capacity(void) { return fh::kBatch; }

fh_status fh_compress_mixed_batch(const fh_mixed_item* items, int32_t count, void* stream)
{
    using namespace fh;
    if (count < 0) return FH_ERR_BAD_COUNT;
    if (count > 0 && !items) return FH_ERR_NULL;
    for (int32_t i = 0; i < count; ++i) {                     // everything is checked before the first launch
        int64_t numel;
        const fh_status st = check_compress(items[i], &numel);
        if (st != FH_OK) return st;
    }
    // a tensor that keeps nothing is the plain quantiser's: its kernels do not look at channels at all
    fh_item plain[kBatch];
    int32_t plain_count = 0;
    for (int32_t k = 0; k <= count; ++k) {
        if (k < count && items[k].raw_channels == 0) {
            const fh_mixed_item& it = items[k];
            fh_item& p = plain[plain_count++];
            p = fh_item{};
            p.x = it.x; p.x_dtype = it.x_dtype; p.out_dtype = FH_F32;
            p.numel = it.outer * it.channels * it.inner;
            p.packed = it.packed; p.packed_cap = it.packed_cap; p.meta = it.meta; p.meta_cap = it.meta_cap;
            p.params = it.params;
        }
        if (plain_count == kBatch || (k == count && plain_count > 0)) {
            const fh_status st = fh_compress_batch(plain, plain_count, stream);
            if (st != FH_OK) return st;
            plain_count = 0;
        }
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    int32_t i = 0;
    while (i < count) {                                       // runs of one dtype and group size
        Batch<MixedCompressJob> b;
        reset(b);
        const int dtype = items[i].x_dtype, G = items[i].params.group_size;
        const int tile = compress_tile_elems(dtype, G);
        while (i < count && items[i].x_dtype == dtype && items[i].params.group_size == G) {
            const fh_mixed_item& it = items[i];
            int64_t numel;
            check_compress(it, &numel);
            if (numel == 0 || it.raw_channels == 0) { ++i; continue; }
            MixedCompressJob job;
            job.it.x = it.x;
            job.it.packed = static_cast<uint8_t*>(it.packed);
            job.it.meta = static_cast<float*>(it.meta);
            job.it.numel = numel;
            job.it.packed_padded = fh_packed_bytes(numel, it.params.bits);
            job.it.seed = it.params.seed;
            job.it.tensor_id = it.params.tensor_id;
            job.it.bits = it.params.bits;
            job.it.stochastic = it.params.rounding == FH_ROUND_STOCHASTIC ? 1 : 0;
            job.cm = make_map(it.slots, it.raw, it.channels, it.inner, it.raw_channels, it.rows_in_use);
            if (!push(b, job, (numel + tile - 1) / tile)) break;      // launch what is there, go on with this item
            ++i;
        }
        if (b.count == 0) continue;
        seal(b);
        if (launch_compress_mixed(b, dtype, G, s) != hipSuccess) return FH_ERR_LAUNCH;
    }
    return FH_OK;
}

fh_status fh_decompress_mixed_batch(const fh_mixed_item* items, int32_t count, void* stream)
{
    using namespace fh;
    if (count < 0) return FH_ERR_BAD_COUNT;
    if (count > 0 && !items) return FH_ERR_NULL;
    for (int32_t i = 0; i < count; ++i) {
        int64_t numel;
        const fh_status st = check_decompress(items[i], &numel);
        if (st != FH_OK) return st;
    }
    fh_item plain[kBatch];                                    // tensors that kept nothing: the plain kernels
    int32_t plain_count = 0;
    for (int32_t k = 0; k <= count; ++k) {
        if (k < count && items[k].raw_channels == 0) {
            const fh_mixed_item& it = items[k];
            fh_item& p = plain[plain_count++];
            p = fh_item{};
            p.x_dtype = FH_F32; p.out_dtype = it.out_dtype;
            p.numel = it.outer * it.channels * it.inner;
            p.packed = it.packed; p.packed_cap = it.packed_cap; p.meta = it.meta; p.meta_cap = it.meta_cap;
            p.out = it.out; p.out_cap = it.out_cap;
            p.params = it.params;
        }
        if (plain_count == kBatch || (k == count && plain_count > 0)) {
            const fh_status st = fh_decompress_batch(plain, plain_count, stream);
            if (st != FH_OK) return st;
            plain_count = 0;
        }
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    int32_t i = 0;
    while (i < count) {
        Batch<MixedDecompressJob> b;
        reset(b);
        const int dtype = items[i].out_dtype, G = items[i].params.group_size;
        const int tile = decompress_tile_elems(dtype, G);
        while (i < count && items[i].out_dtype == dtype && items[i].params.group_size == G) {
            const fh_mixed_item& it = items[i];
            int64_t numel;
            check_decompress(it, &numel);
            if (numel == 0 || it.raw_channels == 0) { ++i; continue; }
            MixedDecompressJob job;
            job.it.packed = static_cast<const uint8_t*>(it.packed);
            job.it.meta = static_cast<const float*>(it.meta);
            job.it.out = it.out;
            job.it.numel = numel;
            job.it.bits = it.params.bits;
            job.it.pad = 0;
            job.cm = make_map(it.slots, it.raw, it.channels, it.inner, it.raw_channels, it.rows_in_use);
            job.raw_dtype = it.raw_dtype;
            job.pad = 0;
            if (!push(b, job, (numel + tile - 1) / tile)) break;
            ++i;
        }
        if (b.count == 0) continue;
        seal(b);
        if (launch_decompress_mixed(b, dtype, G, s) != hipSuccess) return FH_ERR_LAUNCH;
    }
    return FH_OK;
}

fh_status fh_compress_mixed(const void* x, fh_dtype x_dtype, int64_t outer, int64_t channels, int64_t inner,
                            const fh_params* params, const void* slots, int64_t raw_channels,
                            void* packed, size_t packed_cap, void* meta, size_t meta_cap,
                            void* raw, size_t raw_cap, void* stream)
{
    if (!params) return FH_ERR_NULL;
    fh_mixed_item it = {};
    it.x = x; it.x_dtype = x_dtype; it.out_dtype = FH_F32;
    it.outer = outer; it.channels = channels; it.inner = inner;
    it.slots = slots; it.raw_channels = raw_channels;
    it.packed = packed; it.packed_cap = packed_cap; it.meta = meta; it.meta_cap = meta_cap;
    it.raw = raw; it.raw_cap = raw_cap; it.raw_dtype = x_dtype;
    it.params = *params;
    return fh_compress_mixed_batch(&it, 1, stream);
}

fh_status fh_decompress_mixed(const void* packed, const void* meta, const void* raw, fh_dtype raw_dtype,
                              int64_t outer, int64_t channels, int64_t inner,
                              const fh_params* params, const void* slots, int64_t raw_channels,
                              fh_dtype out_dtype, void* out, size_t out_cap, void* stream)
{
    if (!params) return FH_ERR_NULL;
    fh_mixed_item it = {};
    it.x_dtype = FH_F32; it.out_dtype = out_dtype;
    it.outer = outer; it.channels = channels; it.inner = inner;
    it.slots = slots; it.raw_channels = raw_channels;
    it.packed = const_cast<void*>(packed); it.meta = const_cast<void*>(meta);
    it.raw = const_cast<void*>(raw); it.raw_dtype = raw_dtype;
    it.out = out; it.out_cap = out_cap;
    it.params = *params;
    // the single call takes no capacities for its inputs: they are what the shape implies
    int64_t numel = 0;
    if (fh::check_shape(outer, channels, inner, raw_channels, &numel) == FH_OK && numel > 0 &&
        (raw_dtype == FH_F32 || raw_dtype == FH_BF16)) {
        it.packed_cap = fh_packed_bytes(numel, params->bits);
        it.meta_cap = fh_meta_bytes(numel, params->group_size);
        it.raw_cap = fh_raw_bytes(outer, raw_channels, inner, raw_dtype);
    }
    return fh_decompress_mixed_batch(&it, 1, stream);
}

}  // extern "C"
