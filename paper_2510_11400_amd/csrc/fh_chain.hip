// The channel-wise mix compressor as one call each way (paper Section 4.4.1 from its first
// sentence to its last; Algorithm 1 sees exactly these two actions, compress and decompress):
//
//   forward   classify channels (three-sigma rule) -> number the salient ones -> quantise the
//             normal channels, salient ones to a raw store -> the raw store's feature maps as
//             sparse blocks (CSR) and dense blocks (Lorenzo prediction within an error bound)
//             -> Huffman coding of the index stream;
//   backward  Huffman decoding -> maps rebuilt -> normal channels dequantised, salient channels
//             taken from the maps.
//
// Every stage is the library's own batched call; this file only lays the caller's two buffers
// out, strings the calls together on one stream, and adds two small kernels: one that numbers
// the salient channels of every tensor of the call, clears the raw stores (rows of unused slots
// must read as zero for the sparse stage) and the headers, and one that adds up what a tensor's
// stored form occupies.  Sizes that depend on the data (stream lengths) never visit the host:
// the sparse stage's totals feed the Huffman stage through device memory.
#include "../../include/fedhybrid.h"

#include "fh_batch.hpp"

#include <vector>

namespace fh {
namespace {

constexpr int kPrepThreads = 1024;
constexpr int kSlotPerThread = 16;                 // 1024 * 16 = the largest channel count
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

struct PrepItem {
    const uint8_t* mask;
    int16_t*       slots;
    uint64_t*      header;                         // 8 words, cleared; [7] = slots in use
    u32x4*         raw;                            // cleared: raw_vectors 16-byte vectors
    uint64_t       raw_vectors;
    int32_t        channels, raw_channels;
    uint32_t       blocks;                         // workgroups of this item
};

// Workgroup 0 of an item: slots[c] = number of salient channels before c while that is below
// raw_channels, -1 for every other channel (each thread owns 16 consecutive channels, the
// per-thread counts are scanned through LDS), and the header cleared.  All workgroups of the
// item: the raw store cleared.
__global__ __launch_bounds__(kPrepThreads) void chain_prepare_kernel(const Batch<PrepItem> batch)
{
    uint32_t block;
    const PrepItem& it = batch.item[batch_item(batch, blockIdx.x, block)];
    const u32x4 zero = {0u, 0u, 0u, 0u};
    for (uint64_t v = (uint64_t)block * kPrepThreads + threadIdx.x; v < it.raw_vectors; v += (uint64_t)it.blocks * kPrepThreads)
        it.raw[v] = zero;
    if (block != 0) return;                                   // workgroup-uniform
    __shared__ int scan[kPrepThreads];
    const int t = threadIdx.x;
    const int first = t * kSlotPerThread;
    int mine = 0;
    for (int k = 0; k < kSlotPerThread; ++k) {
        const int c = first + k;
        if (c < it.channels && it.mask[c] != 0) ++mine;
    }
    scan[t] = mine;
    __syncthreads();
    for (int step = 1; step < kPrepThreads; step <<= 1) {     // inclusive scan, all threads reach every barrier
        const int add = t >= step ? scan[t - step] : 0;
        __syncthreads();
        scan[t] += add;
        __syncthreads();
    }
    int rank = scan[t] - mine;                                // salient channels before this thread's first
    for (int k = 0; k < kSlotPerThread; ++k) {
        const int c = first + k;
        if (c >= it.channels) break;
        const bool salient = it.mask[c] != 0;
        it.slots[c] = (int16_t)(salient && rank < it.raw_channels ? rank : -1);
        if (salient) ++rank;
    }
    if (t < 7) it.header[t] = 0u;
    if (t == kPrepThreads - 1) it.header[7] = (uint64_t)(scan[t] < it.raw_channels ? scan[t] : it.raw_channels);
}

struct SummaryItem {
    uint64_t* header;
    uint64_t  fixed_bytes;                         // header + slots + codes + meta + info
    uint32_t  value_size;                          // bytes per element of the value stream
    int32_t   entropy;
};
struct SummaryBatch { int32_t count; SummaryItem item[kBatch]; };

__global__ void chain_summary_kernel(const SummaryBatch batch)
{
    const int i = threadIdx.x;
    if (i >= batch.count) return;
    const SummaryItem& it = batch.item[i];
    it.header[6] = it.fixed_bytes + it.header[0] * it.value_size + (it.entropy ? it.header[4] : it.header[1]);
}

size_t up(size_t v) { return (v + 255u) & ~(size_t)255u; }
size_t elem_size(int dtype) { return dtype == FH_F32 ? 4u : 2u; }
bool aligned(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

// Everything about an item that does not involve its buffers.
fh_status check_shape(const fh_mix_item& it, int64_t* numel)
{
    if (it.x_dtype != FH_F32 && it.x_dtype != FH_BF16) return FH_ERR_BAD_DTYPE;
    if (it.reserved != 0 || it.quant.reserved != 0) return FH_ERR_BAD_PARAM;
    if (it.quant.group_size != 64 && it.quant.group_size != 128 && it.quant.group_size != 256) return FH_ERR_BAD_GROUP;
    if (it.quant.bits != 2 && it.quant.bits != 4 && it.quant.bits != 8) return FH_ERR_BAD_BITS;
    if (it.quant.rounding != FH_ROUND_NEAREST && it.quant.rounding != FH_ROUND_STOCHASTIC) return FH_ERR_BAD_ROUND;
    if (it.outer < 0 || it.channels < 1 || it.channels > 16384 || it.inner < 1) return FH_ERR_BAD_SHAPE;
    if (it.raw_channels < 0 || it.raw_channels > it.channels) return FH_ERR_BAD_SHAPE;
    if (!(it.k_sigma > 0.0) || it.min_outliers < 1) return FH_ERR_BAD_PARAM;
    if (it.entropy != 0 && it.entropy != 1) return FH_ERR_BAD_PARAM;
    const int64_t limit = (int64_t)1 << 31;                   // the routed quantiser indexes elements with 32 bits
    if (it.inner > limit || it.channels * it.inner > limit) return FH_ERR_BAD_NUMEL;
    if (it.outer > limit / (it.channels * it.inner)) return FH_ERR_BAD_NUMEL;
    *numel = it.outer * it.channels * it.inner;
    const int64_t kept = it.outer * it.raw_channels * it.inner;
    if (kept > 0) {
        if (it.window != 2 && it.window != 4 && it.window != 8) return FH_ERR_BAD_PARAM;
        if (it.maps < 1 || it.h < 1 || it.w < 1) return FH_ERR_BAD_SHAPE;
        if (it.h > kept || it.w > kept / it.h || it.maps != kept / (it.h * it.w) || it.maps * it.h * it.w != kept)
            return FH_ERR_BAD_SHAPE;                          // the maps must be exactly the raw store
    }
    return FH_OK;
}

fh_status layout_of(const fh_mix_item& it, fh_mix_regions* r)
{
    int64_t numel = 0;
    const fh_status st = check_shape(it, &numel);
    if (st != FH_OK) return st;
    *r = fh_mix_regions{};
    const int64_t kept = it.outer * it.raw_channels * it.inner;
    r->packed_bytes = fh_packed_bytes(numel, it.quant.bits);
    r->meta_bytes = fh_meta_bytes(numel, it.quant.group_size);
    r->slots_bytes = 2u * (size_t)it.channels;
    r->raw_bytes = (size_t)kept * elem_size(it.x_dtype);
    r->classify_ws_bytes = fh_classify_workspace_bytes(numel);
    if (kept > 0) {
        r->info_bytes = fh_sparse_info_bytes(it.maps, it.h, it.w, it.window);
        r->values_cap = r->raw_bytes;
        r->indices_cap = fh_sparse_index_bytes(it.maps, it.h, it.w, it.window);
        r->sparse_ws_bytes = fh_sparse_workspace_bytes(it.maps, it.h, it.w, it.window);
        if (r->indices_cap >= ((size_t)1 << 32)) return FH_ERR_BAD_NUMEL;
        if (it.entropy) {
            r->huffman_cap = fh_huffman_stream_bytes(r->indices_cap);
            r->huffman_ws_bytes = fh_huffman_workspace_bytes(r->indices_cap);
        }
    }
    size_t at = 0;
    const auto place = [&at](size_t bytes) { const size_t here = at; at += up(bytes); return here; };
    r->header = place(64);
    r->slots = place(r->slots_bytes);
    r->packed = place(r->packed_bytes);
    r->meta = place(r->meta_bytes);
    r->info = place(r->info_bytes);
    r->values = place(r->values_cap);
    r->indices = it.entropy ? 0 : place(r->indices_cap);
    r->huffman = it.entropy ? place(r->huffman_cap) : 0;
    r->store_bytes = at;
    at = 0;
    r->stats = place(32);
    r->counts = place(4u * (size_t)it.channels);
    r->mask = place((size_t)it.channels);
    r->classify_ws = place(r->classify_ws_bytes);
    r->raw = place(r->raw_bytes);
    r->sparse_ws = place(r->sparse_ws_bytes);
    r->indices_ws = it.entropy ? place(r->indices_cap) : 0;
    r->huffman_ws = place(r->huffman_ws_bytes);
    r->workspace_bytes = at;
    return FH_OK;
}

fh_status check_item(const fh_mix_item& it, bool forward, fh_mix_regions* r, int64_t* numel)
{
    fh_status st = layout_of(it, r);
    if (st != FH_OK) return st;
    check_shape(it, numel);
    if (!forward && it.out_dtype != FH_F32 && it.out_dtype != FH_BF16) return FH_ERR_BAD_DTYPE;
    if (!it.store || !it.workspace) return FH_ERR_NULL;
    if (*numel > 0 && (forward ? !it.x : !it.out)) return FH_ERR_NULL;
    if (!aligned(it.store, 256) || !aligned(it.workspace, 256) || !aligned(forward ? it.x : it.out, 16)) return FH_ERR_ALIGNMENT;
    if (it.store_cap < r->store_bytes || it.workspace_cap < r->workspace_bytes) return FH_ERR_BUFFER_TOO_SMALL;
    if (!forward && it.out_cap < (size_t)*numel * elem_size(it.out_dtype)) return FH_ERR_BUFFER_TOO_SMALL;
    return FH_OK;
}

uint8_t* at(void* base, size_t off) { return static_cast<uint8_t*>(base) + off; }

}  // namespace
}  // namespace fh

extern "C" {

fh_status fh_mix_layout(const fh_mix_item* item, fh_mix_regions* regions)
{
    if (!item || !regions) return FH_ERR_NULL;
    return fh::layout_of(*item, regions);
}

fh_status fh_mix_compress_batch(const fh_mix_item* items, int32_t count, void* stream)
{
    using namespace fh;
    if (count < 0) return FH_ERR_BAD_COUNT;
    if (count > 0 && !items) return FH_ERR_NULL;
    std::vector<fh_mix_regions> reg((size_t)count);
    std::vector<int64_t> numel((size_t)count);
    for (int32_t i = 0; i < count; ++i) {                     // everything is checked before the first launch
        const fh_status st = check_item(items[i], true, &reg[i], &numel[i]);
        if (st != FH_OK) return st;
    }
    if (count == 0) return FH_OK;
    hipStream_t s = static_cast<hipStream_t>(stream);
    fh_status st;

    // 1. three-sigma statistics, outlier counts, salient mask
    std::vector<fh_classify_item> cls((size_t)count);
    for (int32_t i = 0; i < count; ++i) {
        const fh_mix_item& it = items[i];
        fh_classify_item& c = cls[i];
        c = fh_classify_item{};
        c.x = it.x; c.x_dtype = it.x_dtype;
        c.outer = it.outer; c.channels = it.channels; c.inner = it.inner;
        c.k_sigma = it.k_sigma; c.min_outliers = it.min_outliers;
        c.workspace = at(it.workspace, reg[i].classify_ws); c.workspace_cap = reg[i].classify_ws_bytes;
        c.stats = at(it.workspace, reg[i].stats); c.counts = at(it.workspace, reg[i].counts);
        c.mask = at(it.workspace, reg[i].mask);
    }
    if ((st = fh_classify_channels_batch(cls.data(), count, stream)) != FH_OK) return st;

    // 2. slots from the masks; headers and raw stores cleared
    for (int32_t i = 0; i < count;) {
        Batch<PrepItem> b;
        reset(b);
        for (; i < count && b.count < kBatch; ++i) {
            const fh_mix_item& it = items[i];
            PrepItem p;
            p.mask = at(it.workspace, reg[i].mask);
            p.slots = reinterpret_cast<int16_t*>(at(it.store, reg[i].slots));
            p.header = reinterpret_cast<uint64_t*>(at(it.store, reg[i].header));
            p.raw = reinterpret_cast<u32x4*>(at(it.workspace, reg[i].raw));
            p.raw_vectors = (reg[i].raw_bytes + 15u) / 16u;   // the region is padded to 256 bytes
            p.channels = (int32_t)it.channels;
            p.raw_channels = (int32_t)it.raw_channels;
            const uint64_t want = (p.raw_vectors + (uint64_t)kPrepThreads * 8u - 1u) / ((uint64_t)kPrepThreads * 8u);
            p.blocks = (uint32_t)(want < 1u ? 1u : want > 1024u ? 1024u : want);
            push(b, p, p.blocks);
        }
        seal(b);
        hipLaunchKernelGGL(chain_prepare_kernel, dim3(b.block_start[b.count]), dim3(kPrepThreads), 0, s, b);
    }

    // 3. normal channels quantised, salient channels to the raw store
    std::vector<fh_mixed_item> mix((size_t)count);
    for (int32_t i = 0; i < count; ++i) {
        const fh_mix_item& it = items[i];
        fh_mixed_item& m = mix[i];
        m = fh_mixed_item{};
        m.x = it.x; m.x_dtype = it.x_dtype; m.out_dtype = FH_F32;
        m.outer = it.outer; m.channels = it.channels; m.inner = it.inner;
        m.slots = at(it.store, reg[i].slots); m.raw_channels = it.raw_channels;
        m.packed = at(it.store, reg[i].packed); m.packed_cap = reg[i].packed_bytes;
        m.meta = at(it.store, reg[i].meta); m.meta_cap = reg[i].meta_bytes;
        m.raw = at(it.workspace, reg[i].raw); m.raw_cap = reg[i].raw_bytes; m.raw_dtype = it.x_dtype;
        m.params = it.quant;
        m.rows_in_use = at(it.store, reg[i].header) + 7 * sizeof(uint64_t);
    }
    if ((st = fh_compress_mixed_batch(mix.data(), count, stream)) != FH_OK) return st;

    // 4. the raw stores as sparse / predicted blocks; 5. their index streams Huffman-coded
    std::vector<fh_sparse_encode_item> sp;
    std::vector<fh_huffman_encode_item> hf;
    for (int32_t i = 0; i < count; ++i) {
        const fh_mix_item& it = items[i];
        if (reg[i].raw_bytes == 0) continue;
        uint64_t* header = reinterpret_cast<uint64_t*>(at(it.store, reg[i].header));
        fh_sparse_encode_item e = {};
        e.x = at(it.workspace, reg[i].raw); e.dtype = it.x_dtype; e.n = it.window;
        e.maps = it.maps; e.h = it.h; e.w = it.w; e.tau = it.tau; e.eps = it.eps;
        e.info = at(it.store, reg[i].info); e.info_cap = reg[i].info_bytes;
        e.values = at(it.store, reg[i].values); e.values_cap = reg[i].values_cap;
        e.indices = it.entropy ? at(it.workspace, reg[i].indices_ws) : at(it.store, reg[i].indices);
        e.indices_cap = reg[i].indices_cap;
        e.totals = header;
        e.workspace = at(it.workspace, reg[i].sparse_ws); e.workspace_cap = reg[i].sparse_ws_bytes;
        sp.push_back(e);
        if (it.entropy) {
            fh_huffman_encode_item h = {};
            h.bytes = e.indices; h.n = reg[i].indices_cap; h.n_device = header + 1;
            h.stream_out = at(it.store, reg[i].huffman); h.stream_cap = reg[i].huffman_cap;
            h.totals = header + 4;
            h.workspace = at(it.workspace, reg[i].huffman_ws); h.workspace_cap = reg[i].huffman_ws_bytes;
            hf.push_back(h);
        }
    }
    if (!sp.empty() && (st = fh_sparse_encode_batch(sp.data(), (int32_t)sp.size(), stream)) != FH_OK) return st;
    if (!hf.empty() && (st = fh_huffman_encode_batch(hf.data(), (int32_t)hf.size(), stream)) != FH_OK) return st;

    // 6. what each stored form occupies
    for (int32_t i = 0; i < count;) {
        SummaryBatch b;
        b.count = 0;
        for (; i < count && b.count < kBatch; ++i) {
            SummaryItem& q = b.item[b.count++];
            q.header = reinterpret_cast<uint64_t*>(at(items[i].store, reg[i].header));
            q.fixed_bytes = 64u + reg[i].packed_bytes + reg[i].meta_bytes +
                            (reg[i].raw_bytes ? reg[i].slots_bytes + reg[i].info_bytes : 0u);
            q.value_size = (uint32_t)elem_size(items[i].x_dtype);
            q.entropy = items[i].entropy;
        }
        hipLaunchKernelGGL(chain_summary_kernel, dim3(1), dim3(64), 0, s, b);
    }
    return hipGetLastError() == hipSuccess ? FH_OK : FH_ERR_LAUNCH;
}

fh_status fh_mix_decompress_batch(const fh_mix_item* items, int32_t count, void* stream)
{
    using namespace fh;
    if (count < 0) return FH_ERR_BAD_COUNT;
    if (count > 0 && !items) return FH_ERR_NULL;
    std::vector<fh_mix_regions> reg((size_t)count);
    std::vector<int64_t> numel((size_t)count);
    for (int32_t i = 0; i < count; ++i) {
        const fh_status st = check_item(items[i], false, &reg[i], &numel[i]);
        if (st != FH_OK) return st;
    }
    if (count == 0) return FH_OK;
    fh_status st;

    // the index streams back, then the maps (the raw stores), then the tensors
    std::vector<fh_huffman_decode_item> hf;
    std::vector<fh_sparse_decode_item> sp;
    for (int32_t i = 0; i < count; ++i) {
        const fh_mix_item& it = items[i];
        if (reg[i].raw_bytes == 0) continue;
        const uint64_t* header = reinterpret_cast<const uint64_t*>(at(it.store, reg[i].header));
        const void* indices = it.entropy ? at(it.workspace, reg[i].indices_ws) : at(it.store, reg[i].indices);
        if (it.entropy) {
            fh_huffman_decode_item h = {};
            h.stream_in = at(it.store, reg[i].huffman); h.stream_bytes = reg[i].huffman_cap;
            h.n = reg[i].indices_cap; h.n_device = header + 1;
            h.out = at(it.workspace, reg[i].indices_ws); h.out_cap = reg[i].indices_cap;
            hf.push_back(h);
        }
        fh_sparse_decode_item d = {};
        d.info = at(it.store, reg[i].info);
        d.values = at(it.store, reg[i].values); d.values_bytes = reg[i].values_cap;
        d.indices = indices; d.indices_bytes = reg[i].indices_cap;
        d.dtype = it.x_dtype; d.n = it.window; d.maps = it.maps; d.h = it.h; d.w = it.w; d.eps = it.eps;
        d.out = at(it.workspace, reg[i].raw); d.out_cap = reg[i].raw_bytes;
        d.workspace = at(it.workspace, reg[i].sparse_ws); d.workspace_cap = reg[i].sparse_ws_bytes;
        sp.push_back(d);
    }
    if (!hf.empty() && (st = fh_huffman_decode_batch(hf.data(), (int32_t)hf.size(), stream)) != FH_OK) return st;
    if (!sp.empty() && (st = fh_sparse_decode_batch(sp.data(), (int32_t)sp.size(), stream)) != FH_OK) return st;

    std::vector<fh_mixed_item> mix((size_t)count);
    for (int32_t i = 0; i < count; ++i) {
        const fh_mix_item& it = items[i];
        fh_mixed_item& m = mix[i];
        m = fh_mixed_item{};
        m.x_dtype = FH_F32; m.out_dtype = it.out_dtype;
        m.outer = it.outer; m.channels = it.channels; m.inner = it.inner;
        m.slots = at(it.store, reg[i].slots); m.raw_channels = it.raw_channels;
        m.packed = at(it.store, reg[i].packed); m.packed_cap = reg[i].packed_bytes;
        m.meta = at(it.store, reg[i].meta); m.meta_cap = reg[i].meta_bytes;
        m.raw = at(it.workspace, reg[i].raw); m.raw_cap = reg[i].raw_bytes; m.raw_dtype = it.x_dtype;
        m.out = it.out; m.out_cap = it.out_cap;
        m.params = it.quant;
        m.rows_in_use = at(it.store, reg[i].header) + 7 * sizeof(uint64_t);
    }
    return fh_decompress_mixed_batch(mix.data(), count, stream);
}

fh_status fh_mix_compress(const fh_mix_item* item, void* stream)
{
    return item ? fh_mix_compress_batch(item, 1, stream) : FH_ERR_NULL;
}

fh_status fh_mix_decompress(const fh_mix_item* item, void* stream)
{
    return item ? fh_mix_decompress_batch(item, 1, stream) : FH_ERR_NULL;
}

}  // extern "C"
