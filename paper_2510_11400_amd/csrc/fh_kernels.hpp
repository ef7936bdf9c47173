// Kernel argument blocks and launcher declarations shared by the kernel files and
// the C ABI.  A launch covers up to kMaxItems tensors: the descriptors travel by
// value in the kernel-argument segment (no device-side table, no allocation), and
// each workgroup finds its tensor by a binary search over tile_start[].
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "fh_batch.hpp"
#include "fh_channels.hpp"

namespace fh {

constexpr int kMaxItems = 48;

struct CompressItem {
    const void* x;                     // device, 16-byte aligned
    uint8_t*    packed;                // device, 16-byte aligned
    float*      meta;                  // device, 8-byte aligned; {scale, zero} per group
    int64_t     numel;
    uint64_t    packed_padded;         // bytes to write at `packed` (multiple of 16)
    uint64_t    seed;
    uint64_t    tensor_id;
    int32_t     bits;                  // 2 | 4 | 8
    int32_t     stochastic;            // 0 | 1
};

struct CompressBatch {
    int32_t      count;
    uint32_t     tile_start[kMaxItems + 1];   // exclusive prefix sum of tiles per item
    CompressItem item[kMaxItems];
};

struct DecompressItem {
    const uint8_t* packed;
    const float*   meta;
    void*          out;                // device, 16-byte aligned
    int64_t        numel;
    int32_t        bits;
    int32_t        pad;
};

struct DecompressBatch {
    int32_t        count;
    uint32_t       tile_start[kMaxItems + 1];
    DecompressItem item[kMaxItems];
};

static_assert(sizeof(CompressBatch) <= 4096, "kernel arguments must fit the 4 KiB segment");
static_assert(sizeof(DecompressBatch) <= 4096, "kernel arguments must fit the 4 KiB segment");

// The item a workgroup's tile belongs to: the last one whose first tile is <= bid.  Entries
// past the last item repeat the total (> bid), so every entry may be compared.  Two rounds of
// independent scalar loads -- every 8th entry, then the entries inside that run -- instead of a
// binary search's chain of six dependent ones: a wave cannot issue its first data load before
// this is done.
static_assert(kMaxItems == 48, "find_item walks 6 runs of 8");
__device__ __forceinline__ int find_item(const uint32_t (&tile_start)[kMaxItems + 1], uint32_t bid)
{
    int run = 0;
#pragma unroll
    for (int k = 1; k < kMaxItems / 8; ++k) run += tile_start[8 * k] <= bid ? 1 : 0;
    const int first = 8 * run;
    int lo = first;
#pragma unroll
    for (int i = 1; i < 8; ++i) lo += tile_start[first + i] <= bid ? 1 : 0;
    return lo;
}

// Elements one workgroup covers (same for every bit width, so tile_start[] can be
// built on the host without knowing which variant a tile dispatches to).
int compress_tile_elems(int dtype, int group_size);
int decompress_tile_elems(int out_dtype, int group_size);

// Enqueue one launch; tile_start[count] workgroups.  dtype: 0 = f32, 1 = bf16.
hipError_t launch_compress(const CompressBatch& b, int dtype, int group_size, hipStream_t s);
hipError_t launch_decompress(const DecompressBatch& b, int out_dtype, int group_size, hipStream_t s);

// The same for [outer][channels][inner] tensors some of whose channels are kept verbatim in a raw
// store instead of being quantised (at most 2^31 elements each; up to kBatch tensors per launch).
struct MixedCompressJob {
    CompressItem it;
    ChannelMap   cm;
};
struct MixedDecompressJob {
    DecompressItem it;
    ChannelMap     cm;
    int32_t        raw_dtype;
    int32_t        pad;
};
hipError_t launch_compress_mixed(const Batch<MixedCompressJob>& b, int dtype, int group_size, hipStream_t s);
hipError_t launch_decompress_mixed(const Batch<MixedDecompressJob>& b, int out_dtype, int group_size, hipStream_t s);

}  // namespace fh
