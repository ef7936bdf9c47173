// Several tensors per launch: descriptors travel by value in the kernel-argument segment and a
// workgroup finds its tensor by a scalar search over the exclusive prefix sums of the tensors'
// workgroup counts (entries past the last tensor repeat the total).
#pragma once

#include <hip/hip_runtime.h>
#include <limits.h>
#include <stdint.h>

namespace fh {

constexpr int kBatch = 16;

template <typename Item> struct Batch {
    int32_t  count;
    uint32_t block_start[kBatch + 1];
    Item     item[kBatch];
};

// index of the tensor workgroup `bid` works on; `local` = its workgroup number inside that tensor
template <typename Item>
__device__ __forceinline__ int batch_item(const Batch<Item>& b, uint32_t bid, uint32_t& local)
{
    int lo = 0, hi = b.count;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (b.block_start[mid] <= bid) lo = mid; else hi = mid;
    }
    local = bid - b.block_start[lo];
    return lo;
}

// host side: append an item that needs `blocks` workgroups; false when the launch is full
template <typename Item>
inline bool push(Batch<Item>& b, const Item& item, int64_t blocks)
{
    if (b.count == kBatch || (uint64_t)b.block_start[b.count] + (uint64_t)blocks > (uint64_t)INT_MAX) return false;
    b.item[b.count] = item;
    b.block_start[b.count + 1] = b.block_start[b.count] + (uint32_t)blocks;
    ++b.count;
    return true;
}
template <typename Item> inline void seal(Batch<Item>& b)
{
    for (int k = b.count + 1; k <= kBatch; ++k) b.block_start[k] = b.block_start[b.count];
}
template <typename Item> inline void reset(Batch<Item>& b) { b.count = 0; b.block_start[0] = 0; }

}  // namespace fh
