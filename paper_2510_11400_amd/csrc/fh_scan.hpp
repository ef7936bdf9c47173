// Prefix sums over a wave of 64 lanes on the vector ALU (data-parallel-primitive adds, no LDS):
// four shifts inside each row of 16 lanes, then the last lane of rows 0 and 2 onto rows 1 and
// 3, then lane 31 onto rows 2 and 3.  Shared by the stream-compaction passes of the sparse
// storage and of the entropy stage.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fh {

// v + (the lane the control word names, 0 where there is none or the row is masked out)
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ uint32_t dpp_add(uint32_t v)
{
    return v + (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, ROW_MASK, 0xf, false);
}
// every lane of the wave must be active
__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t v)
{
    v = dpp_add<0x111, 0xf>(v);                               // row_shr:1
    v = dpp_add<0x112, 0xf>(v);                               // row_shr:2
    v = dpp_add<0x114, 0xf>(v);                               // row_shr:4
    v = dpp_add<0x118, 0xf>(v);                               // row_shr:8
    v = dpp_add<0x142, 0xa>(v);                               // row_bcast:15 onto rows 1 and 3
    v = dpp_add<0x143, 0xc>(v);                               // row_bcast:31 onto rows 2 and 3
    return v;
}
// lane 63's value, in a scalar register
__device__ __forceinline__ uint32_t last_lane(uint32_t v) { return (uint32_t)__builtin_amdgcn_readlane((int)v, 63); }

}  // namespace fh
