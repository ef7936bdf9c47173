// Device-side building blocks for the gfx950 group quantiser: cross-lane min/max,
// Philox4x32-10, bf16 conversion, 128-bit memory access.  Wave size is 64.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "fh_types.hpp"

namespace fh {


// ---- streaming memory access --------------------------------------------------------
// The activation and the restored tensor are each touched once per call and are far larger
// than any cache: they are loaded and stored with the non-temporal hint (measured on MI355X:
// ordinary loads of the activation evict the code stream from the memory-side cache and cost
// the round trip 15 %; stores with the sc1 / sc0 sc1 scope bits, which write through, restore the
// 2 GiB mixed set 2 % slower than the non-temporal ones when the codes are cold and 13 % slower
// back to back, although they are 7-8 % faster on the two small-group sets).
template <typename T>
__device__ __forceinline__ T stream_load(const T* p) { return __builtin_nontemporal_load(p); }
template <typename T>
__device__ __forceinline__ void stream_store(T* p, T v) { __builtin_nontemporal_store(v, p); }
// The code stream and the meta pairs are small and are read back by the backward side: ordinary
// stores and loads.  Measured with the memory-side cache displaced between the two sides
// (2 GiB mixed set): non-temporal code stores cost the forward side 3 %, non-temporal code
// loads the backward side 8 % (lanes share the words they read); with the two sides back to
// back, ordinary accesses let the backward side find the latest codes in that cache.
template <typename T>
__device__ __forceinline__ void code_store(T* p, T v) { *p = v; }
template <typename T>
__device__ __forceinline__ T code_load(const T* p) { return *p; }

// ---- min / max ---------------------------------------------------------------------
// Written as the machine instructions themselves.  The inputs are finite by contract,
// so no NaN canonicalisation is wanted in front of them, and the result must not
// depend on how a compiler folds min/max against infinities.  v_min_f32 / v_max_f32
// return the smaller / larger operand; for +0 vs -0 either may come back, which the
// caller canonicalises.
__device__ __forceinline__ float vmin(float a, float b)
{
    float r;
    asm volatile("v_min_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}
__device__ __forceinline__ float vmax(float a, float b)
{
    float r;
    asm volatile("v_max_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}
__device__ __forceinline__ float vmin3(float a, float b, float c)
{
    float r;
    asm volatile("v_min3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}
__device__ __forceinline__ float vmax3(float a, float b, float c)
{
    float r;
    asm volatile("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}

// ---- cross-lane min / max ----------------------------------------------------------
// One DPP step folds a lane with its partner inside the 16-lane row: xor 1 and xor 2
// through quad_perm, then row_half_mirror (lane i <-> 7-i of its 8) once quads are
// uniform, then row_mirror (i <-> 15-i) once halves are uniform.  min and max chains
// are interleaved so that each DPP read sits two wait states after the VALU write of
// its register (a hazard the compiler cannot see inside an asm block): the other
// chain's instruction plus one s_nop.  The block opens and closes with s_nop 1 so it
// is safe against whatever the compiler schedules around it.
#define FH_DPP_STEP(CTRL)                                                           \
    "v_min_f32_dpp %0, %0, %0 " CTRL " row_mask:0xf bank_mask:0xf\n\t"              \
    "v_max_f32_dpp %1, %1, %1 " CTRL " row_mask:0xf bank_mask:0xf\n\t"
template <int LANES>
__device__ __forceinline__ void row_minmax(float& mn, float& mx)
{
    static_assert(LANES == 4 || LANES == 8 || LANES == 16, "within one DPP row");
    if constexpr (LANES == 4) {
        asm volatile("s_nop 1\n\t" FH_DPP_STEP("quad_perm:[1,0,3,2]") "s_nop 0\n\t"
                     FH_DPP_STEP("quad_perm:[2,3,0,1]") "s_nop 1" : "+v"(mn), "+v"(mx));
    } else if constexpr (LANES == 8) {
        asm volatile("s_nop 1\n\t" FH_DPP_STEP("quad_perm:[1,0,3,2]") "s_nop 0\n\t"
                     FH_DPP_STEP("quad_perm:[2,3,0,1]") "s_nop 0\n\t"
                     FH_DPP_STEP("row_half_mirror") "s_nop 1" : "+v"(mn), "+v"(mx));
    } else {
        asm volatile("s_nop 1\n\t" FH_DPP_STEP("quad_perm:[1,0,3,2]") "s_nop 0\n\t"
                     FH_DPP_STEP("quad_perm:[2,3,0,1]") "s_nop 0\n\t"
                     FH_DPP_STEP("row_half_mirror") "s_nop 0\n\t"
                     FH_DPP_STEP("row_mirror") "s_nop 1" : "+v"(mn), "+v"(mx));
    }
}
#undef FH_DPP_STEP

// Both halves of a permlane swap of a value with itself (gfx950).  The second operand
// goes through an empty asm so the compiler treats the two inputs as unrelated values:
// the swap moves data between lanes, and its two results differ even when its two
// inputs are the same register.
template <int WIDTH>
__device__ __forceinline__ void self_swap(float v, float& first, float& second)
{
    const uint32_t a = __builtin_bit_cast(uint32_t, v);
    uint32_t b = a;
    asm volatile("" : "+v"(b));
    u32x2 r;
    if constexpr (WIDTH == 16) r = __builtin_amdgcn_permlane16_swap(a, b, false, false);
    else r = __builtin_amdgcn_permlane32_swap(a, b, false, false);
    const uint32_t r0 = r.x, r1 = r.y;   // scalars first: bit_cast wants an object, not a vector lane
    first = __builtin_bit_cast(float, r0);
    second = __builtin_bit_cast(float, r1);
}

// Min and max over aligned runs of LANES consecutive lanes; every lane of the run
// ends with the run's result.  min/max are exact and order-independent, so any
// exchange order gives the same value.  All 64 lanes must be active.
template <int LANES>
__device__ __forceinline__ void group_minmax(float& mn, float& mx)
{
    static_assert(LANES == 4 || LANES == 8 || LANES == 16 || LANES == 32 || LANES == 64, "run length");
    row_minmax<(LANES < 16 ? LANES : 16)>(mn, mx);
    if constexpr (LANES >= 32) {
        // v_permlane16_swap exchanges the odd 16-lane rows of its first operand with the
        // even rows of its second: two copies of v come back as rows {0,0,2,2} and
        // {1,1,3,3}, whose min/max is the 32-lane result.
        float a, b;
        self_swap<16>(mn, a, b);  mn = vmin(a, b);
        self_swap<16>(mx, a, b);  mx = vmax(a, b);
    }
    if constexpr (LANES >= 64) {
        // v_permlane32_swap exchanges lanes 32..63 of the first operand with lanes 0..31
        // of the second: {lo,lo} and {hi,hi}.
        float a, b;
        self_swap<32>(mn, a, b);  mn = vmin(a, b);
        self_swap<32>(mx, a, b);  mx = vmax(a, b);
    }
}

// The value held by the neighbouring lane (lane ^ 1).
__device__ __forceinline__ float from_pair_lane(float v)
{
    return __builtin_bit_cast(float,
        __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), 0xB1, 0xF, 0xF, true));   // quad_perm [1,0,3,2]
}

// ---- Philox4x32-10 ---------------------------------------------------------------
// Salmon, Moraes, Dror, Shaw, "Parallel random numbers: as easy as 1, 2, 3" (SC'11),
// Section 3.3: ten rounds of
//   (c0,c1,c2,c3) <- (hi(M1*c2) ^ c1 ^ k0, lo(M1*c2), hi(M0*c0) ^ c3 ^ k1, lo(M0*c0)),
// the key advancing by the Weyl constants between rounds.  The key schedule is
// wave-uniform, so it lives in scalar registers.
__device__ __forceinline__ u32x4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                               uint32_t k0, uint32_t k1)
{
    constexpr uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;
    constexpr uint32_t W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint64_t p0 = (uint64_t)M0 * c0;
        const uint64_t p1 = (uint64_t)M1 * c2;
        // three-way xor in one v_bitop3_b32 (truth table 0x96)
        const uint32_t n0 = __builtin_amdgcn_bitop3_b32((uint32_t)(p1 >> 32), c1, k0, 0x96);
        const uint32_t n2 = __builtin_amdgcn_bitop3_b32((uint32_t)(p0 >> 32), c3, k1, 0x96);
        c1 = (uint32_t)p1;
        c3 = (uint32_t)p0;
        c0 = n0;
        c2 = n2;
        k0 += W0;
        k1 += W1;
    }
    return u32x4{c0, c1, c2, c3};
}

}  // namespace fh
