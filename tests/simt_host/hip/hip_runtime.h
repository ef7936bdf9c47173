// A stand-in for <hip/hip_runtime.h> that runs HIP kernels on the CPU, one workgroup at a time, one
// OS thread per work-item.  TEST INFRASTRUCTURE ONLY: it exists so that the index arithmetic of the
// library's decoders can be executed under AddressSanitizer on streams no encoder wrote (see
// test_decoder_bounds_host.py); nothing in the package builds against it or loads what is built with it.
//
// What it models: threadIdx / blockIdx / blockDim / gridDim, __shared__ (one copy: workgroups run one
// after the other), __syncthreads, atomics, and the wave-level operations the decoders use (__ballot,
// readlane, the row_shr / row_bcast data-parallel-primitive controls, mbcnt, the wavefront-scope fence) for waves of 64.  A
// wave-level exchange needs every lane of the wave that has not left the kernel to take part, as on
// the hardware when the wave is converged; readfirstlane is only used on wave-uniform values in the
// sources compiled here and returns its argument.
#pragma once

#include <atomic>
#include <barrier>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <memory>
#include <thread>
#include <vector>

struct dim3 {
    unsigned x, y, z;
    constexpr dim3(unsigned x_ = 1, unsigned y_ = 1, unsigned z_ = 1) : x(x_), y(y_), z(z_) {}
};

typedef void* hipStream_t;
enum hipError_t { hipSuccess = 0, hipErrorUnknown = 999 };
inline hipError_t hipGetLastError() { return hipSuccess; }

namespace simt {

struct Wave {
    std::barrier<> bar;
    uint64_t slot[64];
    bool here[64];                                            // lanes that exist in this wave
    explicit Wave(int lanes) : bar(lanes) { for (int i = 0; i < 64; ++i) { slot[i] = 0; here[i] = i < lanes; } }
};
struct Group {
    std::barrier<> bar;
    explicit Group(int threads) : bar(threads) {}
};
struct Ctx {
    dim3 thread, block, block_dim, grid_dim;
    Wave* wave = nullptr;
    Group* group = nullptr;
    unsigned lane = 0;
};
inline thread_local Ctx ctx;

// every lane publishes `v`, then reads the slot of lane `from(lane)` (or keeps `otherwise` when that is negative)
template <typename F>
inline uint64_t exchange(uint64_t v, uint64_t otherwise, F from)
{
    Wave& w = *ctx.wave;
    w.slot[ctx.lane] = v;
    w.bar.arrive_and_wait();
    const int src = from((int)ctx.lane);
    const uint64_t got = (src >= 0 && src < 64 && w.here[src]) ? w.slot[src] : otherwise;
    w.bar.arrive_and_wait();
    return got;
}

inline uint64_t ballot(bool p)
{
    Wave& w = *ctx.wave;
    w.slot[ctx.lane] = p ? 1u : 0u;
    w.bar.arrive_and_wait();
    uint64_t m = 0;
    for (int i = 0; i < 64; ++i) if (w.here[i] && w.slot[i]) m |= (uint64_t)1 << i;
    w.bar.arrive_and_wait();
    return m;
}

// __builtin_amdgcn_update_dpp for the controls used here: row_shr:1..15 (0x111..0x11f), row_bcast:15 (0x142),
// row_bcast:31 (0x143); bank mask 0xf.
inline int update_dpp(int old, int src, int ctrl, int row_mask, int /*bank_mask*/, bool bound_ctrl)
{
    const int lane = (int)ctx.lane, row = lane >> 4;
    const bool row_on = (row_mask >> row) & 1;
    const uint64_t keep = (uint64_t)(uint32_t)old;
    int source = -1;
    if (ctrl >= 0x111 && ctrl <= 0x11f) {
        const int n = ctrl - 0x110;
        source = (lane & 15) >= n ? lane - n : -1;
    } else if (ctrl == 0x142) {
        source = row >= 1 ? 16 * row - 1 : -1;
    } else if (ctrl == 0x143) {
        source = row >= 2 ? 31 : -1;
    } else {
        std::fprintf(stderr, "simt: data-parallel-primitive control 0x%x is not modelled\n", ctrl);
        std::abort();
    }
    const uint64_t got = exchange((uint64_t)(uint32_t)src, bound_ctrl ? 0u : keep, [&](int) { return source; });
    return row_on ? (int)(uint32_t)got : old;
}

inline int readlane(int v, int k) { return (int)(uint32_t)exchange((uint64_t)(uint32_t)v, 0u, [&](int) { return k; }); }

inline uint32_t mbcnt_lo(uint32_t mask, uint32_t acc)
{
    const unsigned l = ctx.lane;
    const uint32_t below = l >= 32 ? 0xffffffffu : ((1u << l) - 1u);
    return acc + (uint32_t)__builtin_popcount(mask & below);
}
inline uint32_t mbcnt_hi(uint32_t mask, uint32_t acc)
{
    const unsigned l = ctx.lane;
    const uint32_t below = l <= 32 ? 0u : (l >= 64 ? 0xffffffffu : ((1u << (l - 32)) - 1u));
    return acc + (uint32_t)__builtin_popcount(mask & below);
}

// One OS thread per work-item of a workgroup, reused for every workgroup of the launch; the workgroups run one
// after the other (there is one copy of each __shared__ variable).
template <typename Body>
inline void launch(dim3 grid, dim3 block, Body body)
{
    const unsigned threads = block.x, waves_per_group = (threads + 63u) / 64u;
    if (grid.x == 0 || threads == 0) return;
    std::vector<std::unique_ptr<Group>> groups;
    std::vector<std::unique_ptr<Wave>> waves;
    for (unsigned b = 0; b < grid.x; ++b) {
        groups.emplace_back(new Group((int)threads));
        for (unsigned t = 0; t < threads; t += 64) waves.emplace_back(new Wave((int)(threads - t < 64 ? threads - t : 64)));
    }
    std::barrier<> next_group((int)threads);
    std::vector<std::thread> pool;
    pool.reserve(threads);
    for (unsigned t = 0; t < threads; ++t) {
        pool.emplace_back([&, t] {
            for (unsigned b = 0; b < grid.x; ++b) {
                ctx.thread = dim3(t);
                ctx.block = dim3(b);
                ctx.block_dim = block;
                ctx.grid_dim = grid;
                ctx.wave = waves[b * waves_per_group + (t >> 6)].get();
                ctx.group = groups[b].get();
                ctx.lane = t & 63u;
                body();
                ctx.wave->bar.arrive_and_drop();              // a work-item that has left takes part in nothing further
                ctx.group->bar.arrive_and_drop();
                next_group.arrive_and_wait();
            }
        });
    }
    for (auto& th : pool) th.join();
}

template <typename T> inline T atomic_add(T* p, T v) { return __atomic_fetch_add(p, v, __ATOMIC_RELAXED); }
template <typename T> inline T atomic_max(T* p, T v)
{
    T seen = __atomic_load_n(p, __ATOMIC_RELAXED);
    while (seen < v && !__atomic_compare_exchange_n(p, &seen, v, true, __ATOMIC_RELAXED, __ATOMIC_RELAXED)) {}
    return seen;
}
template <typename T> inline T atomic_min(T* p, T v)
{
    T seen = __atomic_load_n(p, __ATOMIC_RELAXED);
    while (seen > v && !__atomic_compare_exchange_n(p, &seen, v, true, __ATOMIC_RELAXED, __ATOMIC_RELAXED)) {}
    return seen;
}

}  // namespace simt

#define __global__
#define __device__
#define __host__
#define __shared__ static
#define __forceinline__ inline
#define __launch_bounds__(...)
#define __align__(n) __attribute__((aligned(n)))

#define threadIdx (simt::ctx.thread)
#define blockIdx (simt::ctx.block)
#define blockDim (simt::ctx.block_dim)
#define gridDim (simt::ctx.grid_dim)

#define __syncthreads() (simt::ctx.group->bar.arrive_and_wait())
#define __ballot(p) (simt::ballot(p))
#define __builtin_amdgcn_ballot_w64(p) (simt::ballot(p))
#define __popcll(x) (__builtin_popcountll(x))
#define __popc(x) (__builtin_popcount(x))
#define __umulhi(a, b) ((uint32_t)(((uint64_t)(uint32_t)(a) * (uint64_t)(uint32_t)(b)) >> 32))
#define __builtin_amdgcn_readfirstlane(v) (v)
#define __builtin_amdgcn_readlane(v, k) (simt::readlane((v), (k)))
#define __builtin_amdgcn_update_dpp(old, src, ctrl, rm, bm, bc) (simt::update_dpp((old), (src), (ctrl), (rm), (bm), (bc)))
#define __builtin_amdgcn_mbcnt_lo(m, a) (simt::mbcnt_lo((m), (a)))
#define __builtin_amdgcn_mbcnt_hi(m, a) (simt::mbcnt_hi((m), (a)))
#define atomicAdd(p, v) (simt::atomic_add((p), (v)))
#define atomicMax(p, v) (simt::atomic_max((p), (v)))
#define atomicMin(p, v) (simt::atomic_min((p), (v)))
#define atomicOr(p, v) (__atomic_fetch_or((p), (v), __ATOMIC_RELAXED))
// where the sources rely on the LDS operations of one wave completing in order, they say so with a wavefront-scope
// fence in converged code: here, where the lanes are threads of their own, that is a barrier over the wave
#define __builtin_amdgcn_fence(order, scope) (simt::ctx.wave->bar.arrive_and_wait())

#define hipLaunchKernelGGL(kernel, grid, block, lds, stream, ...) \
    simt::launch((grid), (block), [&] { kernel(__VA_ARGS__); })
