// Sparse-block storage of salient-channel feature maps on gfx950 (paper Section 4.4.1: a
// binary non-zero mask is mean-filtered by n x n average pooling and compared with a
// threshold tau; sparse blocks are stored in Compressed Sparse Row format, dense blocks are
// kept as they are; zeros come back exactly).
//
// The pooling windows ("tiles" below, to keep them apart from GPU workgroups) are independent,
// and what each contributes to the two output streams is known from one byte of information,
// so the streams are laid out by a prefix sum over tiles -- stream compaction:
//   pass 1  one thread per tile: count non-zeros, decide sparse / dense, write the tile's info
//           byte; the tiles of a workgroup (256, or 128 for the largest window) form a group,
//           whose sums are added up;
//   pass 2  one thread per tile: the group's base is the sum of the sums before it (each
//           workgroup adds them up itself while there are few; a scan kernel in between does
//           it once there are many), offsets inside the group come from a scan over the
//           workgroup, then the tile's values and CSR structure go to their final place.
// What a workgroup's tiles write is one contiguous slice of each stream, so the threads put
// their pieces together in LDS and the workgroup moves the slice with aligned 16-byte
// vectors (thread-per-tile stores would touch every cache line of the slice once per element).
// Restoring runs the same passes with the info bytes as the only input of pass 1; the slices
// come into LDS the same way and every thread rebuilds its tile from there.
// A thread reads its whole tile with unconditional loads (addresses clamped into the tile) before
// it looks at any value, so it waits for memory once, not once per element.
// With an error bound, dense blocks are stored by first-order Lorenzo prediction on the lattice
// of step 2*eps (same section: prediction from decompressed neighbours, errors within the bound
// quantised to a byte, outliers kept intact) instead of verbatim; a thread runs the recurrence
// of its block in registers.
// Apart from one division and one multiplication per element in that mode, everything here is
// integer and byte work; results do not depend on launch geometry.
#include "../../include/fedhybrid.h"

#include "fh_batch.hpp"
#include "fh_channels.hpp"
#include "fh_scan.hpp"

namespace fh {
namespace {

// tiles (threads) per workgroup: fewer for the largest window, whose slices are four times as long
template <int N> struct Group {
    static constexpr int kTiles = N == 8 ? 128 : 256;
    static constexpr int kWaves = kTiles / 64;
};
constexpr int kMaxWaves = 4;
constexpr int kScanThreads = 512;
constexpr uint64_t kStreamedFrom = (uint64_t)128 << 20;    // bytes of maps in a launch from which the first pass streams
constexpr uint32_t kSelfScanLimit = 2048;          // up to this many workgroups each adds up the sums before it

struct Sums {                                      // what a run of tiles writes
    uint64_t values, index_bytes, sparse_tiles;
};
__device__ __forceinline__ Sums operator+(const Sums& a, const Sums& b)
{
    return Sums{a.values + b.values, a.index_bytes + b.index_bytes, a.sparse_tiles + b.sparse_tiles};
}

struct MapShape {
    const void* x;             // [maps][h][w] (encode: input; decode: output)
    uint32_t h, w, n;
    uint32_t tiles;            // maps * BH * BW
    ExactDiv bw, bh;           // tile index -> (map, tile row, tile column)
    uint32_t BW, BH;
    float two_eps;             // lattice step of the predictive form of dense tiles; 0 = verbatim
    uint32_t rows_are_vectors; // w is a multiple of n and the maps are 16-byte aligned: a tile row is one
                               // aligned vector of n elements (every tile is n wide)
};

struct TilePos {
    uint64_t origin;           // element index of the tile's first element
    uint32_t rows, cols;
};
__device__ __forceinline__ TilePos tile_pos(const MapShape& s, uint32_t b)
{
    const uint32_t row_of_tiles = div_exact(b, s.bw);         // m * BH + bi
    const uint32_t bj = b - row_of_tiles * s.BW;
    const uint32_t m = div_exact(row_of_tiles, s.bh);
    const uint32_t bi = row_of_tiles - m * s.BH;
    const uint32_t r0 = bi * s.n, c0 = bj * s.n;
    TilePos t;
    t.rows = s.h - r0 < s.n ? s.h - r0 : s.n;
    t.cols = s.w - c0 < s.n ? s.w - c0 : s.n;
    t.origin = ((uint64_t)m * s.h + r0) * s.w + c0;
    return t;
}

// One set of maps in a launch (fh_batch.hpp: a launch serves up to kBatch of them).
struct Job {
    MapShape  shape;           // x: the maps (encode: input; decode: output)
    uint8_t*  info;            // one byte per tile (encode: written; decode: read)
    Sums*     wg;              // per-workgroup sums, or their exclusive prefixes once `scanned`
    void*     values;          // the two streams (encode: written; decode: read)
    uint8_t*  indices;
    uint64_t* totals;          // encode: {values, index bytes, sparse tiles, dense tiles}; may be null
    uint64_t  value_count;     // decode: valid prefix of the streams
    uint64_t  index_count;
    float     tau;
    uint32_t  scanned;         // this set has so many workgroups that a scan kernel runs between the passes
    uint32_t  wg_count;
};

// what a tile with this info byte adds to the streams
__device__ __forceinline__ Sums tile_sums(uint32_t info, const TilePos& t, bool predictive)
{
    // non-zeros | elements | outliers: never more than the tile has (an encoder cannot write more; a foreign byte
    // that claims more must not make a workgroup's slice outgrow its staging area)
    const uint32_t claimed = info & 0x7fu, room = t.rows * t.cols;
    const uint32_t count = claimed < room ? claimed : room;
    if (info & 0x80u) return Sums{count, predictive ? t.rows * t.cols : 0u, 0u};
    return Sums{count, t.rows + 1u + count, 1u};
}

template <typename T> __device__ __forceinline__ uint32_t bits_of(T v);
template <> __device__ __forceinline__ uint32_t bits_of<uint32_t>(uint32_t v) { return v; }
template <> __device__ __forceinline__ uint32_t bits_of<uint16_t>(uint16_t v) { return v; }

// ---- the predictive form of a dense tile -----------------------------------------------------
template <typename Bits> __device__ __forceinline__ float value_of(Bits b);
template <> __device__ __forceinline__ float value_of<uint32_t>(uint32_t b) { return __builtin_bit_cast(float, b); }
template <> __device__ __forceinline__ float value_of<uint16_t>(uint16_t b) { return __builtin_bit_cast(float, (uint32_t)b << 16); }
template <typename Bits> __device__ __forceinline__ Bits stored_of(float f);
template <> __device__ __forceinline__ uint32_t stored_of<uint32_t>(float f) { return __builtin_bit_cast(uint32_t, f); }
template <> __device__ __forceinline__ uint16_t stored_of<uint16_t>(float f) { return (uint16_t)bf16_bits(f); }

// the lattice point of x (0 when it has none) and whether it has one
__device__ __forceinline__ int32_t lattice(float x, float two_eps, bool& ok)
{
    const float t = x / two_eps;                              // IEEE division
    ok = __builtin_fabsf(t) < 0x1p22f;                        // false for NaN and infinities
    return ok ? (int32_t)__builtin_rintf(t) : 0;
}

// Code bytes of a tile (0 = outlier) and the number of outliers; elements outside the tile
// (zero padding) are never counted.  q(r,c) is predicted by q(r,c-1) + q(r-1,c) - q(r-1,c-1)
// with zeros outside the tile.
template <typename Bits, int N>
__device__ __forceinline__ uint32_t lorenzo_codes(const Bits (&e)[N][N], const TilePos& t, float two_eps,
                                                  uint8_t (&code)[N][N])
{
    int32_t q[N][N];
    uint32_t outliers = 0;
#pragma unroll
    for (int r = 0; r < N; ++r) {
#pragma unroll
        for (int c = 0; c < N; ++c) {
            bool ok;
            q[r][c] = lattice(value_of<Bits>(e[r][c]), two_eps, ok);
            const int32_t left = c > 0 ? q[r][c - 1] : 0, up = r > 0 ? q[r - 1][c] : 0;
            const int32_t diag = (r > 0 && c > 0) ? q[r - 1][c - 1] : 0;
            const int32_t d = q[r][c] - (left + up - diag);
            const bool coded = ok && d > -128 && d < 128;
            code[r][c] = coded ? (uint8_t)(d + 128) : (uint8_t)0;
            if (!coded && r < (int)t.rows && c < (int)t.cols) ++outliers;
        }
    }
    return outliers;
}

// ---- sums over a wave and a workgroup -----------------------------------------------------------
// Inside a wave every running sum here stays below 2^32 (a wave covers at most 64 groups of
// 256 tiles, a tile writes at most 127 values and 73 index bytes), so lanes scan three 32-bit
// words with data-parallel-primitive adds on the vector ALU: four shifts inside each row of 16
// lanes, then the last lane of rows 0 and 2 onto rows 1 and 3, then lane 31 onto rows 2 and 3.
// Across waves and workgroups the sums are 64 bits wide and meet in LDS.
struct Sums32 {
    uint32_t values, index_bytes, sparse_tiles;
};
__device__ __forceinline__ Sums32 narrow(const Sums& s)
{
    return Sums32{(uint32_t)s.values, (uint32_t)s.index_bytes, (uint32_t)s.sparse_tiles};
}

__device__ __forceinline__ Sums32 wave_inclusive_scans(const Sums32& s)
{
    return Sums32{wave_inclusive_scan(s.values), wave_inclusive_scan(s.index_bytes), wave_inclusive_scan(s.sparse_tiles)};
}
// the wave's total, from the inclusive sums: lane 63's, in scalar registers
__device__ __forceinline__ Sums wave_total(const Sums32& inclusive)
{
    return Sums{(uint32_t)__builtin_amdgcn_readlane((int)inclusive.values, 63),
                (uint32_t)__builtin_amdgcn_readlane((int)inclusive.index_bytes, 63),
                (uint32_t)__builtin_amdgcn_readlane((int)inclusive.sparse_tiles, 63)};
}

// the waves' totals through LDS: what the waves before this one add up to, and all of them
template <int WAVES>
__device__ __forceinline__ Sums across_waves(const Sums& wave_sum, uint64_t* lds /* [3 * WAVES] */, Sums* all)
{
    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    if (lane == 0u) { lds[3 * wave] = wave_sum.values; lds[3 * wave + 1] = wave_sum.index_bytes; lds[3 * wave + 2] = wave_sum.sparse_tiles; }
    __syncthreads();
    Sums before = {0, 0, 0}, total = {0, 0, 0};
#pragma unroll
    for (int v = 0; v < WAVES; ++v) {
        const Sums w = {lds[3 * v], lds[3 * v + 1], lds[3 * v + 2]};
        if ((uint32_t)v < wave) before = before + w;
        total = total + w;
    }
    __syncthreads();                                          // lds may be reused right away
    *all = total;
    return before;
}

// Workgroup-wide exclusive scan of what each thread's tile writes.
template <int WAVES>
__device__ __forceinline__ Sums workgroup_exclusive_scan(Sums mine, uint64_t* lds /* [3 * WAVES] */, Sums* total)
{
    const Sums32 own = narrow(mine), inc = wave_inclusive_scans(own);
    const Sums before = across_waves<WAVES>(wave_total(inc), lds, total);
    return Sums{before.values + inc.values - own.values, before.index_bytes + inc.index_bytes - own.index_bytes,
                before.sparse_tiles + inc.sparse_tiles - own.sparse_tiles};
}

// Workgroup-wide sum; a thread's part is below 2^32 / 64.
template <int WAVES>
__device__ __forceinline__ Sums workgroup_sum(Sums part, uint64_t* lds /* [3 * WAVES] */)
{
    Sums total;
    across_waves<WAVES>(wave_total(wave_inclusive_scans(narrow(part))), lds, &total);
    return total;
}

// The tile's elements, row-major, zeros where the tile has no element.  Every load is
// unconditional -- out-of-tile positions read a clamped in-tile address -- so all N*N loads
// are in flight together.  Plain loads by default: the second pass over the maps finds in the
// memory-side cache what the first one read whenever a layer's kept channels fit there.  STREAM:
// non-temporal loads, for the first pass over sets that fit no cache (measured on 371 MB of maps:
// 68 us against 98 us with plain loads; on 23 MB plain loads are the faster by 5 %).
// N elements of Bits as one vector.  A row of a tile is known to be 16-byte aligned at most (the maps are, and a
// row is a multiple of 16 bytes), so the 32-byte vector of eight fp32 elements must not claim 32.
template <typename Bits, int N> struct RowVec {
    typedef Bits full __attribute__((ext_vector_type(N)));
    typedef full type __attribute__((aligned(sizeof(full) < 16 ? sizeof(full) : 16)));
};

template <typename Bits, int N, bool STREAM = false>
__device__ __forceinline__ void load_tile(const Bits* x, const TilePos& t, uint32_t w, bool rows_are_vectors,
                                          Bits (&e)[N][N])
{
    if (rows_are_vectors) {                                   // wave-uniform
        typedef typename RowVec<Bits, N>::type vec;
#pragma unroll
        for (int r = 0; r < N; ++r) {
            const uint32_t rr = r < (int)t.rows ? r : t.rows - 1;
            const vec* p = reinterpret_cast<const vec*>(x + (uint64_t)rr * w);
            const vec v = STREAM ? __builtin_nontemporal_load(p) : *p;
#pragma unroll
            for (int c = 0; c < N; ++c) e[r][c] = r < (int)t.rows ? v[c] : (Bits)0;
        }
        return;
    }
#pragma unroll
    for (int r = 0; r < N; ++r) {
        const uint32_t rr = r < (int)t.rows ? r : t.rows - 1;
#pragma unroll
        for (int c = 0; c < N; ++c) {
            const uint32_t cc = c < (int)t.cols ? c : t.cols - 1;
            e[r][c] = x[(uint64_t)rr * w + cc];
        }
    }
#pragma unroll
    for (int r = 0; r < N; ++r)
#pragma unroll
        for (int c = 0; c < N; ++c)
            if (!(r < (int)t.rows && c < (int)t.cols)) e[r][c] = (Bits)0;
}

// The tile back to the map (only elements that exist).
template <typename Bits, int N>
__device__ __forceinline__ void store_tile(Bits* out, const TilePos& t, uint32_t w, bool rows_are_vectors,
                                           const Bits (&e)[N][N])
{
    if (rows_are_vectors) {
        typedef typename RowVec<Bits, N>::type vec;
#pragma unroll
        for (int r = 0; r < N; ++r) {
            if (r < (int)t.rows) {
                vec v;
#pragma unroll
                for (int c = 0; c < N; ++c) v[c] = e[r][c];
                __builtin_nontemporal_store(v, reinterpret_cast<vec*>(out + (uint64_t)r * w));   // read by no kernel of this library
            }
        }
        return;
    }
#pragma unroll
    for (int r = 0; r < N; ++r)
#pragma unroll
        for (int c = 0; c < N; ++c)
            if (r < (int)t.rows && c < (int)t.cols) out[(uint64_t)r * w + c] = e[r][c];
}

// What the tiles of all earlier workgroups write.  `scanned`: wg[] already holds exclusive
// prefixes (the scan kernel ran); otherwise it holds per-workgroup sums and they are added up
// here, a workgroup's width at a time.
template <int WAVES>
__device__ __forceinline__ Sums workgroup_base(const Sums* __restrict__ wg, bool scanned, uint32_t block,
                                               uint64_t* lds)
{
    if (scanned) return wg[block];
    Sums part = {0, 0, 0};
    for (uint32_t i = threadIdx.x; i < block; i += WAVES * 64) part = part + wg[i];
    return workgroup_sum<WAVES>(part, lds);
}

// ---- a workgroup's slice of a stream, staged in LDS --------------------------------------------
// Byte i of the slice sits at stage[phase + i], phase = the slice's address mod 16, so 16-byte
// chunks of LDS and of the stream line up: whole chunks move as one vector per thread, the
// (at most 15 + 15) bytes before the first and after the last whole chunk byte by byte.
// Neighbouring workgroups' slices may share a chunk; each writes only its own bytes of it.
typedef uint32_t chunk16 __attribute__((ext_vector_type(4), may_alias));
template <typename T> struct Alias { typedef T __attribute__((may_alias)) type; };

__device__ __forceinline__ uint32_t phase_of(const void* p) { return (uint32_t)(reinterpret_cast<uintptr_t>(p) & 15u); }

template <int THREADS>
__device__ __forceinline__ void stage_to_stream(const uint8_t* stage, uint8_t* dst, uint32_t nbytes)
{
    const uint32_t phase = phase_of(dst), end = phase + nbytes;
    uint8_t* g0 = dst - phase;                                // 16-byte aligned
    const uint32_t first = (phase + 15u) >> 4, last = end >> 4;       // whole chunks [first, last)
    for (uint32_t c = first + threadIdx.x; c < last; c += THREADS)
        *reinterpret_cast<chunk16*>(g0 + 16u * c) = *reinterpret_cast<const chunk16*>(stage + 16u * c);
    const uint32_t head_end = first * 16u < end ? first * 16u : end;
    const uint32_t tail = last * 16u > head_end ? last * 16u : head_end;
    uint32_t i = phase + threadIdx.x;
    if (i < head_end) g0[i] = stage[i];
    i = tail + threadIdx.x;
    if (i < end) g0[i] = stage[i];
}

// A slice of a stream into LDS, in two steps so that the loads of both slices of a workgroup are requested before
// the first of them is waited for: `request` asks for a thread's first K whole vectors and for the bytes before the
// first and after the last whole vector, `commit` puts them into the stage and brings what is left K vectors at a
// time.  (A loop of load, wait, LDS store costs one memory latency per iteration: up to ten in a row for the two
// slices, 157 -> 137 us for the decode of 0.37 GB of maps.)
template <int K> struct SliceLoads {
    chunk16 got[K];
    uint8_t head_byte, tail_byte;
};
struct SliceShape {
    const uint8_t* g0;                             // the 16-byte boundary at or below the slice's first byte
    uint32_t phase, end, first, last, head_end, tail;   // bytes [phase, end) from g0; whole vectors [first, last)
};
__device__ __forceinline__ SliceShape slice_shape(const uint8_t* src, uint32_t nbytes)
{
    SliceShape s;
    s.phase = phase_of(src);
    s.end = s.phase + nbytes;
    s.g0 = src - s.phase;
    s.first = (s.phase + 15u) >> 4;
    s.last = s.end >> 4;
    s.head_end = s.first * 16u < s.end ? s.first * 16u : s.end;
    s.tail = s.last * 16u > s.head_end ? s.last * 16u : s.head_end;
    return s;
}
template <int THREADS, int K>
__device__ __forceinline__ void slice_request(SliceLoads<K>& l, const uint8_t* src, uint32_t nbytes)
{
    const SliceShape s = slice_shape(src, nbytes);
    const uint32_t ih = s.phase + threadIdx.x, it = s.tail + threadIdx.x;
    l.head_byte = l.tail_byte = 0;
    if (ih < s.head_end) l.head_byte = s.g0[ih];
    if (it < s.end) l.tail_byte = s.g0[it];
#pragma unroll
    for (int k = 0; k < K; ++k) {
        const uint32_t c = s.first + threadIdx.x + k * THREADS;
        l.got[k] = chunk16{0u, 0u, 0u, 0u};
        if (c < s.last) l.got[k] = *reinterpret_cast<const chunk16*>(s.g0 + 16u * c);
    }
}
template <int THREADS, int K>
__device__ __forceinline__ void slice_commit(const SliceLoads<K>& l, uint8_t* stage, const uint8_t* src, uint32_t nbytes)
{
    const SliceShape s = slice_shape(src, nbytes);
    const uint32_t ih = s.phase + threadIdx.x, it = s.tail + threadIdx.x;
#pragma unroll
    for (int k = 0; k < K; ++k) {
        const uint32_t c = s.first + threadIdx.x + k * THREADS;
        if (c < s.last) *reinterpret_cast<chunk16*>(stage + 16u * c) = l.got[k];
    }
    if (ih < s.head_end) stage[ih] = l.head_byte;
    if (it < s.end) stage[it] = l.tail_byte;
    for (uint32_t c0 = s.first + threadIdx.x + K * THREADS; c0 < s.last; c0 += K * THREADS) {
        chunk16 more[K];
#pragma unroll
        for (int k = 0; k < K; ++k) {
            const uint32_t c = c0 + k * THREADS;
            more[k] = chunk16{0u, 0u, 0u, 0u};
            if (c < s.last) more[k] = *reinterpret_cast<const chunk16*>(s.g0 + 16u * c);
        }
#pragma unroll
        for (int k = 0; k < K; ++k) {
            const uint32_t c = c0 + k * THREADS;
            if (c < s.last) *reinterpret_cast<chunk16*>(stage + 16u * c) = more[k];
        }
    }
}

// LDS of a workgroup: a tile puts at most N*N values and N*N + N + 1 index bytes into the streams
// (a sparse tile whose every element is a non-zero: tau >= 1).  16 bytes for the phase; the
// decoder may read up to N bytes / one value past a tile's piece (and discards them).
template <typename Bits, int N> struct Stage {
    static constexpr int kValueBytes = Group<N>::kTiles * N * N * (int)sizeof(Bits) + 32;
    static constexpr int kIndexBytes = Group<N>::kTiles * (N * N + N + 1) + 32;
};

// occupancy of a tile, bit r*N + c for element (r, c)
template <int N> struct TileMask { typedef uint32_t type; };
template <> struct TileMask<8> { typedef uint64_t type; };
__device__ __forceinline__ uint32_t popcount(uint32_t m) { return (uint32_t)__builtin_popcount(m); }
__device__ __forceinline__ uint32_t popcount(uint64_t m) { return (uint32_t)__builtin_popcountll(m); }

// the elements a tile has (edge tiles are smaller than the window)
template <int N>
__device__ __forceinline__ typename TileMask<N>::type valid_mask(const TilePos& t)
{
    typedef typename TileMask<N>::type M;
    const uint32_t row = (1u << t.cols) - 1u;
    M m = 0;
#pragma unroll
    for (int r = 0; r < N; ++r)
        if (r < (int)t.rows) m |= (M)row << (r * N);
    return m;
}

// The occupancy a sparse tile's CSR structure describes: row r owns entries
// [row_ptr[r], row_ptr[r+1]), their column bytes ascending (as the encoder writes them), so
// entry k is the k-th set bit.  Bytes that do not describe a tile (a foreign stream) yield some
// mask; nothing outside the tile's piece plus N bytes is read.
template <int N>
__device__ __forceinline__ typename TileMask<N>::type csr_mask(const uint8_t* si, const TilePos& t, uint32_t count)
{
    typedef typename TileMask<N>::type M;
    uint32_t rp[N + 1];
#pragma unroll
    for (int r = 0; r <= N; ++r) rp[r] = si[r <= (int)t.rows ? r : t.rows];
    const uint8_t* col = si + t.rows + 1;
    M m = 0;
#pragma unroll
    for (int r = 0; r < N; ++r) {
        const uint32_t start = rp[r] < count ? rp[r] : count;
        const uint32_t len = rp[r + 1] > rp[r] ? rp[r + 1] - rp[r] : 0u;
        uint32_t cols[N];
#pragma unroll
        for (int j = 0; j < N; ++j) cols[j] = col[start + j];
        uint32_t row = 0;
#pragma unroll
        for (int j = 0; j < N; ++j)
            if ((uint32_t)j < len && start + j < count && cols[j] < t.cols) row |= 1u << cols[j];
        if (r < (int)t.rows) m |= (M)row << (r * N);
    }
    return m;
}

// ---- pass 1: what each group of tiles (a workgroup of pass 3) will write -------------------------
constexpr int kGroupsPerWorkgroup = 4;             // decode: waves of a pass-1 workgroup, a group each

// encode: non-zero count, density, info byte; one thread per tile, one workgroup per group.  (A wave per group with
// four tiles of a lane in flight and no barrier was measured: 7 % slower on 371 MB of maps, 35 % slower on 23 MB,
// where it leaves too few waves.)
template <typename Bits, int N, bool STREAM>
__global__ __launch_bounds__(Group<N>::kTiles) void sparse_count_kernel(const Batch<Job> batch)
{
    constexpr int T = Group<N>::kTiles, WAVES = Group<N>::kWaves;
    __shared__ uint64_t lds[3 * kMaxWaves];
    uint32_t block;
    const Job& job = batch.item[batch_item(batch, blockIdx.x, block)];
    const MapShape& s = job.shape;
    const float tau = job.tau;
    uint8_t* info = job.info;
    const uint32_t b = block * T + threadIdx.x;
    Sums mine = {0, 0, 0};
    if (b < s.tiles) {
        const TilePos t = tile_pos(s, b);
        Bits e[N][N];
        load_tile<Bits, N, STREAM>(static_cast<const Bits*>(s.x) + t.origin, t, s.w, s.rows_are_vectors != 0u, e);
        uint32_t nnz = 0;
#pragma unroll
        for (int r = 0; r < N; ++r)
#pragma unroll
            for (int c = 0; c < N; ++c) nnz += bits_of<Bits>(e[r][c]) != 0u ? 1u : 0u;   // padding is zero
        const uint32_t area = t.rows * t.cols;
        const float density = (float)nnz / (float)area;       // IEEE division: average pooling of the mask
        uint32_t byte = density <= tau ? nnz : (0x80u | area);
        if ((byte & 0x80u) && s.two_eps > 0.0f) {             // dense, within the error bound: count the outliers
            uint8_t code[N][N];
            byte = 0x80u | lorenzo_codes<Bits, N>(e, t, s.two_eps, code);
        }
        info[b] = (uint8_t)byte;
        mine = tile_sums(byte, t, s.two_eps > 0.0f);
    }
    const Sums total = workgroup_sum<WAVES>(mine, lds);
    if (threadIdx.x == 0) job.wg[block] = total;
}

// decode: the same sums from the info bytes.  A wave owns a group: a lane takes the tiles lane,
// lane + 64, ... of it and the group's sums are a wave reduction with no barrier.
template <int N>
__global__ __launch_bounds__(64 * kGroupsPerWorkgroup) void sparse_sums_kernel(const Batch<Job> batch)
{
    constexpr int T = Group<N>::kTiles, PER_LANE = T / 64;
    uint32_t block;
    const Job& job = batch.item[batch_item(batch, blockIdx.x, block)];
    const MapShape& s = job.shape;
    const uint32_t lane = threadIdx.x & 63u, group = block * kGroupsPerWorkgroup + (threadIdx.x >> 6);
    if (group >= job.wg_count) return;
    uint32_t byte[PER_LANE];
#pragma unroll
    for (int j = 0; j < PER_LANE; ++j) {
        const uint32_t b = group * T + j * 64 + lane;
        byte[j] = job.info[b < s.tiles ? b : s.tiles - 1u];
    }
    Sums mine = {0, 0, 0};
#pragma unroll
    for (int j = 0; j < PER_LANE; ++j) {
        const uint32_t b = group * T + j * 64 + lane;
        if (b < s.tiles) mine = mine + tile_sums(byte[j], tile_pos(s, b), s.two_eps > 0.0f);
    }
    const Sums total = wave_total(wave_inclusive_scans(narrow(mine)));
    if (lane == 0u) job.wg[group] = total;
}

// ---- pass 2: exclusive scan of the group sums, in place; totals -----------------------------------
// One workgroup per set; sets with few groups skip it (pass 3 adds up the sums itself).  A
// round covers kScanRows rows of kScanThreads consecutive groups, thread t taking the t-th
// group of every row (contiguous loads and stores; the next round's loads are in flight while
// this one is scanned).  Each row is scanned inside the waves; the (row, wave) totals of the
// round -- 32 numbers per field, still below 2^32 together -- are scanned by the first wave
// in row-major order and handed back through LDS; a 64-bit carry links the rounds.
constexpr int kScanRows = 4;

__global__ __launch_bounds__(kScanThreads) void sparse_scan_kernel(const Batch<Job> batch)
{
    constexpr int WAVES = kScanThreads / 64, CELLS = kScanRows * WAVES;
    constexpr uint32_t ROUND = kScanThreads * kScanRows;
    static_assert(CELLS < 64, "one wave scans a round's (row, wave) totals");
    const Job& job = batch.item[blockIdx.x];
    if (!job.scanned) return;                                 // workgroup-uniform
    Sums* wg_sums = job.wg;
    const uint32_t count = job.wg_count, tiles = job.shape.tiles;
    __shared__ Sums32 cell_total[CELLS];                      // inclusive end of wave w's part of row j, at [j * WAVES + w]
    __shared__ Sums32 cell_before[CELLS + 1];                 // what precedes a cell in its round; [CELLS]: the whole round
    const uint32_t t = threadIdx.x, lane = t & 63u, wave = t >> 6;
    Sums carry = {0, 0, 0};
    Sums next[kScanRows];
#pragma unroll
    for (int j = 0; j < kScanRows; ++j) {
        const uint32_t i = j * kScanThreads + t;
        next[j] = i < count ? wg_sums[i] : Sums{0, 0, 0};
    }
#pragma nounroll
    for (uint32_t base = 0; base < count; base += ROUND) {    // workgroup-uniform trip count
        Sums32 own[kScanRows], inc[kScanRows];
#pragma unroll
        for (int j = 0; j < kScanRows; ++j) {
            const uint32_t i = base + ROUND + j * kScanThreads + t;
            own[j] = narrow(next[j]);
            next[j] = i < count ? wg_sums[i] : Sums{0, 0, 0};
        }
#pragma unroll
        for (int j = 0; j < kScanRows; ++j) {
            inc[j] = wave_inclusive_scans(own[j]);
            if (lane == 63u) cell_total[j * WAVES + wave] = inc[j];
        }
        __syncthreads();
        if (wave == 0u) {
            const Sums32 mine = lane < (uint32_t)CELLS ? cell_total[lane] : Sums32{0, 0, 0};
            const Sums32 upto = wave_inclusive_scans(mine);
            if (lane < (uint32_t)CELLS)
                cell_before[lane] = Sums32{upto.values - mine.values, upto.index_bytes - mine.index_bytes,
                                           upto.sparse_tiles - mine.sparse_tiles};
            if (lane == (uint32_t)CELLS - 1u) cell_before[CELLS] = upto;
        }
        __syncthreads();
#pragma unroll
        for (int j = 0; j < kScanRows; ++j) {
            const uint32_t i = base + j * kScanThreads + t;
            const Sums32 before = cell_before[j * WAVES + wave];
            if (i < count)
                wg_sums[i] = Sums{carry.values + before.values + inc[j].values - own[j].values,
                                  carry.index_bytes + before.index_bytes + inc[j].index_bytes - own[j].index_bytes,
                                  carry.sparse_tiles + before.sparse_tiles + inc[j].sparse_tiles - own[j].sparse_tiles};
        }
        const Sums32 round = cell_before[CELLS];
        carry = carry + Sums{round.values, round.index_bytes, round.sparse_tiles};
    }
    uint64_t* totals = job.totals;
    if (t == 0 && totals) {
        totals[0] = carry.values;
        totals[1] = carry.index_bytes;
        totals[2] = carry.sparse_tiles;
        totals[3] = (uint64_t)tiles - carry.sparse_tiles;
    }
}

// ---- pass 3 (encode): values and CSR structure to their place ---------------------------------------
template <typename Bits, int N, bool STREAM>
__global__ __launch_bounds__(Group<N>::kTiles) void sparse_write_kernel(const Batch<Job> batch)
{
    constexpr int T = Group<N>::kTiles, WAVES = Group<N>::kWaves;
    typedef typename Alias<Bits>::type StagedBits;
    __shared__ uint64_t lds[3 * kMaxWaves];
    __shared__ __attribute__((aligned(16))) uint8_t stage_v[Stage<Bits, N>::kValueBytes];
    __shared__ __attribute__((aligned(16))) uint8_t stage_i[Stage<Bits, N>::kIndexBytes];
    uint32_t block;
    const Job& job = batch.item[batch_item(batch, blockIdx.x, block)];
    const MapShape& s = job.shape;
    const uint8_t* info = job.info;
    const Sums* wg = job.wg;
    const bool scanned = job.scanned != 0u;
    uint64_t* totals = job.totals;
    const uint32_t b = block * T + threadIdx.x;
    const bool live = b < s.tiles;
    TilePos t = {0, 1, 1};
    uint32_t byte = 0x80u;
    Sums mine = {0, 0, 0};
    Bits e[N][N];
    if (live) {
        t = tile_pos(s, b);
        byte = info[b];
        mine = tile_sums(byte, t, s.two_eps > 0.0f);
        load_tile<Bits, N, STREAM>(static_cast<const Bits*>(s.x) + t.origin, t, s.w, s.rows_are_vectors != 0u, e);
    }
    const Sums base = workgroup_base<WAVES>(wg, scanned, block, lds);
    Sums total;
    const Sums before = workgroup_exclusive_scan<WAVES>(mine, lds, &total);
    if (!scanned && totals && block == job.wg_count - 1 && threadIdx.x == 0) {
        totals[0] = base.values + total.values;
        totals[1] = base.index_bytes + total.index_bytes;
        totals[2] = base.sparse_tiles + total.sparse_tiles;
        totals[3] = (uint64_t)s.tiles - totals[2];
    }
    // this workgroup's slices of the two streams
    Bits* value_slice = static_cast<Bits*>(job.values) + base.values;
    uint8_t* index_slice = job.indices + base.index_bytes;
    if (live) {
        StagedBits* v = reinterpret_cast<StagedBits*>(stage_v + phase_of(value_slice)) + before.values;
        uint8_t* idx = stage_i + phase_of(index_slice) + before.index_bytes;
        if ((byte & 0x80u) && s.two_eps > 0.0f) {             // dense, predictive: code bytes + outliers
            uint8_t code[N][N];
            lorenzo_codes<Bits, N>(e, t, s.two_eps, code);
            uint32_t k = 0;
#pragma unroll
            for (int r = 0; r < N; ++r)
#pragma unroll
                for (int c = 0; c < N; ++c)
                    if (r < (int)t.rows && c < (int)t.cols) {
                        idx[r * t.cols + c] = code[r][c];
                        if (code[r][c] == 0) v[k++] = e[r][c];
                    }
        } else if (byte & 0x80u) {                            // dense: the tile, row-major
#pragma unroll
            for (int r = 0; r < N; ++r)
#pragma unroll
                for (int c = 0; c < N; ++c)
                    if (r < (int)t.rows && c < (int)t.cols) v[r * t.cols + c] = e[r][c];
        } else {                                              // sparse: row_ptr, then columns; values alongside
            uint8_t* col = idx + t.rows + 1;
            uint32_t k = 0;
#pragma unroll
            for (int r = 0; r < N; ++r) {
                if (r <= (int)t.rows) idx[r] = (uint8_t)k;    // r == rows: the closing entry
#pragma unroll
                for (int c = 0; c < N; ++c) {
                    if (bits_of<Bits>(e[r][c]) != 0u) {       // padding is zero, so it never gets here
                        v[k] = e[r][c];
                        col[k] = (uint8_t)c;
                        ++k;
                    }
                }
            }
            if ((int)t.rows == N) idx[N] = (uint8_t)k;
        }
    }
    __syncthreads();
    stage_to_stream<T>(stage_v, reinterpret_cast<uint8_t*>(value_slice), (uint32_t)total.values * (uint32_t)sizeof(Bits));
    stage_to_stream<T>(stage_i, index_slice, (uint32_t)total.index_bytes);
}

// ---- pass 3 (decode): tiles back from the streams -------------------------------------------------
// A stream this library did not write must not make the kernel read or write out of bounds:
// only the part of a slice that lies inside the stream is staged, a tile whose piece would
// leave the stream is zero-filled, and whatever the staged bytes say, a thread reads no further
// than N bytes / one value past its own piece.
template <typename Bits, int N>
__global__ __launch_bounds__(Group<N>::kTiles) void sparse_read_kernel(const Batch<Job> batch)
{
    constexpr int T = Group<N>::kTiles, WAVES = Group<N>::kWaves;
    typedef typename Alias<Bits>::type StagedBits;
    typedef typename TileMask<N>::type Mask;
    __shared__ uint64_t lds[3 * kMaxWaves];
    __shared__ __attribute__((aligned(16))) uint8_t stage_v[Stage<Bits, N>::kValueBytes];
    __shared__ __attribute__((aligned(16))) uint8_t stage_i[Stage<Bits, N>::kIndexBytes];
    uint32_t block;
    const Job& job = batch.item[batch_item(batch, blockIdx.x, block)];
    const MapShape& s = job.shape;
    const uint8_t* info = job.info;
    const Sums* wg = job.wg;
    const bool scanned = job.scanned != 0u;
    const uint64_t value_count = job.value_count, index_count = job.index_count;
    const uint32_t b = block * T + threadIdx.x;
    const bool live = b < s.tiles;
    TilePos t = {0, 1, 1};
    uint32_t byte = 0x80u;
    Sums mine = {0, 0, 0};
    if (live) {
        t = tile_pos(s, b);
        byte = info[b];
        mine = tile_sums(byte, t, s.two_eps > 0.0f);
    }
    const Sums base = workgroup_base<WAVES>(wg, scanned, block, lds);
    Sums total;
    const Sums before = workgroup_exclusive_scan<WAVES>(mine, lds, &total);

    // what the streams hold of this workgroup's slices
    const Bits* value_slice = static_cast<const Bits*>(job.values) + base.values;
    const uint8_t* index_slice = job.indices + base.index_bytes;
    uint64_t have_v = base.values < value_count ? value_count - base.values : 0u;
    uint64_t have_i = base.index_bytes < index_count ? index_count - base.index_bytes : 0u;
    if (have_v > total.values) have_v = total.values;
    if (have_i > total.index_bytes) have_i = total.index_bytes;
    {
        SliceLoads<4> of_values;
        SliceLoads<2> of_indices;
        const uint32_t value_bytes = (uint32_t)have_v * (uint32_t)sizeof(Bits);
        slice_request<T, 4>(of_values, reinterpret_cast<const uint8_t*>(value_slice), value_bytes);
        slice_request<T, 2>(of_indices, index_slice, (uint32_t)have_i);
        slice_commit<T, 4>(of_values, stage_v, reinterpret_cast<const uint8_t*>(value_slice), value_bytes);
        slice_commit<T, 2>(of_indices, stage_i, index_slice, (uint32_t)have_i);
    }
    __syncthreads();
    if (!live) return;

    const StagedBits* v = reinterpret_cast<const StagedBits*>(stage_v + phase_of(value_slice)) + before.values;
    const uint8_t* idx = stage_i + phase_of(index_slice) + before.index_bytes;
    const uint32_t count = mine.values;                       // the byte's count, at most the tile's elements
    const uint32_t last = count > 0u ? count - 1u : 0u;       // reads of values are clamped to the tile's piece
    const bool in_bounds = before.values + mine.values <= have_v && before.index_bytes + mine.index_bytes <= have_i;
    Bits* out = static_cast<Bits*>(const_cast<void*>(s.x)) + t.origin;
    Bits e[N][N];
#pragma unroll
    for (int r = 0; r < N; ++r)
#pragma unroll
        for (int c = 0; c < N; ++c) e[r][c] = (Bits)0;

    if (in_bounds && (byte & 0x80u) && s.two_eps > 0.0f) {    // dense, predictive
        uint8_t code[N][N];                                   // all code bytes first (clamped addresses)
#pragma unroll
        for (int r = 0; r < N; ++r)
#pragma unroll
            for (int c = 0; c < N; ++c) {
                const uint32_t rr = r < (int)t.rows ? r : t.rows - 1, cc = c < (int)t.cols ? c : t.cols - 1;
                code[r][c] = idx[rr * t.cols + cc];
            }
        int32_t q[N][N];
        uint32_t used = 0;
#pragma unroll
        for (int r = 0; r < N; ++r) {
#pragma unroll
            for (int c = 0; c < N; ++c) {
                const int32_t left = c > 0 ? q[r][c - 1] : 0, up = r > 0 ? q[r - 1][c] : 0;
                const int32_t diag = (r > 0 && c > 0) ? q[r - 1][c - 1] : 0;
                q[r][c] = 0;
                if (r < (int)t.rows && c < (int)t.cols) {
                    if (code[r][c] == 0) {                    // an outlier: unchanged, and back on the lattice
                        e[r][c] = used < count ? (Bits)v[used] : (Bits)0;
                        ++used;
                        bool ok;
                        q[r][c] = lattice(value_of<Bits>(e[r][c]), s.two_eps, ok);
                    } else {
                        q[r][c] = left + up - diag + ((int32_t)code[r][c] - 128);
                        e[r][c] = stored_of<Bits>((float)q[r][c] * s.two_eps);
                    }
                }
            }
        }
    } else if (in_bounds) {
        // verbatim: a dense tile holds every element it has, a sparse one those its CSR structure
        // names; either way the k-th set bit of the occupancy is the k-th value of the piece
        Mask m = 0;
        if (byte & 0x80u) {
            if (count == t.rows * t.cols) m = valid_mask<N>(t);
        } else if (count > 0u) {
            m = csr_mask<N>(idx, t, count);
        }
#pragma unroll
        for (int r = 0; r < N; ++r)
#pragma unroll
            for (int c = 0; c < N; ++c) {
                const int p = r * N + c;
                const uint32_t rank = popcount((Mask)(m & (((Mask)1 << p) - 1)));
                if ((m >> p) & 1) e[r][c] = (Bits)v[rank < last ? rank : last];
            }
    }
    store_tile<Bits, N>(out, t, s.w, s.rows_are_vectors != 0u, e);
}

// ---- host side ------------------------------------------------------------------------------------
bool aligned(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }
size_t elem_size(int dtype) { return dtype == FH_F32 ? 4u : 2u; }

constexpr int64_t kMaxElems = (int64_t)1 << 31;

// tiles of the whole input, or -1 when the shape is not served
int64_t tile_count(int64_t maps, int64_t h, int64_t w, int64_t n)
{
    if (maps < 0 || h < 1 || w < 1 || (n != 2 && n != 4 && n != 8)) return -1;
    if (h > kMaxElems || w > kMaxElems || h * w > kMaxElems) return -1;
    if (maps > kMaxElems / (h * w)) return -1;
    return maps * ((h + n - 1) / n) * ((w + n - 1) / n);
}

int tiles_per_workgroup(int n) { return n == 8 ? Group<8>::kTiles : Group<4>::kTiles; }
uint32_t workgroups(int64_t tiles, int n) { return (uint32_t)((tiles + tiles_per_workgroup(n) - 1) / tiles_per_workgroup(n)); }

MapShape make_shape(const void* x, int64_t h, int64_t w, int n, int64_t tiles, float eps)
{
    MapShape s;
    s.x = x;
    s.two_eps = eps > 0.0f ? eps + eps : 0.0f;                // also 0 for NaN
    s.rows_are_vectors = (w % n == 0 && (reinterpret_cast<uintptr_t>(x) & 15u) == 0u) ? 1u : 0u;
    s.h = (uint32_t)h; s.w = (uint32_t)w; s.n = (uint32_t)n;
    s.tiles = (uint32_t)tiles;
    s.BH = (uint32_t)((h + n - 1) / n);
    s.BW = (uint32_t)((w + n - 1) / n);
    s.bw = make_exact_div(s.BW);
    s.bh = make_exact_div(s.BH);
    return s;
}

fh_status check_shape(int64_t maps, int64_t h, int64_t w, int32_t n, int64_t* tiles)
{
    if (n != 2 && n != 4 && n != 8) return FH_ERR_BAD_PARAM;
    if (maps < 0 || h < 1 || w < 1) return FH_ERR_BAD_SHAPE;
    *tiles = tile_count(maps, h, w, n);
    return *tiles < 0 ? FH_ERR_BAD_NUMEL : FH_OK;
}

}  // namespace
}  // namespace fh

extern "C" {

size_t fh_sparse_info_bytes(int64_t maps, int64_t h, int64_t w, int32_t n)
{
    const int64_t t = fh::tile_count(maps, h, w, n);
    return t < 0 ? 0 : (size_t)t;
}

size_t fh_sparse_index_bytes(int64_t maps, int64_t h, int64_t w, int32_t n)
{
    const int64_t t = fh::tile_count(maps, h, w, n);
    return t < 0 ? 0 : (size_t)t * (size_t)(n + 1) + (size_t)(maps * h * w);
}

size_t fh_sparse_workspace_bytes(int64_t maps, int64_t h, int64_t w, int32_t n)
{
    const int64_t t = fh::tile_count(maps, h, w, n);
    if (t < 0) return 0;
    return sizeof(fh::Sums) * (size_t)(fh::workgroups(t, n) > 0 ? fh::workgroups(t, n) : 1);
}

}  // extern "C"

namespace {

using namespace fh;

fh_status check_encode(const fh_sparse_encode_item& it, int64_t* tiles)
{
    if (it.dtype != FH_F32 && it.dtype != FH_BF16) return FH_ERR_BAD_DTYPE;
    const fh_status st = check_shape(it.maps, it.h, it.w, it.n, tiles);
    if (st != FH_OK) return st;
    if (!it.totals || !it.workspace) return FH_ERR_NULL;
    if (!aligned(it.totals, 8) || !aligned(it.workspace, 8)) return FH_ERR_ALIGNMENT;
    if (it.workspace_cap < fh_sparse_workspace_bytes(it.maps, it.h, it.w, it.n)) return FH_ERR_BUFFER_TOO_SMALL;
    if (*tiles == 0) return FH_OK;
    if (!it.x || !it.info || !it.values || !it.indices) return FH_ERR_NULL;
    if (!aligned(it.x, 4) || !aligned(it.values, 4)) return FH_ERR_ALIGNMENT;
    if (it.info_cap < (size_t)*tiles || it.values_cap < (size_t)(it.maps * it.h * it.w) * elem_size(it.dtype) ||
        it.indices_cap < fh_sparse_index_bytes(it.maps, it.h, it.w, it.n))
        return FH_ERR_BUFFER_TOO_SMALL;
    return FH_OK;
}

fh_status check_decode(const fh_sparse_decode_item& it, int64_t* tiles)
{
    if (it.dtype != FH_F32 && it.dtype != FH_BF16) return FH_ERR_BAD_DTYPE;
    if (it.reserved != 0) return FH_ERR_BAD_PARAM;
    const fh_status st = check_shape(it.maps, it.h, it.w, it.n, tiles);
    if (st != FH_OK) return st;
    if (*tiles == 0) return FH_OK;
    if (!it.info || !it.out || !it.workspace) return FH_ERR_NULL;
    if ((it.values_bytes > 0 && !it.values) || (it.indices_bytes > 0 && !it.indices)) return FH_ERR_NULL;
    if (!aligned(it.out, 4) || !aligned(it.values, 4) || !aligned(it.workspace, 8)) return FH_ERR_ALIGNMENT;
    if (it.workspace_cap < fh_sparse_workspace_bytes(it.maps, it.h, it.w, it.n)) return FH_ERR_BUFFER_TOO_SMALL;
    if (it.out_cap < (size_t)(it.maps * it.h * it.w) * elem_size(it.dtype)) return FH_ERR_BUFFER_TOO_SMALL;
    return FH_OK;
}

template <typename Kernel>
void launch_tiles(Kernel kernel, const Batch<Job>& b, int threads, hipStream_t s)
{
    if (b.count > 0) hipLaunchKernelGGL(kernel, dim3(b.block_start[b.count]), dim3(threads), 0, s, b);
}

// the (dtype, window) instantiation of a templated pass
#define FH_SPARSE_PICK(KERNEL, DTYPE, NN)                                                         \
    ((DTYPE) == FH_F32 ? ((NN) == 2 ? KERNEL<uint32_t, 2> : (NN) == 4 ? KERNEL<uint32_t, 4> : KERNEL<uint32_t, 8>)  \
                       : ((NN) == 2 ? KERNEL<uint16_t, 2> : (NN) == 4 ? KERNEL<uint16_t, 4> : KERNEL<uint16_t, 8>))

#define FH_SPARSE_PICK_STREAM(KERNEL, DTYPE, NN, ST)                                              \
    ((DTYPE) == FH_F32 ? ((NN) == 2 ? KERNEL<uint32_t, 2, ST> : (NN) == 4 ? KERNEL<uint32_t, 4, ST> : KERNEL<uint32_t, 8, ST>)  \
                       : ((NN) == 2 ? KERNEL<uint16_t, 2, ST> : (NN) == 4 ? KERNEL<uint16_t, 4, ST> : KERNEL<uint16_t, 8, ST>))

// jobs of one run (same dtype and window): every set with tiles in `tiled`, all sets in `all`
struct Run {
    Batch<Job> tiled, grouped, all;                // pass 3 | pass 1 (several groups per workgroup) | scan
    bool any_scan;
};

void add_job(Run& run, Job job, int64_t tiles)
{
    job.wg_count = workgroups(tiles, (int)job.shape.n);
    job.scanned = (tiles == 0 || job.wg_count > kSelfScanLimit) ? 1u : 0u;   // an empty set: the scan kernel writes its totals
    if (job.scanned) run.any_scan = true;
    if (tiles > 0) {
        push(run.tiled, job, job.wg_count);
        push(run.grouped, job, (job.wg_count + kGroupsPerWorkgroup - 1) / kGroupsPerWorkgroup);
    }
    push(run.all, job, 1);
}

}  // namespace

extern "C" {

int32_t fh_sparse_batch_capacity(void) { return fh::kBatch; }

fh_status fh_sparse_encode_batch(const fh_sparse_encode_item* items, int32_t count, void* stream)
{
    if (count < 0) return FH_ERR_BAD_COUNT;
    if (count > 0 && !items) return FH_ERR_NULL;
    for (int32_t i = 0; i < count; ++i) {                     // everything is checked before the first launch
        int64_t tiles;
        const fh_status st = check_encode(items[i], &tiles);
        if (st != FH_OK) return st;
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    bool launched = false;
    int32_t i = 0;
    while (i < count) {                                       // runs of one dtype and window, at most kBatch long
        Run run;
        reset(run.tiled);
        reset(run.grouped);
        reset(run.all);
        run.any_scan = false;
        const int dtype = items[i].dtype, n = items[i].n;
        uint64_t run_bytes = 0;
        while (i < count && run.all.count < kBatch && items[i].dtype == dtype && items[i].n == n) {
            const fh_sparse_encode_item& it = items[i];
            int64_t tiles;
            check_encode(it, &tiles);
            if ((uint64_t)run.tiled.block_start[run.tiled.count] + workgroups(tiles, n) > (uint64_t)INT_MAX) {
                if (run.all.count == 0) return FH_ERR_BAD_NUMEL;
                break;
            }
            Job job;
            job.shape = make_shape(it.x, it.h, it.w, it.n, tiles, it.eps);
            job.info = static_cast<uint8_t*>(it.info);
            job.wg = static_cast<Sums*>(it.workspace);
            job.values = it.values;
            job.indices = static_cast<uint8_t*>(it.indices);
            job.totals = static_cast<uint64_t*>(it.totals);
            job.value_count = job.index_count = 0;
            job.tau = it.tau;
            add_job(run, job, tiles);
            run_bytes += (uint64_t)it.maps * (uint64_t)it.h * (uint64_t)it.w * elem_size(it.dtype);
            ++i;
        }
        launched = true;
        seal(run.tiled);
        seal(run.grouped);
        seal(run.all);
// maps that no cache will hold until the second pass are read with the non-temporal hint in both
        const bool streamed = run_bytes >= kStreamedFrom;
        if (streamed) launch_tiles(FH_SPARSE_PICK_STREAM(sparse_count_kernel, dtype, n, true), run.tiled, tiles_per_workgroup(n), s);
        else launch_tiles(FH_SPARSE_PICK_STREAM(sparse_count_kernel, dtype, n, false), run.tiled, tiles_per_workgroup(n), s);
        if (run.any_scan)
            hipLaunchKernelGGL(sparse_scan_kernel, dim3(run.all.count), dim3(kScanThreads), 0, s, run.all);
        if (streamed) launch_tiles(FH_SPARSE_PICK_STREAM(sparse_write_kernel, dtype, n, true), run.tiled, tiles_per_workgroup(n), s);
        else launch_tiles(FH_SPARSE_PICK_STREAM(sparse_write_kernel, dtype, n, false), run.tiled, tiles_per_workgroup(n), s);
    }
    if (!launched) return FH_OK;
    return hipGetLastError() == hipSuccess ? FH_OK : FH_ERR_LAUNCH;
}

fh_status fh_sparse_decode_batch(const fh_sparse_decode_item* items, int32_t count, void* stream)
{
    if (count < 0) return FH_ERR_BAD_COUNT;
    if (count > 0 && !items) return FH_ERR_NULL;
    for (int32_t i = 0; i < count; ++i) {
        int64_t tiles;
        const fh_status st = check_decode(items[i], &tiles);
        if (st != FH_OK) return st;
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    bool launched = false;
    int32_t i = 0;
    while (i < count) {
        Run run;
        reset(run.tiled);
        reset(run.grouped);
        reset(run.all);
        run.any_scan = false;
        const int dtype = items[i].dtype, n = items[i].n;
        while (i < count && run.all.count < kBatch && items[i].dtype == dtype && items[i].n == n) {
            const fh_sparse_decode_item& it = items[i];
            int64_t tiles;
            check_decode(it, &tiles);
            if (tiles == 0) { ++i; continue; }                // nothing to restore
            if ((uint64_t)run.tiled.block_start[run.tiled.count] + workgroups(tiles, n) > (uint64_t)INT_MAX) {
                if (run.all.count == 0) return FH_ERR_BAD_NUMEL;
                break;
            }
            Job job;
            job.shape = make_shape(it.out, it.h, it.w, it.n, tiles, it.eps);
            job.info = const_cast<uint8_t*>(static_cast<const uint8_t*>(it.info));
            job.wg = static_cast<Sums*>(it.workspace);
            job.values = const_cast<void*>(it.values);
            job.indices = const_cast<uint8_t*>(static_cast<const uint8_t*>(it.indices));
            job.totals = nullptr;
            job.value_count = it.values_bytes / elem_size(it.dtype);
            job.index_count = it.indices_bytes;
            job.tau = 0.0f;
            add_job(run, job, tiles);
            ++i;
        }
        if (run.tiled.count == 0) continue;                   // only empty sets in this run
        launched = true;
        seal(run.tiled);
        seal(run.grouped);
        seal(run.all);
        launch_tiles(n == 2 ? sparse_sums_kernel<2> : n == 4 ? sparse_sums_kernel<4> : sparse_sums_kernel<8>, run.grouped,
                     64 * kGroupsPerWorkgroup, s);
        if (run.any_scan)
            hipLaunchKernelGGL(sparse_scan_kernel, dim3(run.all.count), dim3(kScanThreads), 0, s, run.all);
        launch_tiles(FH_SPARSE_PICK(sparse_read_kernel, dtype, n), run.tiled, tiles_per_workgroup(n), s);
    }
    if (!launched) return FH_OK;
    return hipGetLastError() == hipSuccess ? FH_OK : FH_ERR_LAUNCH;
}

fh_status fh_sparse_encode(const void* x, fh_dtype dtype, int64_t maps, int64_t h, int64_t w, int32_t n, float tau,
                           float eps, void* info, size_t info_cap, void* values, size_t values_cap,
                           void* indices, size_t indices_cap, void* totals,
                           void* workspace, size_t workspace_cap, void* stream)
{
    fh_sparse_encode_item it;
    it.x = x; it.dtype = dtype; it.n = n; it.maps = maps; it.h = h; it.w = w; it.tau = tau; it.eps = eps;
    it.info = info; it.info_cap = info_cap; it.values = values; it.values_cap = values_cap;
    it.indices = indices; it.indices_cap = indices_cap; it.totals = totals;
    it.workspace = workspace; it.workspace_cap = workspace_cap;
    return fh_sparse_encode_batch(&it, 1, stream);
}

fh_status fh_sparse_decode(const void* info, const void* values, size_t values_bytes,
                           const void* indices, size_t indices_bytes, fh_dtype dtype,
                           int64_t maps, int64_t h, int64_t w, int32_t n, float eps,
                           void* out, size_t out_cap, void* workspace, size_t workspace_cap, void* stream)
{
    fh_sparse_decode_item it;
    it.info = info; it.values = values; it.values_bytes = values_bytes;
    it.indices = indices; it.indices_bytes = indices_bytes;
    it.dtype = dtype; it.n = n; it.maps = maps; it.h = h; it.w = w; it.eps = eps; it.reserved = 0;
    it.out = out; it.out_cap = out_cap; it.workspace = workspace; it.workspace_cap = workspace_cap;
    return fh_sparse_decode_batch(&it, 1, stream);
}

}  // extern "C"
