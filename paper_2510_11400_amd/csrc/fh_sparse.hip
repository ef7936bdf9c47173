// Sparse-block storage of salient-channel feature maps on gfx950 (paper Section 4.4.1: a
// binary non-zero mask is mean-filtered by n x n average pooling and compared with a
// threshold tau; sparse blocks are stored in Compressed Sparse Row format, dense blocks are
// kept as they are; zeros come back exactly).
//
// The pooling windows ("tiles" below, to keep them apart from GPU workgroups) are independent,
// and what each contributes to the two output streams is known from one byte of information,
// so the streams are laid out by a prefix sum over tiles -- stream compaction:
//   pass 1  one thread per tile: count non-zeros, decide sparse / dense, write the tile's info
//           byte; each workgroup adds up what its 256 tiles will write;
//   pass 2  one thread per tile: the workgroup's base is the sum of the sums before it (each
//           workgroup adds them up itself while there are few; a scan kernel in between does
//           it once there are many), offsets inside the workgroup come from a scan through
//           LDS, then the tile's values and CSR structure go to their final place.
// Restoring runs the same passes with the info bytes as the only input of pass 1.
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

namespace fh {
namespace {

constexpr int kTileThreads = 256;                  // tiles per workgroup
constexpr int kScanThreads = 1024;
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
    const uint32_t count = info & 0x7fu;                      // non-zeros | elements | outliers
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

// Workgroup-wide exclusive scan of what each thread's tile writes.  A tile writes at most 127
// values and 73 index bytes, so a workgroup's running sums fit 20-bit fields of one 64-bit
// word: lanes scan that word with wave shuffles, and the four wave totals meet in LDS.
constexpr int kTileWaves = kTileThreads / 64;
__device__ __forceinline__ uint64_t pack_sums(const Sums& s)
{
    return s.values | (s.index_bytes << 20) | (s.sparse_tiles << 40);
}
__device__ __forceinline__ Sums unpack_sums(uint64_t p)
{
    return Sums{p & 0xfffffu, (p >> 20) & 0xfffffu, p >> 40};
}
__device__ __forceinline__ Sums workgroup_exclusive_scan(Sums mine, uint64_t* lds /* [kTileWaves] */, Sums* total)
{
    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    const uint64_t own = pack_sums(mine);
    uint64_t inc = own;
#pragma unroll
    for (int step = 1; step < 64; step <<= 1) {
        const uint64_t up = __shfl_up(inc, step, 64);
        if (lane >= (uint32_t)step) inc += up;
    }
    if (lane == 63u) lds[wave] = inc;
    __syncthreads();
    uint64_t before = 0, all = 0;
#pragma unroll
    for (int v = 0; v < kTileWaves; ++v) {
        const uint64_t t = lds[v];
        if ((uint32_t)v < wave) before += t;
        all += t;
    }
    __syncthreads();                                          // lds may be reused right away
    *total = unpack_sums(all);
    return unpack_sums(before + inc - own);
}

// Workgroup-wide sum of full-width sums.
__device__ __forceinline__ Sums workgroup_sum(Sums part, uint64_t* lds /* [3 * kTileWaves] */)
{
    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    uint64_t a = part.values, b = part.index_bytes, c = part.sparse_tiles;
#pragma unroll
    for (int step = 32; step >= 1; step >>= 1) {
        a += __shfl_xor(a, step, 64);
        b += __shfl_xor(b, step, 64);
        c += __shfl_xor(c, step, 64);
    }
    if (lane == 0u) { lds[3 * wave] = a; lds[3 * wave + 1] = b; lds[3 * wave + 2] = c; }
    __syncthreads();
    Sums total = {0, 0, 0};
#pragma unroll
    for (int v = 0; v < kTileWaves; ++v) total = total + Sums{lds[3 * v], lds[3 * v + 1], lds[3 * v + 2]};
    __syncthreads();
    return total;
}

// The tile's elements, row-major, zeros where the tile has no element.  Every load is
// unconditional -- out-of-tile positions read a clamped in-tile address -- so all N*N loads
// are in flight together.
template <typename Bits, int N> struct RowVec {               // N elements of Bits as one vector
    typedef Bits type __attribute__((ext_vector_type(N)));
};

template <typename Bits, int N>
__device__ __forceinline__ void load_tile(const Bits* x, const TilePos& t, uint32_t w, bool rows_are_vectors,
                                          Bits (&e)[N][N])
{
    if (rows_are_vectors) {                                   // wave-uniform
        typedef typename RowVec<Bits, N>::type vec;
#pragma unroll
        for (int r = 0; r < N; ++r) {
            const uint32_t rr = r < (int)t.rows ? r : t.rows - 1;
            const vec v = *reinterpret_cast<const vec*>(x + (uint64_t)rr * w);
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
                *reinterpret_cast<vec*>(out + (uint64_t)r * w) = v;
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
// here, 256 at a time.
__device__ __forceinline__ Sums workgroup_base(const Sums* __restrict__ wg, bool scanned, uint32_t block,
                                               uint64_t* lds)
{
    if (scanned) return wg[block];
    Sums part = {0, 0, 0};
    for (uint32_t i = threadIdx.x; i < block; i += kTileThreads) part = part + wg[i];
    return workgroup_sum(part, lds);
}

// ---- pass 1 (encode): non-zero count, density, info byte, workgroup sums ---------------------
template <typename Bits, int N>
__global__ __launch_bounds__(kTileThreads) void sparse_count_kernel(const Batch<Job> batch)
{
    __shared__ uint64_t lds[3 * kTileWaves];
    uint32_t block;
    const Job& job = batch.item[batch_item(batch, blockIdx.x, block)];
    const MapShape& s = job.shape;
    const float tau = job.tau;
    uint8_t* info = job.info;
    Sums* wg_sums = job.wg;
    const uint32_t b = block * kTileThreads + threadIdx.x;
    Sums mine = {0, 0, 0};
    if (b < s.tiles) {
        const TilePos t = tile_pos(s, b);
        Bits e[N][N];
        load_tile<Bits, N>(static_cast<const Bits*>(s.x) + t.origin, t, s.w, s.rows_are_vectors != 0u, e);
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
    Sums total;
    workgroup_exclusive_scan(mine, lds, &total);
    if (threadIdx.x == 0) wg_sums[block] = total;
}

// ---- pass 1 (decode): workgroup sums from the info bytes --------------------------------------
__global__ __launch_bounds__(kTileThreads) void sparse_sums_kernel(const Batch<Job> batch)
{
    __shared__ uint64_t lds[3 * kTileWaves];
    uint32_t block;
    const Job& job = batch.item[batch_item(batch, blockIdx.x, block)];
    const MapShape& s = job.shape;
    const uint32_t b = block * kTileThreads + threadIdx.x;
    Sums mine = {0, 0, 0};
    if (b < s.tiles) mine = tile_sums(job.info[b], tile_pos(s, b), s.two_eps > 0.0f);
    Sums total;
    workgroup_exclusive_scan(mine, lds, &total);
    if (threadIdx.x == 0) job.wg[block] = total;
}

// ---- pass 2: exclusive scan of the workgroup sums, in place; totals -----------------------------
// one workgroup per set; sets with few workgroups skip it (their workgroups add up the sums themselves)
__global__ __launch_bounds__(kScanThreads) void sparse_scan_kernel(const Batch<Job> batch)
{
    const Job& job = batch.item[blockIdx.x];
    if (!job.scanned) return;                                 // workgroup-uniform
    Sums* wg_sums = job.wg;
    const uint32_t count = job.wg_count, tiles = job.shape.tiles;
    uint64_t* totals = job.totals;
    __shared__ Sums lds[kScanThreads];
    const int t = threadIdx.x;
    Sums carry = {0, 0, 0};
    for (uint32_t base = 0; base < count; base += kScanThreads) {     // every thread walks every chunk
        const uint32_t i = base + t;
        const Sums mine = i < count ? wg_sums[i] : Sums{0, 0, 0};
        lds[t] = mine;
        __syncthreads();
        for (int step = 1; step < kScanThreads; step <<= 1) {
            Sums add = {0, 0, 0};
            if (t >= step) add = lds[t - step];
            __syncthreads();
            lds[t] = lds[t] + add;
            __syncthreads();
        }
        const Sums inclusive = lds[t];
        const Sums chunk = lds[kScanThreads - 1];
        if (i < count)
            wg_sums[i] = Sums{carry.values + inclusive.values - mine.values,
                              carry.index_bytes + inclusive.index_bytes - mine.index_bytes,
                              carry.sparse_tiles + inclusive.sparse_tiles - mine.sparse_tiles};
        carry = carry + chunk;
        __syncthreads();
    }
    if (t == 0 && totals) {
        totals[0] = carry.values;
        totals[1] = carry.index_bytes;
        totals[2] = carry.sparse_tiles;
        totals[3] = (uint64_t)tiles - carry.sparse_tiles;
    }
}

// ---- pass 3 (encode): values and CSR structure to their place ---------------------------------------
template <typename Bits, int N>
__global__ __launch_bounds__(kTileThreads) void sparse_write_kernel(const Batch<Job> batch)
{
    __shared__ uint64_t lds[3 * kTileWaves];
    uint32_t block;
    const Job& job = batch.item[batch_item(batch, blockIdx.x, block)];
    const MapShape& s = job.shape;
    const uint8_t* info = job.info;
    const Sums* wg = job.wg;
    const bool scanned = job.scanned != 0u;
    Bits* values = static_cast<Bits*>(job.values);
    uint8_t* indices = job.indices;
    uint64_t* totals = job.totals;
    const uint32_t b = block * kTileThreads + threadIdx.x;
    const bool live = b < s.tiles;
    TilePos t = {0, 1, 1};
    uint32_t byte = 0x80u;
    Sums mine = {0, 0, 0};
    Bits e[N][N];
    if (live) {
        t = tile_pos(s, b);
        byte = info[b];
        mine = tile_sums(byte, t, s.two_eps > 0.0f);
        load_tile<Bits, N>(static_cast<const Bits*>(s.x) + t.origin, t, s.w, s.rows_are_vectors != 0u, e);
    }
    const Sums base = workgroup_base(wg, scanned, block, lds);
    Sums total;
    const Sums before = workgroup_exclusive_scan(mine, lds, &total);
    if (!scanned && totals && block == job.wg_count - 1 && threadIdx.x == 0) {
        totals[0] = base.values + total.values;
        totals[1] = base.index_bytes + total.index_bytes;
        totals[2] = base.sparse_tiles + total.sparse_tiles;
        totals[3] = (uint64_t)s.tiles - totals[2];
    }
    if (!live) return;
    Bits* v = values + base.values + before.values;
    if ((byte & 0x80u) && s.two_eps > 0.0f) {                 // dense, predictive: code bytes + outliers
        uint8_t code[N][N];
        lorenzo_codes<Bits, N>(e, t, s.two_eps, code);
        uint8_t* codes = indices + base.index_bytes + before.index_bytes;
        uint32_t k = 0;
#pragma unroll
        for (int r = 0; r < N; ++r)
#pragma unroll
            for (int c = 0; c < N; ++c)
                if (r < (int)t.rows && c < (int)t.cols) {
                    codes[r * t.cols + c] = code[r][c];
                    if (code[r][c] == 0) v[k++] = e[r][c];
                }
    } else if (byte & 0x80u) {                                // dense: the tile, row-major
#pragma unroll
        for (int r = 0; r < N; ++r)
#pragma unroll
            for (int c = 0; c < N; ++c)
                if (r < (int)t.rows && c < (int)t.cols) v[r * t.cols + c] = e[r][c];
    } else {                                                  // sparse: row_ptr, then columns; values alongside
        uint8_t* row_ptr = indices + base.index_bytes + before.index_bytes;
        uint8_t* col = row_ptr + t.rows + 1;
        uint32_t k = 0;
#pragma unroll
        for (int r = 0; r < N; ++r) {
            if (r <= (int)t.rows) row_ptr[r] = (uint8_t)k;    // r == rows: the closing entry
#pragma unroll
            for (int c = 0; c < N; ++c) {
                if (bits_of<Bits>(e[r][c]) != 0u) {           // padding is zero, so it never gets here
                    v[k] = e[r][c];
                    col[k] = (uint8_t)c;
                    ++k;
                }
            }
        }
        if ((int)t.rows == N) row_ptr[N] = (uint8_t)k;
    }
}

// ---- pass 3 (decode): tiles back from the streams -------------------------------------------------
// A stream this library did not write must not make the kernel read or write out of bounds:
// a tile whose slice would leave a stream is zero-filled, entries outside the tile are dropped.
template <typename Bits, int N>
__global__ __launch_bounds__(kTileThreads) void sparse_read_kernel(const Batch<Job> batch)
{
    __shared__ uint64_t lds[3 * kTileWaves];
    uint32_t block;
    const Job& job = batch.item[batch_item(batch, blockIdx.x, block)];
    const MapShape& s = job.shape;
    const uint8_t* info = job.info;
    const Sums* wg = job.wg;
    const bool scanned = job.scanned != 0u;
    const Bits* values = static_cast<const Bits*>(job.values);
    const uint64_t value_count = job.value_count, index_count = job.index_count;
    const uint8_t* indices = job.indices;
    const uint32_t b = block * kTileThreads + threadIdx.x;
    const bool live = b < s.tiles;
    TilePos t = {0, 1, 1};
    uint32_t byte = 0x80u;
    Sums mine = {0, 0, 0};
    if (live) {
        t = tile_pos(s, b);
        byte = info[b];
        mine = tile_sums(byte, t, s.two_eps > 0.0f);
    }
    const Sums base = workgroup_base(wg, scanned, block, lds);
    Sums total;
    const Sums before = workgroup_exclusive_scan(mine, lds, &total);
    if (!live) return;
    Bits* out = static_cast<Bits*>(const_cast<void*>(s.x)) + t.origin;
    const uint64_t v0 = base.values + before.values, i0 = base.index_bytes + before.index_bytes;
    const uint32_t count = byte & 0x7fu;
    const bool in_bounds = v0 + mine.values <= value_count && i0 + mine.index_bytes <= index_count;
    const Bits* v = values + v0;
    if ((byte & 0x80u) && s.two_eps > 0.0f) {                 // dense, predictive
        if (!in_bounds) {
            const Bits zeros[N][N] = {};
            store_tile<Bits, N>(out, t, s.w, s.rows_are_vectors != 0u, zeros);
            return;
        }
        const uint8_t* codes = indices + i0;
        uint8_t code[N][N];                                   // all code bytes first (clamped addresses)
#pragma unroll
        for (int r = 0; r < N; ++r)
#pragma unroll
            for (int c = 0; c < N; ++c) {
                const uint32_t rr = r < (int)t.rows ? r : t.rows - 1, cc = c < (int)t.cols ? c : t.cols - 1;
                code[r][c] = codes[rr * t.cols + cc];
            }
        int32_t q[N][N];
        Bits e[N][N];
        uint32_t used = 0;
#pragma unroll
        for (int r = 0; r < N; ++r) {
#pragma unroll
            for (int c = 0; c < N; ++c) {
                const int32_t left = c > 0 ? q[r][c - 1] : 0, up = r > 0 ? q[r - 1][c] : 0;
                const int32_t diag = (r > 0 && c > 0) ? q[r - 1][c - 1] : 0;
                q[r][c] = 0;
                e[r][c] = (Bits)0;
                if (r < (int)t.rows && c < (int)t.cols) {
                    if (code[r][c] == 0) {                    // an outlier: unchanged, and back on the lattice
                        e[r][c] = used < count ? v[used] : (Bits)0;
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
        store_tile<Bits, N>(out, t, s.w, s.rows_are_vectors != 0u, e);
        return;
    }
    if ((byte & 0x80u) && in_bounds && count == t.rows * t.cols) {
        Bits e[N][N];                                         // all loads first (clamped), then the stores
#pragma unroll
        for (int r = 0; r < N; ++r)
#pragma unroll
            for (int c = 0; c < N; ++c) {
                const uint32_t rr = r < (int)t.rows ? r : t.rows - 1, cc = c < (int)t.cols ? c : t.cols - 1;
                e[r][c] = v[rr * t.cols + cc];
            }
        store_tile<Bits, N>(out, t, s.w, s.rows_are_vectors != 0u, e);
        return;
    }
    {
        const Bits zeros[N][N] = {};
        store_tile<Bits, N>(out, t, s.w, s.rows_are_vectors != 0u, zeros);
    }
    if ((byte & 0x80u) || !in_bounds || count == 0u) return;
    const uint8_t* row_ptr = indices + i0;
    const uint8_t* col = row_ptr + t.rows + 1;
    uint32_t rp[N + 1];                                       // row_ptr[1..rows], clamped reads
#pragma unroll
    for (int r = 1; r <= N; ++r) rp[r] = row_ptr[r <= (int)t.rows ? r : t.rows];
    // entries in chunks of 8, each chunk's loads issued together; the row of entry k is the
    // number of rows that end at or before k
    for (uint32_t k0 = 0; k0 < count; k0 += 8) {
        uint32_t cc[8];
        Bits vv[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint32_t k = k0 + j < count ? k0 + j : count - 1;
            cc[j] = col[k];
            vv[j] = v[k];
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint32_t k = k0 + j;
            uint32_t r = 0;
#pragma unroll
            for (int q = 1; q <= N; ++q) r += (q <= (int)t.rows && rp[q] <= k) ? 1u : 0u;
            if (k < count && r < t.rows && cc[j] < t.cols) out[(uint64_t)r * s.w + cc[j]] = vv[j];
        }
    }
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

uint32_t workgroups(int64_t tiles) { return (uint32_t)((tiles + kTileThreads - 1) / kTileThreads); }

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
    return sizeof(fh::Sums) * (size_t)(fh::workgroups(t) > 0 ? fh::workgroups(t) : 1);
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
void launch_tiles(Kernel kernel, const Batch<Job>& b, hipStream_t s)
{
    if (b.count > 0) hipLaunchKernelGGL(kernel, dim3(b.block_start[b.count]), dim3(kTileThreads), 0, s, b);
}

// the (dtype, window) instantiation of a templated pass
#define FH_SPARSE_PICK(KERNEL, DTYPE, NN)                                                         \
    ((DTYPE) == FH_F32 ? ((NN) == 2 ? KERNEL<uint32_t, 2> : (NN) == 4 ? KERNEL<uint32_t, 4> : KERNEL<uint32_t, 8>)  \
                       : ((NN) == 2 ? KERNEL<uint16_t, 2> : (NN) == 4 ? KERNEL<uint16_t, 4> : KERNEL<uint16_t, 8>))

// jobs of one run (same dtype and window): every set with tiles in `tiled`, all sets in `all`
struct Run {
    Batch<Job> tiled, all;
    bool any_scan;
};

void add_job(Run& run, Job job, int64_t tiles)
{
    job.wg_count = workgroups(tiles);
    job.scanned = (tiles == 0 || job.wg_count > kSelfScanLimit) ? 1u : 0u;   // an empty set: the scan kernel writes its totals
    if (job.scanned) run.any_scan = true;
    if (tiles > 0) push(run.tiled, job, job.wg_count);
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
        reset(run.all);
        run.any_scan = false;
        const int dtype = items[i].dtype, n = items[i].n;
        while (i < count && run.all.count < kBatch && items[i].dtype == dtype && items[i].n == n) {
            const fh_sparse_encode_item& it = items[i];
            int64_t tiles;
            check_encode(it, &tiles);
            if ((uint64_t)run.tiled.block_start[run.tiled.count] + workgroups(tiles) > (uint64_t)INT_MAX) {
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
            ++i;
        }
        launched = true;
        seal(run.tiled);
        seal(run.all);
        launch_tiles(FH_SPARSE_PICK(sparse_count_kernel, dtype, n), run.tiled, s);
        if (run.any_scan)
            hipLaunchKernelGGL(sparse_scan_kernel, dim3(run.all.count), dim3(kScanThreads), 0, s, run.all);
        launch_tiles(FH_SPARSE_PICK(sparse_write_kernel, dtype, n), run.tiled, s);
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
        reset(run.all);
        run.any_scan = false;
        const int dtype = items[i].dtype, n = items[i].n;
        while (i < count && run.all.count < kBatch && items[i].dtype == dtype && items[i].n == n) {
            const fh_sparse_decode_item& it = items[i];
            int64_t tiles;
            check_decode(it, &tiles);
            if (tiles == 0) { ++i; continue; }                // nothing to restore
            if ((uint64_t)run.tiled.block_start[run.tiled.count] + workgroups(tiles) > (uint64_t)INT_MAX) {
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
        seal(run.all);
        launch_tiles(sparse_sums_kernel, run.tiled, s);
        if (run.any_scan)
            hipLaunchKernelGGL(sparse_scan_kernel, dim3(run.all.count), dim3(kScanThreads), 0, s, run.all);
        launch_tiles(FH_SPARSE_PICK(sparse_read_kernel, dtype, n), run.tiled, s);
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
