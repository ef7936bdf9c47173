// Huffman coding of a byte stream on gfx950 (paper Section 4.4.1: the quantisation codes of
// the predictive form are encoded with Huffman coding; restoring starts with Huffman
// decoding).  The paper names the coder only; the definition used (tie-breaks, 24-bit limit,
// canonical codes, layout) is the one in include/fedhybrid.h.
//
// A variable-length code is sequential per symbol, so the stream is cut into chunks of 256
// symbols that start on a 32-bit word; the decoder gives a chunk to a thread, the encoder to
// sixteen lanes.  Encoding is stream compaction again:
//   histogram   LDS counters, one copy per bank and the copies interleaved, so that no two lanes
//               of a half-wave meet in a bank whatever the bytes are; added to the global
//               histogram at the end;
//   code        one workgroup: the used symbols are ranked by (count, symbol) in parallel, one
//               lane runs the two-queue construction over the ranked leaves (at most 255
//               merges) and walks the tree for the depths; counts are halved and the
//               construction repeated while a code would exceed 24 bits; canonical codes;
//   count       a wave reads four chunks at a time with one 16-byte load per lane and adds the
//               code lengths up over each chunk's sixteen lanes: the chunk's length in words;
//   scan        the sums of groups of 256 chunks (a workgroup of the count pass) are scanned by
//               one workgroup;
//   write       word counts become offsets (group base + a scan over the workgroup); a wave
//               then codes four chunks at a time, every lane placing the bits of its sixteen
//               symbols in an LDS area by OR, and stores the four chunks' words -- one
//               contiguous piece -- with consecutive lanes on consecutive words.
// Decoding needs no pass but one: the offsets are part of the stream.  A workgroup rebuilds the
// canonical tables from the 256 lengths (a 12-bit lookup table for the short codes, first-code /
// count comparisons for the longer ones), stages the payload slice of 768 chunks in LDS (150 of
// the compute unit's 160 KiB: one workgroup of twelve waves each), and a thread decodes its chunk
// from there; the tables serve several such groups in long streams.
// Everything here is integer work; results do not depend on launch geometry.
#include "../../include/fedhybrid.h"

#include "fh_batch.hpp"
#include "fh_scan.hpp"

namespace fh {
namespace {

constexpr int kChunk = 256;                        // symbols per chunk (= per thread)
constexpr int kThreads = 256;                      // chunks per workgroup: a group
constexpr int kMaxLen = 24;
constexpr int kChunkWordsMax = kChunk * kMaxLen / 32;
constexpr int kHistCopies = 32;                     // one per LDS bank
constexpr int kHistBlocksMax = 640;                // histogram workgroups per stream: 2.5 per compute unit
constexpr int kFastBits = 12;
constexpr int kBurst = 8;                          // decode: 16-byte output vectors held back and stored together
// decode: chunks per workgroup.  The payload slice in LDS is what limits the chunks in flight on a compute unit,
// and the decode waits on dependent instructions, not on a unit: one workgroup with the whole LDS holds 768
// chunks (twelve waves) where workgroups of 256 with their own tables held 512.
constexpr int kDecodeThreads = 768;
constexpr int kDecodeThreadsSmall = 256;           // ... of a launch that would leave compute units idle with 768
// decode: LDS for a workgroup's payload slice, in words per chunk: 48 (6 bits per symbol) is what fits beside the
// tables when one workgroup of 768 takes the whole LDS; two workgroups of 256 per unit have room for 64 (8 bits per
// symbol: any slice fits on average, and streams of 7-8 bits per symbol no longer fall back to the rings)
template <int THREADS> struct StageWords { static constexpr int kPerChunk = THREADS >= 768 ? 46 : 64; };
constexpr int kSecondEntries = 2048;               // decode: entries of the table behind the fast one
constexpr int kComputeUnits = 256;                 // MI355X

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

struct Layout {                                    // where things are in the stream and in the workspace
    uint8_t*  len;                                 // [256]
    uint32_t* offsets;                             // [chunks + 1]
    uint32_t* payload;
    uint32_t* hist;                                // workspace: [256]
    uint32_t* table;                               // workspace: [256], code << 8 | length
    uint32_t* group_sums;                          // workspace: [groups]
    uint64_t* totals;                              // {stream bytes used, payload bits}
    const uint8_t* in;
    uint64_t  n;                                   // symbols (an upper bound when n_dev is set)
    const uint64_t* n_dev;                         // device: the symbol count, known only on the stream; or null
    uint32_t  chunks, groups;
    uint32_t  hist_blocks;                         // workgroups of the histogram pass
};

__device__ __forceinline__ uint64_t chunks_for(uint64_t n) { return (n + 255u) >> 8; }

// The layout a kernel works with.  When the symbol count lives in device memory (it is the
// output of an earlier call on the same stream), the host has sized buffers and grids for an
// upper bound; the count itself, and what follows from it -- chunks, groups, where the payload
// starts -- is settled here, and workgroups beyond the real extent find nothing to do.
__device__ __forceinline__ Layout resolved(const Layout& given)
{
    Layout lay = given;
    if (given.n_dev) {
        const uint64_t there = *given.n_dev;
        lay.n = there < given.n ? there : given.n;
        lay.chunks = (uint32_t)chunks_for(lay.n);
        lay.groups = (lay.chunks + 255u) >> 8;
        lay.payload = lay.offsets + lay.chunks + 1;
    }
    return lay;
}

struct DecodeJob {
    const uint8_t*  len;
    const uint32_t* offsets;
    const uint32_t* payload;
    uint8_t*        out;
    uint64_t        n;                                        // symbols (an upper bound when n_dev is set)
    const uint64_t* n_dev;                                    // device: the symbol count; or null
    uint64_t        stream_bytes;                             // the valid prefix of the stream
    uint32_t        payload_words, chunks;
    uint32_t        chunks_per_block;                         // chunks that a workgroup decodes with one set of tables
};

// Every pass serves up to kBatch streams (fh_batch.hpp); the per-stream passes take a workgroup per stream.
__global__ __launch_bounds__(256) void huffman_clear_kernel(const Batch<Layout> batch) { batch.item[blockIdx.x].hist[threadIdx.x] = 0u; }

// ---- histogram ------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void huffman_histogram_kernel(const Batch<Layout> batch)
{
    uint32_t block;
    const Layout lay = resolved(batch.item[batch_item(batch, blockIdx.x, block)]);
    const uint8_t* in = lay.in;
    const uint64_t n = lay.n;
    uint32_t* hist = lay.hist;
    // One copy of the histogram per LDS bank, the copies interleaved so that copy c of every bin lies in bank c:
    // lane l counts in copy l mod 32, and whatever the bytes are no two lanes of a half-wave meet in a bank
    // (bytes clustered around one value would otherwise serialise on the few bins they share).
    __shared__ uint32_t local[256][kHistCopies];
    for (int i = threadIdx.x; i < kHistCopies * 256; i += 256) (&local[0][0])[i] = 0u;
    __syncthreads();
    uint32_t* mine = &local[0][threadIdx.x & (kHistCopies - 1)];
    const uint64_t vectors = n >> 4;                          // `in` is 16-byte aligned
    const uint64_t stride = (uint64_t)lay.hist_blocks * 256;
    uint64_t v = (uint64_t)block * 256 + threadIdx.x;
    u32x4 ahead = v < vectors ? reinterpret_cast<const u32x4*>(in)[v] : u32x4{0u, 0u, 0u, 0u};
    for (; v < vectors; v += stride) {
        const u32x4 w = ahead;
        if (v + stride < vectors) ahead = reinterpret_cast<const u32x4*>(in)[v + stride];   // in flight during the counting
        const uint32_t word[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
        for (int k = 0; k < 4; ++k)
#pragma unroll
            for (int b = 0; b < 4; ++b) atomicAdd(&mine[((word[k] >> (8 * b)) & 0xffu) * kHistCopies], 1u);
    }
    if (block == 0) {                                         // the bytes after the last whole vector
        const uint64_t i = (vectors << 4) + threadIdx.x;
        if (threadIdx.x < 16 && i < n) atomicAdd(&mine[(uint32_t)in[i] * kHistCopies], 1u);
    }
    __syncthreads();
    uint32_t total = 0;
#pragma unroll
    for (int c = 0; c < kHistCopies; ++c) total += local[threadIdx.x][(c + threadIdx.x) & (kHistCopies - 1)];   // a bank per lane
    if (total) atomicAdd(&hist[threadIdx.x], total);
}

// ---- code lengths and canonical codes ---------------------------------------------------------------
// One workgroup of 256 threads, thread s = symbol s.
__global__ __launch_bounds__(256) void huffman_code_kernel(const Batch<Layout> batch)
{
    const Layout& lay = batch.item[blockIdx.x];
    // counts and weights are sums of at most 2^32 - 1 symbols: 32 bits hold them
    __shared__ __align__(16) uint32_t count[256];             // this round's counts, by symbol
    __shared__ uint32_t weight[511];                          // leaves in rank order, then internal nodes as made
    __shared__ uint16_t parent[511];
    __shared__ uint8_t  length[256];
    __shared__ uint32_t code_of[256];
    __shared__ uint32_t in_wave[4][kMaxLen + 2];              // [w][k]: wave w's symbols that are unused (k = 0) / of length k
    __shared__ uint32_t deepest;
    const uint32_t s = threadIdx.x, wave = s >> 6, lane = s & 63u;
    const uint32_t original = lay.hist[s];
    uint32_t c = original;
    for (;;) {                                                // workgroup-uniform; counts halve, so it ends
        count[s] = c;
        length[s] = 0;
        {
            const uint64_t unused = __ballot(c == 0u);
            if (lane == 0) in_wave[wave][0] = (uint32_t)__popcll(unused);
        }
        __syncthreads();
        const int m = 256 - (int)(in_wave[0][0] + in_wave[1][0] + in_wave[2][0] + in_wave[3][0]);   // used symbols
        // used symbols before this one by (count, symbol): those with a smaller count, the unused ones taken off
        // again, plus those of the same count and a smaller value
        uint32_t rank = 0;
#pragma unroll 4
        for (int t = 0; t < 256; t += 4) {
            const u32x4 four = *reinterpret_cast<const u32x4*>(&count[t]);
            const uint32_t o[4] = {four.x, four.y, four.z, four.w};
#pragma unroll
            for (int k = 0; k < 4; ++k) rank += (o[k] < c ? 1u : 0u) + ((o[k] == c && (uint32_t)(t + k) < s) ? 1u : 0u);
        }
        rank -= 256u - (uint32_t)m;
        if (c != 0) weight[rank] = c;
        __syncthreads();
        if (wave == 0) {
            // The merges are one chain of dependent steps.  The whole first wave runs it with every value the same
            // in all lanes and made known as such (readfirstlane), so that counters, comparisons and branches are
            // scalar instructions; the lanes' LDS stores write one value to one address.  (Both queues spread
            // over the lanes of registers, read with v_readlane and a scalar select, measured slower -- 71 us
            // against 58 for 250 merges: what a merge costs is its instruction count, not the LDS latency.  So did
            // a 64-node window of either queue in one register each, 59 us.  Merges that do not depend on each
            // other done by the lanes at once -- the k leaves no heavier than the front node pair up in
            // floor(k / 2) leaf-leaf merges, the k nodes lighter than the front leaf likewise -- give the same
            // depths and take a uniform histogram's 255 merges from 46 to 7 us, but on the index streams of the
            // predictive form leaves and nodes alternate, few steps find a batch, and the dearer step made the
            // kernel slower: 64 us.  And a merge without branches -- the next two nodes of both queues read from
            // register windows by lane index, the two smallest of the four taken by selects -- is some 50
            // instructions with no wait for LDS, and takes the same time to the microsecond.)
            if (lane == 0) deepest = 0u;
            const uint32_t mm = (uint32_t)__builtin_amdgcn_readfirstlane(m);
            if (mm > 1u) {
                // The first two nodes of either queue are at hand -- the front as a scalar, the one behind it
                // requested from LDS when the front was taken -- so that nothing waits for LDS until a further
                // node has been taken.  kNone stands for a node that does not exist (yet): only the root can
                // weigh 2^32 - 1, and the root is never compared.  One of the fronts always exists: before a
                // merge the queues hold two nodes or more.
                constexpr uint32_t kNone = ~(uint32_t)0;
                uint32_t next_leaf = 0, next_internal = mm, made = mm;
                uint32_t leaf0 = (uint32_t)__builtin_amdgcn_readfirstlane(weight[0]);     // leaf next_leaf
                uint32_t leaf1 = weight[1];                                             // leaf next_leaf + 1, in flight
                uint32_t node0 = kNone;                                                 // internal node next_internal
                uint32_t node1 = kNone;                                                 // internal node next_internal + 1
                while (made < 2u * mm - 1u) {                 // at most 255 merges
                    uint32_t sum = 0;
#pragma unroll
                    for (int k = 0; k < 2; ++k) {
                        if (leaf0 <= node0) {                 // a leaf is preferred to an internal node of equal weight
                            sum += leaf0;
                            parent[next_leaf] = (uint16_t)made;
                            ++next_leaf;
                            leaf0 = (uint32_t)__builtin_amdgcn_readfirstlane(leaf1);
                            leaf1 = next_leaf + 1u < mm ? weight[next_leaf + 1u] : kNone;
                        } else {
                            sum += node0;
                            parent[next_internal] = (uint16_t)made;
                            ++next_internal;
                            node0 = (uint32_t)__builtin_amdgcn_readfirstlane(node1);
                            node1 = next_internal + 1u < made ? weight[next_internal + 1u] : kNone;
                        }
                    }
                    weight[made] = sum;
                    if (made == next_internal) node0 = sum;           // the new node is the queue's front,
                    else if (made == next_internal + 1u) node1 = sum; // or the one behind it
                    ++made;
                }
            }
        }
        __syncthreads();
        if (c != 0) {                                         // every leaf walks up to the root: its depth
            uint32_t d = 1;
            if (m > 1) {
                d = 0;
                for (uint32_t node = rank; node != (uint32_t)(2 * m - 2) && d < 256u; ++d) node = parent[node];
            }
            length[s] = (uint8_t)(d < 255u ? d : 255u);
            atomicMax(&deepest, d);
        }
        __syncthreads();
        if (deepest <= (uint32_t)kMaxLen) break;
        if (c != 0) c = (c + 1) >> 1;
        __syncthreads();                                      // everyone has read `deepest` before it is written again
    }
    // canonical codes: by increasing (length, symbol); a symbol's place among those of its length from lane masks
    // inside the wave plus the counts of the waves below
    __shared__ uint32_t first_code[kMaxLen + 2];
    const uint32_t my_length = length[s];
    uint32_t before = 0;
#pragma unroll
    for (int k = 1; k <= kMaxLen; ++k) {
        const uint64_t same = __ballot(my_length == (uint32_t)k);
        if (my_length == (uint32_t)k) before = __builtin_amdgcn_mbcnt_hi((uint32_t)(same >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)same, 0u));
        if (lane == 0) in_wave[wave][k] = (uint32_t)__popcll(same);
    }
    __syncthreads();
    if (s == 0) {
        uint32_t code = 0;
        first_code[0] = first_code[1] = 0u;
#pragma unroll
        for (int l = 2; l <= kMaxLen; ++l) {
            code = (code + in_wave[0][l - 1] + in_wave[1][l - 1] + in_wave[2][l - 1] + in_wave[3][l - 1]) << 1;
            first_code[l] = code;
        }
    }
    __syncthreads();
    if (my_length) for (uint32_t w = 0; w < wave; ++w) before += in_wave[w][my_length];
    code_of[s] = my_length ? first_code[my_length] + before : 0u;
    __syncthreads();
    lay.len[s] = length[s];
    lay.table[s] = (code_of[s] << 8) | length[s];
    // payload bits: every symbol's count times its length (the counts as they were)
    __shared__ uint64_t bit_sum[256];
    bit_sum[s] = (uint64_t)original * length[s];
    __syncthreads();
    for (int step = 128; step >= 1; step >>= 1) {
        if (s < (uint32_t)step) bit_sum[s] += bit_sum[s + step];
        __syncthreads();
    }
    if (s == 0) lay.totals[1] = bit_sum[0];
}

// the symbols of a chunk, 16 at a time; `valid` of them exist
__device__ __forceinline__ void load_symbols(const uint8_t* in, uint64_t first, uint32_t valid, uint32_t (&word)[4])
{
    if (valid >= 16u) {
        const u32x4 w = *reinterpret_cast<const u32x4*>(in + first);
        word[0] = w.x; word[1] = w.y; word[2] = w.z; word[3] = w.w;
        return;
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        word[k] = 0u;
#pragma unroll
        for (int b = 0; b < 4; ++b)
            if ((uint32_t)(4 * k + b) < valid) word[k] |= (uint32_t)in[first + 4 * k + b] << (8 * b);
    }
}

// exclusive prefix over the workgroup of one value per thread; all = the workgroup's total
__device__ __forceinline__ uint32_t workgroup_exclusive_scan(uint32_t mine, uint32_t* lds /* [4] */, uint32_t* all)
{
    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    const uint32_t inc = wave_inclusive_scan(mine);
    if (lane == 63u) lds[wave] = inc;
    __syncthreads();
    uint32_t before = 0, total = 0;
#pragma unroll
    for (int v = 0; v < kThreads / 64; ++v) {
        const uint32_t t = lds[v];
        if ((uint32_t)v < wave) before += t;
        total += t;
    }
    __syncthreads();
    *all = total;
    return before + inc - mine;
}

// ---- count: words per chunk, sums per group -------------------------------------------------------
// Sixteen lanes share a chunk: a wave reads four consecutive chunks, 1 KiB, with one 16-byte load per lane --
// whole cache lines, each fetched once -- and does so for its 64 chunks in sixteen rounds.  (A thread per chunk,
// walking its 256 bytes alone, asks for 16 bytes of every line its wave touches in a round and finds the rest
// gone from the cache when it comes back: measured, that read 1.2 times the input here and 2.9 times in the
// write pass.)
struct PieceOfChunk {                              // what a lane reads in one round
    uint32_t chunk;                                // the chunk (of the stream), which may not exist
    uint32_t have;                                 // symbols of its 16 that exist: 0 .. 16
    uint64_t first;                                // index of the first of them
};
__device__ __forceinline__ PieceOfChunk piece_of(const Layout& lay, uint32_t group, uint32_t wave, uint32_t round, uint32_t lane)
{
    PieceOfChunk p;
    p.chunk = group * kThreads + wave * 64u + round * 4u + (lane >> 4);
    p.first = (uint64_t)p.chunk * kChunk + (lane & 15u) * 16u;
    p.have = p.first >= lay.n ? 0u : lay.n - p.first < 16u ? (uint32_t)(lay.n - p.first) : 16u;
    return p;
}
// does every lane of the wave have all its 16 symbols in this round?  (wave-uniform, from scalar values)
__device__ __forceinline__ bool round_is_whole(const Layout& lay, uint32_t group, uint32_t wave, uint32_t round)
{
    const uint64_t end = ((uint64_t)group * kThreads + wave * 64u + round * 4u + 4u) * kChunk;
    return end <= lay.n;
}
// sum over the 16 lanes that share a chunk, in the last of them (row shifts: a row of the wave is those 16 lanes)
__device__ __forceinline__ uint32_t sum_to_lane_15_of_row(uint32_t v)
{
    v = dpp_add<0x111, 0xf>(v);
    v = dpp_add<0x112, 0xf>(v);
    v = dpp_add<0x114, 0xf>(v);
    v = dpp_add<0x118, 0xf>(v);
    return v;                                                 // inclusive prefix inside the row
}

__global__ __launch_bounds__(kThreads) void huffman_count_kernel(const Batch<Layout> batch)
{
    uint32_t group;
    const Layout lay = resolved(batch.item[batch_item(batch, blockIdx.x, group)]);
    if (group >= lay.groups) return;                          // workgroup-uniform: past the real extent
    __shared__ uint8_t len[256];
    __shared__ uint32_t lds[4];
    len[threadIdx.x] = (uint8_t)(lay.table[threadIdx.x] & 0xffu);
    __syncthreads();
    const uint32_t lane = threadIdx.x & 63u, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    uint32_t closed = 0;                                      // words of the chunks this lane closed (lanes 15, 31, 47, 63)
    constexpr int kRoundsInFlight = 8;
    for (uint32_t round0 = 0; round0 < 16u; round0 += kRoundsInFlight) {
        uint32_t word[kRoundsInFlight][4];
#pragma unroll
        for (int k = 0; k < kRoundsInFlight; ++k) {
            const PieceOfChunk p = piece_of(lay, group, wave, round0 + k, lane);
            if (round_is_whole(lay, group, wave, round0 + k)) {
                const u32x4 w = *reinterpret_cast<const u32x4*>(lay.in + p.first);
                word[k][0] = w.x; word[k][1] = w.y; word[k][2] = w.z; word[k][3] = w.w;
            } else {
                word[k][0] = word[k][1] = word[k][2] = word[k][3] = 0u;
                if (p.have) load_symbols(lay.in, p.first, p.have, word[k]);
            }
        }
#pragma unroll
        for (int k = 0; k < kRoundsInFlight; ++k) {
            const PieceOfChunk p = piece_of(lay, group, wave, round0 + k, lane);
            uint32_t bits = 0;
            if (round_is_whole(lay, group, wave, round0 + k)) {
#pragma unroll
                for (int j = 0; j < 16; ++j) bits += len[(word[k][j >> 2] >> (8 * (j & 3))) & 0xffu];
            } else {
#pragma unroll
                for (int j = 0; j < 16; ++j)
                    if ((uint32_t)j < p.have) bits += len[(word[k][j >> 2] >> (8 * (j & 3))) & 0xffu];
            }
            const uint32_t of_chunk = sum_to_lane_15_of_row(bits);
            if ((lane & 15u) == 15u && p.chunk < lay.chunks) {
                const uint32_t words = (of_chunk + 31u) >> 5;
                lay.offsets[p.chunk] = words;                 // becomes the chunk's offset in the write pass
                closed += words;
            }
        }
    }
    const uint32_t of_wave = wave_inclusive_scan(closed);
    if (lane == 63u) lds[wave] = of_wave;
    __syncthreads();
    if (threadIdx.x == 0) lay.group_sums[group] = lds[0] + lds[1] + lds[2] + lds[3];
}

// ---- scan of the group sums (in place, exclusive); the stream's size --------------------------------
__global__ __launch_bounds__(kThreads) void huffman_scan_kernel(const Batch<Layout> batch)
{
    const Layout lay = resolved(batch.item[blockIdx.x]);
    __shared__ uint32_t lds[4];
    uint32_t carry = 0;
    for (uint32_t base = 0; base < lay.groups; base += kThreads) {         // workgroup-uniform trip count
        const uint32_t i = base + threadIdx.x;
        const uint32_t mine = i < lay.groups ? lay.group_sums[i] : 0u;
        uint32_t total;
        const uint32_t before = workgroup_exclusive_scan(mine, lds, &total);
        if (i < lay.groups) lay.group_sums[i] = carry + before;
        carry += total;
    }
    if (threadIdx.x == 0) {
        lay.offsets[lay.chunks] = carry;
        lay.totals[0] = 256u + 4ull * (lay.chunks + 1ull) + 4ull * carry;
    }
}

// ---- write: offsets and payload -------------------------------------------------------------------
// The same sharing as in the count pass: a wave codes four consecutive chunks per round, sixteen lanes to a chunk,
// each lane its 16 symbols.  A lane looks its 16 codes up, the lengths are prefix-summed over the chunk's lanes,
// and the lane then puts its bits where they belong in the wave's staging area in LDS -- whole words as they fill
// up, with an OR, since the first and the last word of a lane's run are shared with its neighbours.  The four
// chunks are one contiguous piece of the payload (each starts on a word); the wave copies it out with consecutive
// lanes on consecutive words and leaves the area cleared for the next round.  A chunk is at most 192 words
// (24 bits per symbol), so the area fits whatever the stream holds.
constexpr int kRoundWordsMax = 4 * kChunkWordsMax;          // 768 words per wave

__global__ __launch_bounds__(kThreads) void huffman_write_kernel(const Batch<Layout> batch)
{
    uint32_t group;
    const Layout lay = resolved(batch.item[batch_item(batch, blockIdx.x, group)]);
    if (group >= lay.groups) return;                          // workgroup-uniform: past the real extent
    __shared__ uint32_t table[256];
    __shared__ uint32_t lds[4];
    __shared__ uint32_t chunk_at[kThreads + 4];               // word offset of every chunk inside the group's slice; [256..]: the total
    __shared__ uint32_t area[kThreads / 64][kRoundWordsMax + 4];
    table[threadIdx.x] = lay.table[threadIdx.x];
    {
        const uint32_t chunk = group * kThreads + threadIdx.x;
        const bool live = chunk < lay.chunks;
        const uint32_t words = live ? lay.offsets[chunk] : 0u;
        uint32_t total;
        const uint32_t before = workgroup_exclusive_scan(words, lds, &total);   // also the barrier for `table`
        if (live) lay.offsets[chunk] = lay.group_sums[group] + before;
        chunk_at[threadIdx.x] = before;
        if (threadIdx.x < 4u) chunk_at[kThreads + threadIdx.x] = total;
    }
    const uint32_t lane = threadIdx.x & 63u, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    uint32_t* mine = area[wave];
    for (uint32_t w = lane; w < (uint32_t)kRoundWordsMax + 4u; w += 64u) mine[w] = 0u;
    __syncthreads();
    uint32_t* slice = lay.payload + lay.group_sums[group];
    for (uint32_t round = 0; round < 16u; ++round) {
        const PieceOfChunk p = piece_of(lay, group, wave, round, lane);
        const uint32_t chunk0 = wave * 64u + round * 4u;      // of the group: the first of this round's four
        const uint32_t run_at = chunk_at[chunk0], run = chunk_at[chunk0 + 4u] - run_at;   // wave-uniform
        if (run == 0u) break;                                 // nothing from here on (the stream has ended)
        // the lane's codes
        uint32_t word[4] = {0u, 0u, 0u, 0u};
        if (round_is_whole(lay, group, wave, round)) {
            const u32x4 w = *reinterpret_cast<const u32x4*>(lay.in + p.first);
            word[0] = w.x; word[1] = w.y; word[2] = w.z; word[3] = w.w;
        } else if (p.have) {
            load_symbols(lay.in, p.first, p.have, word);
        }
        uint32_t e[16];                                       // code << 8 | length; a symbol that does not exist: length 0
        uint32_t bits = 0;
        if (round_is_whole(lay, group, wave, round)) {
#pragma unroll
            for (int j = 0; j < 16; ++j) e[j] = table[(word[j >> 2] >> (8 * (j & 3))) & 0xffu];
        } else {
#pragma unroll
            for (int j = 0; j < 16; ++j) e[j] = (uint32_t)j < p.have ? table[(word[j >> 2] >> (8 * (j & 3))) & 0xffu] : 0u;
        }
#pragma unroll
        for (int j = 0; j < 16; ++j) bits += e[j] & 0xffu;
        // where the lane's bits start: its chunk's word offset inside the round, then the lanes before it in the chunk
        const uint32_t start = ((chunk_at[chunk0 + (lane >> 4)] - run_at) << 5) + (sum_to_lane_15_of_row(bits) - bits);
        uint32_t at = start >> 5;                             // the word being filled
        uint32_t filled = start & 31u;                        // bits of it that precede this lane's (left as zeros here)
        uint64_t acc = 0;                                     // the low `filled` bits are pending, oldest on top
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const uint32_t l = e[j] & 0xffu;
            acc = (acc << l) | (e[j] >> 8);
            filled += l;
            if (filled >= 32u) {                              // filled < 32 + 24 before this
                filled -= 32u;
                atomicOr(&mine[at], (uint32_t)(acc >> filled));
                ++at;
            }
        }
        if (filled) atomicOr(&mine[at], (uint32_t)(acc << (32u - filled)));      // the rest, zero-padded to the word's end
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");     // LDS operations of one wave complete in order
        for (uint32_t w = lane; w < run; w += 64u) {
            slice[run_at + w] = mine[w];
            mine[w] = 0u;
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    }
}

// One chunk: `valid` symbols from the words next_word(0), next_word(1), ... to dst (16-byte aligned).
// The per-length tables of a stream, in LDS: what a code longer than the fast table's index is decoded with.
struct LongCodes {
    uint32_t per_length[kMaxLen + 2];                         // [k]: codes of length k
    uint32_t first[kMaxLen + 2];                              // [k]: the first (smallest) code of length k
    uint32_t start[kMaxLen + 2];                              // [k]: position in `sorted` of that code's symbol
    uint8_t  sorted[256];                                     // symbols by (length, symbol)
};

// The symbol whose code, longer than kFastBits, is on top of the stream, as symbol | length << 8 like an entry of the
// fast table.
// Canonical codes grow with their length, so the 32-bit windows that start with a code of length <= k are those up
// to last[k]: the length of the code on top is one more than the number of those bounds that the window exceeds -- a
// compare and an add per length, the bounds (the same for the whole workgroup) in scalar registers -- and its place
// among the symbols sorted by (length, symbol) is its value less `first - start` of its length.  `top`: the next
// 32 bits of the stream.
struct LongRegs {
    uint32_t last[kMaxLen - kFastBits - 1];        // [i]: the largest window that starts with a code of length <= kFastBits + 1 + i
};
__device__ __forceinline__ LongRegs long_regs(const LongCodes* t)
{
    LongRegs r;
#pragma unroll
    for (int i = 0; i < kMaxLen - kFastBits - 1; ++i) {
        const int k = kFastBits + 1 + i;
        // left-justified: one past the windows of length <= k (lengths no encoder wrote can claim more than there is)
        const uint64_t end = ((uint64_t)t->first[k] + t->per_length[k]) << (32 - k);
        const uint32_t last = end > 0xffffffffull ? 0xffffffffu : end ? (uint32_t)end - 1u : 0u;
        r.last[i] = (uint32_t)__builtin_amdgcn_readfirstlane((int)last);
    }
    return r;
}
// symbol | length << 8 like an entry of the fast table; the length is kFastBits + 1 at least, whatever the tables say
__device__ __forceinline__ uint32_t decode_long(uint32_t top, const LongRegs& r, const LongCodes* t)
{
    uint32_t length = kFastBits + 1;
#pragma unroll
    for (int i = 0; i < kMaxLen - kFastBits - 1; ++i) length += top > r.last[i] ? 1u : 0u;
    return t->sorted[((top >> (32u - length)) + t->start[length] - t->first[length]) & 0xffu] | (length << 8);
}

// A long code is rare per symbol, but a wave pays for one whenever ANY of its 64 lanes meets one -- one step in six
// on streams of five bits per symbol -- and the walk over the lengths costs several times a short code's step.  So
// there is a second table behind the fast one.  The long codes are the upper end of the code space: the windows
// whose first kFastBits bits are `from` or more.  Those windows' first kFastBits + extra bits, less from << extra,
// index the second table, whose entries are like the fast one's (0: longer still, walk the lengths).  `extra` is
// as large as kSecondEntries allow, the longest code at most; with no long codes, or more long prefixes than
// entries, there is no second table.
struct Second {
    uint32_t extra;                                // bits beyond kFastBits that index the table; 0: no table
    uint32_t from;                                 // the first index (of kFastBits + extra bits) it covers
    uint32_t entries;
};
__device__ __forceinline__ Second second_of(const LongCodes* t)
{
    Second s{0u, 0u, 0u};
    uint32_t longest = 0;
#pragma unroll
    for (int k = kFastBits + 1; k <= kMaxLen; ++k)
        if (__builtin_amdgcn_readfirstlane((int)t->per_length[k])) longest = (uint32_t)k;
    const uint32_t first = (uint32_t)__builtin_amdgcn_readfirstlane((int)t->first[kFastBits + 1]) >> 1;   // as kFastBits bits
    if (longest == 0u || first >= (1u << kFastBits)) return s;
    const uint32_t prefixes = (1u << kFastBits) - first;
    if (prefixes > (uint32_t)kSecondEntries / 2u) return s;
    uint32_t extra = 1;
    while (extra < longest - kFastBits && (prefixes << (extra + 1u)) <= (uint32_t)kSecondEntries) ++extra;
    s.extra = extra;
    s.from = first << extra;
    s.entries = prefixes << extra;
    return s;
}

// The tables of a stream in LDS, and what the threads hold of them in registers.
struct Lookup {
    const uint16_t*  fast;
    const uint16_t*  second;
    const LongCodes* tables;
    Second           behind;
};
// What the next symbol's code decodes to, as symbol | length << 8, from the stream's next 32 bits.
__device__ __forceinline__ uint32_t decode_symbol(const uint16_t* fast, const uint16_t* second, const Second& behind,
                                                  const LongRegs& longer, const LongCodes* tables, uint32_t top)
{
    uint32_t e = fast[top >> (32 - kFastBits)];
    if (!e) {
        if (behind.extra) {                                   // workgroup-uniform
            // below `from` only in a stream that no encoder wrote: any entry will do
            const uint32_t i = (top >> (32u - kFastBits - behind.extra)) - behind.from;
            e = second[i < behind.entries ? i : behind.entries - 1u];
        }
        if (!e) e = decode_long(top, longer, tables);
    }
    return e;
}

template <typename NextWord>
__device__ __forceinline__ void decode_chunk(uint32_t valid, uint8_t* dst, const Lookup table, NextWord next_word)
{
    const LongRegs longer = long_regs(table.tables);
    const Second behind = table.behind;
    const uint16_t* fast = table.fast;
    const uint16_t* second = table.second;
    const LongCodes* tables = table.tables;
    uint32_t taken = 0;                                       // words moved into `buf`
    uint64_t buf = 0;                                         // pending bits, the next one on top
    uint32_t have = 0;
    for (uint32_t half = 0; half < valid; half += 16 * kBurst) {
        u32x4 piece[kBurst];
#pragma unroll
        for (int v = 0; v < kBurst; ++v) {
            uint32_t sixteen[4];
            if (half + 16u * v >= valid) { piece[v] = u32x4{0u, 0u, 0u, 0u}; continue; }
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                uint32_t four = 0;
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    if (have <= 32u) {
                        const uint32_t w = next_word(taken);
                        ++taken;
                        buf |= (uint64_t)w << (32u - have);
                        have += 32u;
                    }
                    const uint32_t e = decode_symbol(fast, second, behind, longer, tables, (uint32_t)(buf >> 32));
                    const uint32_t symbol = e & 0xffu, used_bits = e >> 8;
                    buf <<= used_bits;
                    have -= used_bits;
                    four |= symbol << (8 * b);
                }
                sixteen[q] = four;
            }
            piece[v] = u32x4{sixteen[0], sixteen[1], sixteen[2], sixteen[3]};
        }
        // a whole cache line's worth of stores back to back: the line is complete in the L2 before it can be evicted
#pragma unroll
        for (int v = 0; v < kBurst; ++v) {
            const uint32_t i = half + 16u * v;
            if (i + 16 <= valid) {
                *reinterpret_cast<u32x4*>(dst + i) = piece[v];
            } else if (i < valid) {
                const uint32_t w[4] = {piece[v].x, piece[v].y, piece[v].z, piece[v].w};
                for (uint32_t b = 0; i + b < valid; ++b) dst[i + b] = (uint8_t)(w[b >> 2] >> (8 * (b & 3u)));
            }
        }
    }
}

// The same from words in LDS: no bit buffer to refill (lanes would diverge on when) -- every
// symbol reads the two words its bits start in and shifts them into place, so a step is two
// dependent LDS reads and nothing data-dependent in the control flow.
__device__ __forceinline__ void decode_chunk_staged(uint32_t valid, uint8_t* dst, const Lookup table, const uint32_t* words)
{
    const LongRegs longer = long_regs(table.tables);
    const Second behind = table.behind;
    const uint16_t* fast = table.fast;
    const uint16_t* second = table.second;
    const LongCodes* tables = table.tables;
    // Three words of the chunk stay in registers: w0 holds bit `pos`, w1 follows, w2 is the word after that.  A
    // symbol advances by at most 24 bits, one word, so after it the registers move up by one at most, and w2 is
    // read again for the new position: that read is needed one symbol later, so that a symbol waits for one LDS
    // access in a row (the table) rather than two (words, then table).
    uint32_t pos = 0, at = 0;                                 // bits of the chunk consumed; at = pos / 32
    uint32_t w0 = words[0], w1 = words[1], w2 = words[2];
    for (uint32_t half = 0; half < valid; half += 16 * kBurst) {
        u32x4 piece[kBurst];
#pragma unroll
        for (int v = 0; v < kBurst; ++v) {
            uint32_t sixteen[4];
            if (half + 16u * v >= valid) { piece[v] = u32x4{0u, 0u, 0u, 0u}; continue; }
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                uint32_t four = 0;
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    const uint32_t top = (uint32_t)(((((uint64_t)w0 << 32) | w1) << (pos & 31u)) >> 32);   // the next 32 bits
                    const uint32_t e = decode_symbol(fast, second, behind, longer, tables, top);
                    four |= (e & 0xffu) << (8 * b);
                    pos += e >> 8;
                    const bool crossed = (pos >> 5) != at;
                    w0 = crossed ? w1 : w0;
                    w1 = crossed ? w2 : w1;
                    at = pos >> 5;
                    w2 = words[at + 2];
                }
                sixteen[q] = four;
            }
            piece[v] = u32x4{sixteen[0], sixteen[1], sixteen[2], sixteen[3]};
        }
        // a whole cache line's worth of stores back to back: the line is complete in the L2 before it can be evicted
#pragma unroll
        for (int v = 0; v < kBurst; ++v) {
            const uint32_t i = half + 16u * v;
            if (i + 16 <= valid) {
                *reinterpret_cast<u32x4*>(dst + i) = piece[v];
            } else if (i < valid) {
                const uint32_t w[4] = {piece[v].x, piece[v].y, piece[v].z, piece[v].w};
                for (uint32_t b = 0; i + b < valid; ++b) dst[i + b] = (uint8_t)(w[b >> 2] >> (8 * (b & 3u)));
            }
        }
    }
}

// ---- decode -------------------------------------------------------------------------------------------
// The stream may be foreign: the tables are built from whatever the 256 length bytes say
// (lengths above 24 count as unused), reads of payload words are bounded by the stream's size
// (words outside read as zero), and every loop is bounded by the symbol count.
template <int kDecodeThreads>
__global__ __launch_bounds__(kDecodeThreads) void huffman_decode_kernel(const Batch<DecodeJob> batch)
{
    constexpr int kStageWords = kDecodeThreads * StageWords<kDecodeThreads>::kPerChunk;
    uint32_t block;
    const DecodeJob& job = batch.item[batch_item(batch, blockIdx.x, block)];
    const uint8_t* len_in = job.len;
    const uint32_t* offsets = job.offsets;
    const uint32_t* payload = job.payload;
    uint32_t payload_words = job.payload_words, chunks = job.chunks;
    uint64_t n = job.n;
    if (job.n_dev) {                                          // the count is on the stream: settle what follows from it
        const uint64_t there = *job.n_dev;
        n = there < job.n ? there : job.n;
        chunks = (uint32_t)chunks_for(n);
        payload = offsets + chunks + 1;
        const uint64_t head = 256u + 4u * ((uint64_t)chunks + 1u);
        const uint64_t words = job.stream_bytes > head ? (job.stream_bytes - head) / 4u : 0u;
        payload_words = (uint32_t)(words < 0xffffffffu ? words : 0xffffffffu);
    }
    uint8_t* out = job.out;
    // One object, so that the order is the one written here: the tables that every symbol is looked up in come first,
    // at addresses small enough for the offset field of an LDS instruction (one addition less per symbol).
    struct Local {
        uint16_t  fast[1 << kFastBits];                       // next kFastBits bits -> symbol | length << 8; 0: longer code
        uint16_t  second[kSecondEntries];                     // the same for the long codes' first kFastBits + extra bits
        LongCodes tables;
        uint32_t  in_wave[kThreads / 64][kMaxLen + 2];        // [w][k]: symbols of length k among wave w's 64
        uint32_t  fitting;                                    // chunks of a pass whose slice fits the stage
        __align__(16) uint32_t stage[kStageWords + kChunkWordsMax + 8];   // the workgroup's slice of the payload, or the rings
    };
    __shared__ Local local;
    LongCodes& tables = local.tables;
    uint32_t (&per_length)[kMaxLen + 2] = tables.per_length, (&first)[kMaxLen + 2] = tables.first, (&start)[kMaxLen + 2] = tables.start;
    uint8_t (&sorted)[256] = tables.sorted;
    uint32_t (&in_wave)[kThreads / 64][kMaxLen + 2] = local.in_wave;
    uint16_t (&fast)[1 << kFastBits] = local.fast;
    uint16_t (&second)[kSecondEntries] = local.second;
    uint32_t (&stage)[kStageWords + kChunkWordsMax + 8] = local.stage;
    // threads 0..255 stand for the 256 symbols while the tables are built; the others only fill and wait
    const uint32_t s = threadIdx.x, wave = s >> 6, lane = s & 63u;
    const bool symbol = s < 256u;
    uint32_t l = symbol ? len_in[s] : 0u;
    if (l > (uint32_t)kMaxLen) l = 0u;
    // thread s is symbol s: its rank among the symbols of its length, by lane masks inside the wave ...
    uint32_t before = 0;
#pragma unroll
    for (int k = 1; k <= kMaxLen; ++k) {
        const uint64_t same = __ballot(l == (uint32_t)k);
        if (l == (uint32_t)k) before = __builtin_amdgcn_mbcnt_hi((uint32_t)(same >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)same, 0u));
        if (lane == 0 && symbol) in_wave[wave][k] = (uint32_t)__popcll(same);
    }
    __syncthreads();
    if (s < (uint32_t)kMaxLen + 2u) {
        uint32_t total = 0;
        if (s >= 1u && s <= (uint32_t)kMaxLen)
            for (int w = 0; w < kThreads / 64; ++w) total += in_wave[w][s];
        per_length[s] = total;
    }
    __syncthreads();
    if (s == 0) {
        uint32_t count[kMaxLen + 1];
#pragma unroll
        for (int k = 1; k <= kMaxLen; ++k) count[k] = per_length[k];
        uint32_t code = 0, at = 0;
        first[0] = first[1] = 0u;
        start[0] = start[1] = 0u;
#pragma unroll
        for (int k = 2; k <= kMaxLen; ++k) {
            code = (code + count[k - 1]) << 1;
            at += count[k - 1];
            first[k] = code;
            start[k] = at;
        }
    }
    __syncthreads();
    if (l) {                                                  // ... plus those in the waves below
        for (uint32_t w = 0; w < wave; ++w) before += in_wave[w][l];
        sorted[(start[l] + before) & 0xffu] = (uint8_t)s;
    }
    __syncthreads();
    {
        // the short lengths' tables in registers (the same in every thread)
        uint32_t count_of[kFastBits + 1], first_of[kFastBits + 1], start_of[kFastBits + 1];
#pragma unroll
        for (int k = 1; k <= kFastBits; ++k) { count_of[k] = per_length[k]; first_of[k] = first[k]; start_of[k] = start[k]; }
        for (uint32_t i = s; i < (1u << kFastBits); i += kDecodeThreads) {  // the short codes: what the next kFastBits bits decode to
            uint32_t at = 0, length = 0;
#pragma unroll
            for (int k = kFastBits; k >= 1; --k) {                   // at most one length matches a prefix code
                const uint32_t code = i >> (kFastBits - k);
                if (count_of[k] && code >= first_of[k] && code - first_of[k] < count_of[k]) {
                    at = start_of[k] + code - first_of[k];
                    length = (uint32_t)k;
                }
            }
            fast[i] = length ? (uint16_t)(sorted[at & 0xffu] | (length << 8)) : (uint16_t)0;
        }
    }
    Lookup table;
    table.fast = fast;
    table.second = second;
    table.tables = &tables;
    table.behind = second_of(&tables);
    const LongRegs longer = long_regs(&tables);
    for (uint32_t i = s; i < table.behind.entries; i += kDecodeThreads) {
        const uint32_t width = (uint32_t)kFastBits + table.behind.extra;
        const uint32_t e = decode_long((table.behind.from + i) << (32u - width), longer, &tables);
        second[i] = (e >> 8) <= width ? (uint16_t)e : (uint16_t)0;
    }
    __syncthreads();

    // These tables serve `chunks_per_block` chunks, in passes of as many chunks as there are threads at most.  The payload words of consecutive chunks are one contiguous slice.  A pass takes the chunks whose
    // slice fits the stage -- all of them up to 46 (64) words per chunk on average, fewer on streams that hardly
    // compress, where the threads beyond sit the pass out -- brings the slice into LDS with contiguous loads, and
    // the threads read their words from there (a thread walking its chunk in memory would fetch a cache line per
    // word).  A pass that could seat few of its chunks, and offsets that do not describe a slice (no encoder wrote
    // them), go through per-thread rings instead.
    const uint64_t share = job.chunks_per_block;
    const uint32_t chunk_stop = (uint32_t)((block + 1u) * share < chunks ? (block + 1u) * share : chunks);
    for (uint32_t chunk0 = (uint32_t)(block * share < chunks ? block * share : chunks); chunk0 < chunk_stop;) {
        const uint32_t want = chunk_stop - chunk0 < (uint32_t)kDecodeThreads ? chunk_stop - chunk0 : (uint32_t)kDecodeThreads;
        const uint32_t slice_at = offsets[chunk0];
        // the chunks before the first whose end lies outside the stage (or the payload, or before the slice's start)
        const bool asked = threadIdx.x < want;
        const uint32_t my_end = asked ? offsets[chunk0 + threadIdx.x + 1u] : 0u;
        const bool fits = my_end >= slice_at && my_end - slice_at <= (uint32_t)kStageWords && my_end <= payload_words;
        if (threadIdx.x == 0) local.fitting = want;
        __syncthreads();
        {
            const uint64_t beyond = __ballot(asked && !fits);
            if (beyond && lane == 0) atomicMin(&local.fitting, wave * 64u + (uint32_t)__builtin_ctzll(beyond));
        }
        __syncthreads();
        const uint32_t fitting = local.fitting;
        // (workgroup-uniform) Below three quarters of the threads the rings do better: at eight bits per symbol every
        // chunk is 64 words long, the threads' words lie 64 apart in the stage and all in one LDS bank.
        const bool staged = fitting > 0u && 4u * fitting >= 3u * want;
        const uint32_t take = staged ? fitting : want;        // chunks of this pass
        const uint32_t slice_end = staged ? offsets[chunk0 + fitting] : slice_at;
        const uint32_t chunk = chunk0 + threadIdx.x;
        const bool live = threadIdx.x < take;
        const uint64_t base = (uint64_t)chunk * kChunk;
        const uint32_t valid = !live ? 0u : n - base < (uint64_t)kChunk ? (uint32_t)(n - base) : (uint32_t)kChunk;
        const uint32_t first_word = live ? offsets[chunk] : 0u;
        uint8_t* dst = out + base;
        if (staged) {                                         // workgroup-uniform
            // 16 bytes per load, twelve loads of a thread in flight: one at a time, a slice of ~50 words per thread
            // would cost as many memory latencies.  The stage starts at the 16-byte boundary at or below the
            // slice's first word (`phase` words earlier); what the vectors cover beyond the payload's ends is
            // read as zero.
            const uint32_t slice_words = slice_end - slice_at;
            const uint32_t phase = (uint32_t)(reinterpret_cast<uintptr_t>(payload + slice_at) >> 2) & 3u;
            const uint32_t vectors = (slice_words + phase + 3u) / 4u;
            for (uint32_t v0 = 0; v0 < vectors; v0 += 12u * kDecodeThreads) {
                u32x4 got[12];
#pragma unroll
                for (int k = 0; k < 12; ++k) {
                    const uint32_t v = v0 + k * kDecodeThreads + threadIdx.x;
                    const int64_t w = (int64_t)slice_at + 4 * (int64_t)v - phase;  // below zero in the first vector at most
                    const auto word_at = [&](int64_t g) { return g >= 0 && g < (int64_t)payload_words ? payload[g] : 0u; };
                    got[k] = u32x4{0u, 0u, 0u, 0u};
                    if (v < vectors) {
                        if (w >= 0 && w + 3 < (int64_t)payload_words) got[k] = *reinterpret_cast<const u32x4*>(payload + w);
                        else got[k] = u32x4{word_at(w), word_at(w + 1), word_at(w + 2), word_at(w + 3)};
                    }
                }
#pragma unroll
                for (int k = 0; k < 12; ++k) {
                    const uint32_t v = v0 + k * kDecodeThreads + threadIdx.x;
                    if (v < vectors) *reinterpret_cast<u32x4*>(stage + 4u * v) = got[k];
                }
            }
            __syncthreads();
            // anything at all for a foreign stream: clamped, the reads stay inside the array (a chunk is at most 192 words)
            const uint32_t at = first_word - slice_at < slice_words ? first_word - slice_at : slice_words;
            decode_chunk_staged(valid, dst, table, stage + phase + at);
        } else if (live) {
            // a ring of eight words per thread: when four have been consumed, the four loaded at the
            // previous refill take their place and the next four are requested, so a load has the time
            // of four words' decoding to arrive
            uint32_t* mine = stage + threadIdx.x;             // word k of the ring at mine[(k & 7) * kDecodeThreads]
            uint32_t pending[4];
#pragma unroll
            for (int k = 0; k < 8; ++k) mine[k * kDecodeThreads] = first_word + k < payload_words ? payload[first_word + k] : 0u;
#pragma unroll
            for (int k = 0; k < 4; ++k) pending[k] = first_word + 8 + k < payload_words ? payload[first_word + 8 + k] : 0u;
            decode_chunk(valid, dst, table, [&](uint32_t taken) {
                if ((taken & 3u) == 0u && taken != 0u) {      // a block of four used up: refill the half of the ring just freed
                    const uint32_t slot = (taken + 4u) & 7u;
#pragma unroll
                    for (int k = 0; k < 4; ++k) mine[((slot + k) & 7u) * kDecodeThreads] = pending[k];
                    const uint32_t at = first_word + taken + 8u;
#pragma unroll
                    for (int k = 0; k < 4; ++k) pending[k] = at + k < payload_words ? payload[at + k] : 0u;
                }
                return mine[(taken & 7u) * kDecodeThreads];
            });
        }
        __syncthreads();                                      // the stage is the next pass's
        chunk0 += take;
    }
}

bool aligned(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }
uint64_t chunks_of(uint64_t n) { return (n + kChunk - 1) / kChunk; }
uint64_t groups_of(uint64_t n) { return (chunks_of(n) + kThreads - 1) / kThreads; }
constexpr uint64_t kMaxSymbols = ((uint64_t)1 << 32) - 1;

}  // namespace
}  // namespace fh

extern "C" {

size_t fh_huffman_stream_bytes(uint64_t n)
{
    if (n > fh::kMaxSymbols) return 0;
    return (size_t)(256u + 4u * (fh::chunks_of(n) + 1u) + 4u * (uint64_t)fh::kChunkWordsMax * fh::chunks_of(n));
}

size_t fh_huffman_workspace_bytes(uint64_t n)
{
    if (n > fh::kMaxSymbols) return 0;
    return (size_t)(4u * (256u + 256u + (fh::groups_of(n) > 0 ? fh::groups_of(n) : 1u)));
}

int32_t fh_huffman_batch_capacity(void) { return fh::kBatch; }

}  // extern "C"

namespace {

using namespace fh;

fh_status check_encode(const fh_huffman_encode_item& it)
{
    if (it.n > kMaxSymbols) return FH_ERR_BAD_NUMEL;
    if (!it.stream_out || !it.totals || !it.workspace || (it.n > 0 && !it.bytes)) return FH_ERR_NULL;
    if (!aligned(it.bytes, 16) || !aligned(it.stream_out, 16) || !aligned(it.totals, 8) || !aligned(it.workspace, 16) ||
        !aligned(it.n_device, 8))
        return FH_ERR_ALIGNMENT;
    if (it.stream_cap < fh_huffman_stream_bytes(it.n) || it.workspace_cap < fh_huffman_workspace_bytes(it.n))
        return FH_ERR_BUFFER_TOO_SMALL;
    return FH_OK;
}

fh_status check_decode(const fh_huffman_decode_item& it)
{
    if (it.n > kMaxSymbols) return FH_ERR_BAD_NUMEL;
    if (it.n == 0) return FH_OK;
    if (!it.stream_in || !it.out) return FH_ERR_NULL;
    if (!aligned(it.stream_in, 16) || !aligned(it.out, 16) || !aligned(it.n_device, 8)) return FH_ERR_ALIGNMENT;
    if (it.out_cap < it.n) return FH_ERR_BUFFER_TOO_SMALL;
    // not even the lengths and the offsets (with the count on the device: of the largest stream it may describe)
    if (it.stream_bytes < 256u + 4u * (chunks_of(it.n) + 1u)) return FH_ERR_BUFFER_TOO_SMALL;
    return FH_OK;
}

template <typename Kernel, typename Item>
void launch(Kernel kernel, const Batch<Item>& b, uint32_t grid, hipStream_t s)
{
    if (grid > 0) hipLaunchKernelGGL(kernel, dim3(grid), dim3(kThreads), 0, s, b);
}


}  // namespace

extern "C" {

fh_status fh_huffman_encode_batch(const fh_huffman_encode_item* items, int32_t count, void* stream)
{
    if (count < 0) return FH_ERR_BAD_COUNT;
    if (count > 0 && !items) return FH_ERR_NULL;
    for (int32_t i = 0; i < count; ++i) {                     // everything is checked before the first launch
        const fh_status st = check_encode(items[i]);
        if (st != FH_OK) return st;
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    for (int32_t i = 0; i < count;) {
        // the same streams three times: a workgroup each | by histogram workgroups | by groups of chunks
        Batch<Layout> each, hist, grouped;
        reset(each); reset(hist); reset(grouped);
        while (i < count && each.count < kBatch) {
            const fh_huffman_encode_item& it = items[i];
            Layout lay;
            lay.chunks = (uint32_t)chunks_of(it.n);
            lay.groups = (uint32_t)groups_of(it.n);
            lay.len = static_cast<uint8_t*>(it.stream_out);
            lay.offsets = reinterpret_cast<uint32_t*>(lay.len + 256);
            lay.payload = lay.offsets + lay.chunks + 1;
            lay.hist = static_cast<uint32_t*>(it.workspace);
            lay.table = lay.hist + 256;
            lay.group_sums = lay.table + 256;
            lay.totals = static_cast<uint64_t*>(it.totals);
            lay.in = static_cast<const uint8_t*>(it.bytes);
            lay.n = it.n;
            lay.n_dev = static_cast<const uint64_t*>(it.n_device);
            // about eight vectors per thread, more in long streams: a workgroup clears and adds up 32 KiB of
            // counters and sends 256 atomics to the stream's histogram whatever it counts
            const uint64_t want = it.n == 0 ? 0 : (it.n / 16 + 255) / 256 / 8 + 1;
            lay.hist_blocks = (uint32_t)(want < (uint64_t)kHistBlocksMax ? want : (uint64_t)kHistBlocksMax);
            if ((uint64_t)grouped.block_start[grouped.count] + lay.groups > (uint64_t)INT_MAX) {
                if (each.count == 0) return FH_ERR_BAD_NUMEL;
                break;
            }
            push(each, lay, 1);
            push(hist, lay, lay.hist_blocks);
            push(grouped, lay, lay.groups);
            ++i;
        }
        seal(each); seal(hist); seal(grouped);
        launch(huffman_clear_kernel, each, (uint32_t)each.count, s);
        launch(huffman_histogram_kernel, hist, hist.block_start[hist.count], s);
        launch(huffman_code_kernel, each, (uint32_t)each.count, s);
        launch(huffman_count_kernel, grouped, grouped.block_start[grouped.count], s);
        launch(huffman_scan_kernel, each, (uint32_t)each.count, s);
        launch(huffman_write_kernel, grouped, grouped.block_start[grouped.count], s);
    }
    if (count == 0) return FH_OK;
    return hipGetLastError() == hipSuccess ? FH_OK : FH_ERR_LAUNCH;
}

fh_status fh_huffman_decode_batch(const fh_huffman_decode_item* items, int32_t count, void* stream)
{
    if (count < 0) return FH_ERR_BAD_COUNT;
    if (count > 0 && !items) return FH_ERR_NULL;
    for (int32_t i = 0; i < count; ++i) {
        const fh_status st = check_decode(items[i]);
        if (st != FH_OK) return st;
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    // A workgroup of 768 threads (the whole LDS of a compute unit: one per unit) decodes 768 chunks at a time.
    // A call whose streams together give fewer such groups than the device has compute units would leave
    // units idle for the whole launch; it is cut into groups of 256 chunks instead (workgroups of 256 threads,
    // two per unit): three times as many units at work, each building the tables for a third of the chunks.
    uint64_t wide = 0;
    for (int32_t i = 0; i < count; ++i) wide += (chunks_of(items[i].n) + kDecodeThreads - 1) / kDecodeThreads;
    const bool small = wide < (uint64_t)kComputeUnits;
    const uint64_t per_group = small ? kDecodeThreadsSmall : kDecodeThreads;
    const uint64_t slots = small ? 2u * kComputeUnits : kComputeUnits;         // workgroups the device holds at once
    bool launched = false;
    for (int32_t i = 0; i < count;) {
        DecodeJob job[kBatch];
        uint64_t groups[kBatch], total = 0;
        int jobs = 0;
        for (; i < count && jobs < kBatch; ++i) {
            const fh_huffman_decode_item& it = items[i];
            if (it.n == 0) continue;                          // nothing to restore
            const uint64_t chunks = chunks_of(it.n);
            const uint64_t words = (it.stream_bytes - (256u + 4u * (chunks + 1u))) / 4u;
            DecodeJob& j = job[jobs];
            j.len = static_cast<const uint8_t*>(it.stream_in);
            j.offsets = reinterpret_cast<const uint32_t*>(j.len + 256);
            j.payload = j.offsets + chunks + 1;
            j.out = static_cast<uint8_t*>(it.out);
            j.n = it.n;
            j.n_dev = static_cast<const uint64_t*>(it.n_device);
            j.stream_bytes = it.stream_bytes;
            j.payload_words = (uint32_t)(words < 0xffffffffu ? words : 0xffffffffu);
            j.chunks = (uint32_t)chunks;
            groups[jobs] = (chunks + per_group - 1) / per_group;   // the decoder's own groups
            total += groups[jobs];
            ++jobs;
        }
        // A workgroup builds a stream's tables once and then decodes `chunks_per_block` chunks.  With more groups
        // in the launch than workgroups fit on the device at once, every stream gets its share of that many
        // workgroups, and its chunks are dealt out evenly among them: all of them are resident from the start and
        // finish together (their last pass seats fewer chunks), whereas a launch of 1.4 times as many would run a
        // second, mostly empty round, and whole groups per workgroup would leave compute units without any.
        Batch<DecodeJob> b;
        reset(b);
        for (int k = 0; k < jobs; ++k) {
            uint64_t blocks = total <= slots ? groups[k] : groups[k] * slots / total;
            if (blocks < 1u) blocks = 1u;
            const uint64_t chunks = job[k].chunks;
            job[k].chunks_per_block = (uint32_t)((chunks + blocks - 1u) / blocks);
            if (!push(b, job[k], (int64_t)((chunks + job[k].chunks_per_block - 1u) / job[k].chunks_per_block)))
                return FH_ERR_BAD_NUMEL;                      // cannot happen: a stream has at most 2^16 groups
        }
        seal(b);
        if (b.count > 0) {
            if (small)
                hipLaunchKernelGGL(huffman_decode_kernel<kDecodeThreadsSmall>, dim3(b.block_start[b.count]),
                                   dim3(kDecodeThreadsSmall), 0, s, b);
            else
                hipLaunchKernelGGL(huffman_decode_kernel<kDecodeThreads>, dim3(b.block_start[b.count]),
                                   dim3(kDecodeThreads), 0, s, b);
            launched = true;
        }
    }
    if (!launched) return FH_OK;
    return hipGetLastError() == hipSuccess ? FH_OK : FH_ERR_LAUNCH;
}

fh_status fh_huffman_encode(const void* bytes, uint64_t n, void* stream_out, size_t stream_cap, void* totals,
                            void* workspace, size_t workspace_cap, void* stream)
{
    fh_huffman_encode_item it;
    it.n_device = nullptr;
    it.bytes = bytes; it.n = n; it.stream_out = stream_out; it.stream_cap = stream_cap; it.totals = totals;
    it.workspace = workspace; it.workspace_cap = workspace_cap;
    return fh_huffman_encode_batch(&it, 1, stream);
}

fh_status fh_huffman_decode(const void* stream_in, size_t stream_bytes, uint64_t n, void* out, size_t out_cap,
                            void* stream)
{
    fh_huffman_decode_item it;
    it.n_device = nullptr;
    it.stream_in = stream_in; it.stream_bytes = stream_bytes; it.n = n; it.out = out; it.out_cap = out_cap;
    return fh_huffman_decode_batch(&it, 1, stream);
}

}  // extern "C"
