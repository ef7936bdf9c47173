/*
 * fedhybrid.h -- C ABI of the MI355X (gfx950) activation compressor.
 *
 * What it computes: the quantisation that FedHybrid's local training engine applies
 * to the normal (non-salient) channels of an activation saved in the forward pass,
 * and its inverse on the backward pass (paper Section 3, "Activation compression":
 * compress in forward, decompress during backpropagation; Section 4.4.1,
 * "Channel-wise Mix Compression": normal channels undergo linear-scale
 * quantisation, zeros must survive decompression).  The paper prints no formula,
 * bit width, rounding rule or layout for that quantiser; the definition used is:
 *
 *   - the flattened tensor is cut into consecutive groups of `group_size` elements
 *     (the last may be short);
 *   - per group: mn = min, mx = max, range = mx - mn, L = 2^bits - 1,
 *     zero = mn (with -0.0 stored as +0.0); if range < 2^-100 the group is
 *     degenerate: scale = 0 and every code is 0; otherwise scale = range / L and
 *     codes are taken from q = clamp((x - mn) * (L / range), 0, L) by
 *       nearest:    code = rint(q)                      (ties to even)
 *       stochastic: code = floor(q) + [u < q - floor(q)], u = h / 2^16,
 *     where h are 16 bits of Philox4x32-10 output owned by the element: key = seed,
 *     counter = (element_index / 8, tensor_id), element i taking half-word (i mod 8)
 *     of the four output words in little-endian order;
 *   - codes are bit-packed in element order, element i at bits [(i*bits) mod 8, +bits)
 *     of byte floor(i*bits/8); bytes up to fh_packed_bytes() are zero-filled;
 *   - meta is one {float scale; float zero;} pair per group;
 *   - decompression returns fmaf(code, scale, zero) (single rounding), optionally
 *     rounded to bf16 (nearest even).
 *   All arithmetic is IEEE binary32.  Inputs must be finite with |x| < 2^126.
 *
 * Conventions
 *   - Every data pointer (x, packed, meta, out) is a DEVICE pointer into memory the
 *     caller owns; the parameter and item structs are HOST memory and are read
 *     before the call returns.  The library allocates nothing, keeps no state, and
 *     never synchronises: work is enqueued on `stream` (a hipStream_t passed as
 *     void*, NULL = the default stream) and the caller orders it.
 *   - x, packed and out must be 16-byte aligned, meta 8-byte aligned.
 *   - All argument checks run on the host before anything is launched; a call that
 *     returns an error has touched no device memory.  numel == 0 is FH_OK and
 *     launches nothing.
 *   - Results are a pure function of the arguments: independent of launch geometry,
 *     of batching, and of the device the call runs on.
 */
#ifndef FEDHYBRID_H
#define FEDHYBRID_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum fh_status {
    FH_OK = 0,
    FH_ERR_NULL = 1,             /* a required pointer is NULL */
    FH_ERR_BAD_DTYPE = 2,
    FH_ERR_BAD_GROUP = 3,        /* group_size not in {64, 128, 256} */
    FH_ERR_BAD_BITS = 4,         /* bits not in {2, 4, 8} */
    FH_ERR_BAD_ROUND = 5,
    FH_ERR_BAD_NUMEL = 6,        /* negative, or too large to index */
    FH_ERR_BUFFER_TOO_SMALL = 7, /* a *_cap is below what the call writes or reads */
    FH_ERR_ALIGNMENT = 8,
    FH_ERR_LAUNCH = 9,           /* the HIP runtime refused the launch */
    FH_ERR_BAD_COUNT = 10,       /* negative item count */
    FH_ERR_BAD_SHAPE = 11,       /* outer / channels / inner / raw_channels out of range */
    FH_ERR_BAD_PARAM = 12,       /* k_sigma not positive, min_outliers < 1, a pooling window other than 2, 4, 8,
                                    or a reserved field that is not 0 */
    FH_ERR_SCRATCH_LIMIT = 13    /* the tensor needs more scratch than the library's static buffer holds */
} fh_status;

typedef enum fh_dtype { FH_F32 = 0, FH_BF16 = 1 } fh_dtype;
typedef enum fh_round { FH_ROUND_NEAREST = 0, FH_ROUND_STOCHASTIC = 1 } fh_round;

/* Quantiser parameters of one tensor (host memory). */
typedef struct fh_params {
    int32_t  group_size;   /* 64 | 128 | 256 contiguous elements */
    int32_t  bits;         /* 2 | 4 | 8 */
    int32_t  rounding;     /* fh_round */
    int32_t  reserved;     /* must be 0 */
    uint64_t seed;         /* Philox key; read only when rounding is stochastic */
    uint64_t tensor_id;    /* upper half of the Philox counter; idem */
} fh_params;

/* One tensor of a batched call (host memory; the pointers inside are device
 * pointers).  Fields a call does not use may be NULL / 0:
 *   compress   reads x, writes packed + meta;
 *   decompress reads packed + meta, writes out;
 *   roundtrip  uses all of them. */
typedef struct fh_item {
    const void *x;          int32_t x_dtype;   int32_t out_dtype;   /* fh_dtype */
    int64_t     numel;
    void       *packed;     size_t packed_cap;  /* >= fh_packed_bytes(numel, bits) */
    void       *meta;       size_t meta_cap;    /* >= fh_meta_bytes(numel, group_size) */
    void       *out;        size_t out_cap;     /* >= numel * sizeof(out_dtype) */
    fh_params   params;
} fh_item;

/* ceil(numel * bits / 8) rounded up to a multiple of 16; 0 for numel <= 0 or bad bits. */
size_t fh_packed_bytes(int64_t numel, int32_t bits);
/* 8 * ceil(numel / group_size); 0 for numel <= 0 or group_size <= 0. */
size_t fh_meta_bytes(int64_t numel, int32_t group_size);

/* Forward side (Section 3: the activation is compressed while the forward pass runs;
 * quantiser of Section 4.4.1).  Reads numel elements of x_dtype at x, writes
 * fh_packed_bytes() bytes at packed (padding included, zero) and fh_meta_bytes()
 * bytes at meta. */
fh_status fh_compress(const void *x, fh_dtype x_dtype, int64_t numel, const fh_params *params,
                      void *packed, size_t packed_cap, void *meta, size_t meta_cap, void *stream);

/* Backward side (Section 3: the saved activation is decompressed when backpropagation
 * needs it; Section 4.4.1: floating-point values are rebuilt from the quantisation
 * codes).  Writes numel elements of out_dtype at out.  params->rounding,
 * seed and tensor_id are ignored. */
fh_status fh_decompress(const void *packed, const void *meta, int64_t numel, const fh_params *params,
                        fh_dtype out_dtype, void *out, size_t out_cap, void *stream);

/* fh_compress followed by fh_decompress on the same stream, through the caller's
 * packed/meta buffers: the memory traffic of the method as a training step incurs
 * it (the codes are written to and read back from device memory, not kept in
 * registers). */
fh_status fh_roundtrip(const void *x, fh_dtype x_dtype, int64_t numel, const fh_params *params,
                       void *packed, size_t packed_cap, void *meta, size_t meta_cap,
                       fh_dtype out_dtype, void *out, size_t out_cap, void *stream);

/* The same three operations over a set of tensors, as a training step saves and
 * restores them (Section 4.3: the plan marks many tensors of one model for
 * compression).  Tensors are processed by as few kernel launches as possible (one
 * per run of up to fh_batch_capacity() items that share dtype and group size), so
 * small tensors do not each pay a launch.  Items with numel == 0 are skipped.  All
 * items are validated before the first launch.  Results are identical to calling
 * the single-tensor entry points item by item. */
fh_status fh_compress_batch(const fh_item *items, int32_t count, void *stream);
fh_status fh_decompress_batch(const fh_item *items, int32_t count, void *stream);
fh_status fh_roundtrip_batch(const fh_item *items, int32_t count, void *stream);
int32_t   fh_batch_capacity(void);

/* ---- channel classification -------------------------------------------------------
 * Section 4.4.1 finds outliers with the empirical three-sigma rule and sorts channels
 * into salient (outlier-rich) and normal ones; normal channels are the ones the
 * quantiser above is meant for.  The paper gives the rule's name only; the definition
 * used (k and the outlier count that makes a channel salient are inputs):
 *
 *   - the tensor is viewed as [outer][channels][inner], row-major (NCHW: outer = N,
 *     inner = H*W; [tokens][hidden]: inner = 1);
 *   - S1 = sum x and S2 = sum x*x over all elements in binary64, summed PAIRWISE: the
 *     sequence in element order, zero-padded to a power of two, reduced by a balanced
 *     binary tree (this fixes every rounding, whatever the blocking);
 *   - mean = S1 / N (a total of -0.0 counts as +0.0), variance = max(S2 / N - mean*mean, 0),
 *     threshold = k*k * variance;
 *   - x is an outlier iff d*d > threshold, d = (double)x - mean;
 *   - counts[c] = outliers in channel c; mask[c] = (counts[c] >= min_outliers).
 *
 * x: device, 16-byte aligned, outer*channels*inner elements of x_dtype.
 * workspace: device, 16-byte aligned, >= fh_classify_workspace_bytes(numel) bytes,
 *   scratch for the partial sums (contents undefined afterwards).
 * stats: device, 8-byte aligned, 4 doubles {mean, variance, threshold, numel}.
 * counts: device, uint32[channels].  mask: device, uint8[channels].
 * 1 <= channels <= 16384, inner >= 1, outer >= 0.  outer == 0 zeroes the outputs.
 * Everything is enqueued on `stream`; nothing is allocated or synchronised. */
size_t    fh_classify_workspace_bytes(int64_t numel);
fh_status fh_classify_channels(const void *x, fh_dtype x_dtype, int64_t outer, int64_t channels, int64_t inner,
                               double k_sigma, int64_t min_outliers,
                               void *workspace, size_t workspace_cap,
                               void *stats, void *counts, void *mask, void *stream);

/* fh_classify_channels for callers that cannot allocate device memory and have no workspace to
 * pass: code under HIP graph capture, tight serving loops, harnesses that forbid allocation.
 * The partial sums go to a buffer that is part of the library itself (a device array of
 * fh_classify_static_scratch_bytes() = 4 MiB, held by every GPU the library runs on until the
 * process ends), so the call allocates nothing; inputs and outputs are still the caller's.
 * Results are identical to fh_classify_channels.  A tensor whose
 * fh_classify_workspace_bytes() exceeds that size (more than about 2.68e8 elements) is refused
 * with FH_ERR_SCRATCH_LIMIT before anything is launched.  All calls on one GPU share the
 * buffer: calls that may overlap on one GPU (different streams, different host threads) race;
 * calls on one stream are ordered and safe.  The device is the current one, and `stream` must
 * belong to it. */
size_t    fh_classify_static_scratch_bytes(void);
fh_status fh_classify_channels_static(const void *x, fh_dtype x_dtype, int64_t outer, int64_t channels,
                                      int64_t inner, double k_sigma, int64_t min_outliers,
                                      void *stats, void *counts, void *mask, void *stream);

/* ---- salient channels routed around the quantiser ----------------------------------------
 * Section 4.4.1 quantises only the normal channels, so that the outliers clustered in the
 * salient channels do not stretch the quantiser's range; the paper stores salient channels
 * by a sparse / predictive scheme of its own, this library keeps them verbatim ("raw")
 * beside the quantised stream.  The definition used:
 *
 *   - the tensor is viewed as [outer][channels][inner] as above; element i belongs to
 *     channel (i / inner) mod channels;
 *   - slots[c] (int16) is the row of the raw store that keeps channel c, 0 <= slot <
 *     raw_channels; any other value (fh_channel_slots writes -1) means "normal channel";
 *     no two channels may name the same row (for such a table every access still stays
 *     inside the buffers, but which of the channels the row then holds is unspecified);
 *   - fh_channel_slots numbers the channels whose mask byte is non-zero 0, 1, 2, ... in
 *     channel order; once raw_channels slots are used the remaining ones stay normal;
 *   - raw is [outer][raw_channels][inner] in the input's dtype; an element of a kept channel
 *     is copied bit for bit to raw[(o * raw_channels + slot) * inner + j]; rows of unused
 *     slots are not written;
 *   - the quantiser runs over the flattened tensor exactly as in fh_compress (same groups,
 *     same random bits per element index, same packing), except that elements of kept
 *     channels are invisible to a group's min / max and get code 0; a group without normal
 *     elements has scale = zero = 0;
 *   - fh_decompress_mixed returns fmaf(code, scale, zero) for normal elements and the raw
 *     value, converted to out_dtype (bf16 -> f32 exact, f32 -> bf16 nearest even), for
 *     elements of kept channels.
 *
 * mask: device, uint8[channels] (as fh_classify_channels writes it).  slots: device, 16-byte
 * aligned, int16[channels].  raw: device, 16-byte aligned, fh_raw_bytes() bytes.  The other
 * buffers are as in fh_compress / fh_decompress.  outer * channels * inner <= 2^31,
 * 0 <= raw_channels <= channels.  With raw_channels == 0 the result equals fh_compress's
 * and raw may be NULL.  Everything is enqueued on `stream`; nothing is allocated. */
size_t    fh_raw_bytes(int64_t outer, int64_t raw_channels, int64_t inner, fh_dtype dtype);
fh_status fh_channel_slots(const void *mask, int64_t channels, int64_t raw_channels, void *slots, void *stream);
/* The same, and *used (device uint64, 8-byte aligned) = raw-store rows in use = min(salient channels, raw_channels). */
fh_status fh_channel_slots_used(const void *mask, int64_t channels, int64_t raw_channels, void *slots, void *used,
                                void *stream);
/* The same for several tensors with one launch per fh_mixed_batch_capacity() of them (used may be NULL). */
typedef struct fh_slots_item {
    const void *mask;       int64_t channels, raw_channels;
    void       *slots;      void *used;
} fh_slots_item;
fh_status fh_channel_slots_batch(const fh_slots_item *items, int32_t count, void *stream);
fh_status fh_compress_mixed(const void *x, fh_dtype x_dtype, int64_t outer, int64_t channels, int64_t inner,
                            const fh_params *params, const void *slots, int64_t raw_channels,
                            void *packed, size_t packed_cap, void *meta, size_t meta_cap,
                            void *raw, size_t raw_cap, void *stream);
fh_status fh_decompress_mixed(const void *packed, const void *meta, const void *raw, fh_dtype raw_dtype,
                              int64_t outer, int64_t channels, int64_t inner,
                              const fh_params *params, const void *slots, int64_t raw_channels,
                              fh_dtype out_dtype, void *out, size_t out_cap, void *stream);

/* The same two calls for several tensors (one launch per run of up to fh_mixed_batch_capacity()
 * items that share dtype and group size; items with no element are skipped, items with
 * raw_channels == 0 are served by the plain quantiser's kernels; everything is checked before
 * the first launch; results identical to the single calls).  Compression uses
 * x, x_dtype, the shape, slots, raw_channels, packed, meta, raw (whose dtype is x_dtype) and
 * params; decompression uses packed, meta, raw, raw_dtype, the shape, slots, raw_channels, out,
 * out_dtype and params. */
typedef struct fh_mixed_item {
    const void *x;          int32_t x_dtype;   int32_t out_dtype;   /* fh_dtype */
    int64_t     outer, channels, inner;
    const void *slots;      int64_t raw_channels;
    void       *packed;     size_t packed_cap;
    void       *meta;       size_t meta_cap;
    void       *raw;        size_t raw_cap;    int32_t raw_dtype;   int32_t reserved;
    void       *out;        size_t out_cap;
    fh_params   params;
    const void *rows_in_use;                    /* NULL, or device uint64 (8-byte aligned): raw-store rows in use, as
                                                   fh_channel_slots_used writes it; when it reads 0 by the time the
                                                   stream reaches the call the tensor takes the plain quantiser's
                                                   code path (same bytes, no channel bookkeeping) */
} fh_mixed_item;
fh_status fh_compress_mixed_batch(const fh_mixed_item *items, int32_t count, void *stream);
fh_status fh_decompress_mixed_batch(const fh_mixed_item *items, int32_t count, void *stream);
int32_t   fh_mixed_batch_capacity(void);

/* ---- sparse-block storage of salient-channel feature maps -----------------------------------
 * Section 4.4.1 stores an outlier-rich channel block-wise: a binary mask marks the non-zero
 * values of the h x w map, average pooling with an n x n window turns it into a density per
 * block, blocks whose density does not exceed a threshold tau are sparse and are stored in
 * Compressed Sparse Row format; zeros must come back exactly.  Dense blocks (which the paper
 * hands to a predictive coder) are stored verbatim here.  The paper gives neither n, tau, the
 * pooling stride nor a layout; the definition used:
 *
 *   - input: `maps` maps of h x w elements, row-major, contiguous (for instance the raw store
 *     of fh_compress_mixed with maps = outer * raw_channels, h * w = inner);
 *   - pooling is non-overlapping: a map is cut into ceil(h/n) x ceil(w/n) blocks, edge blocks
 *     are smaller; blocks are numbered map-major, then row-major; n is 2, 4 or 8;
 *   - an element is non-zero iff its bit pattern is not all zero (-0.0 is a value);
 *     density = (float)nnz / (float)area (binary32 division), sparse iff density <= tau;
 *   - info: one byte per block, bit 7 = dense, bits 0..6 = nnz (sparse) or area (dense);
 *   - values: one stream in block order -- the non-zeros of a sparse block in row-major order,
 *     all elements of a dense block in row-major order;
 *   - indices: one byte stream in block order -- per sparse block row_ptr[0..rows] (non-zeros in
 *     the block's rows before r) followed by the column inside the block of each non-zero, in
 *     row-major order (columns ascending inside a row; the decoder relies on that order);
 *   - totals: uint64[4] = {values written, index bytes written, sparse blocks, dense blocks};
 *   - decoding restores the input bit for bit;
 *   - with eps > 0 (the same value on both calls) dense blocks take the section's predictive
 *     form instead of the verbatim one: on the lattice q = rint(x / (2 eps)) (binary32 division;
 *     an element with |x / (2 eps)| >= 2^22, NaN or infinite has no lattice point and counts as
 *     0) each element is predicted by first-order Lorenzo inside its block,
 *     p = q(left) + q(up) - q(up-left) with zeros outside the block; an element with a lattice
 *     point and |q - p| < 128 becomes the code byte q - p + 128, any other element is an
 *     outlier: code byte 0 and its original bits in the value stream.  info = 0x80 | outliers,
 *     the index stream gets the block's code bytes row-major.  Restoring returns outliers
 *     unchanged and (float)q * (2 eps) otherwise (rounded to bf16 for bf16 maps), i.e. within
 *     eps of the input up to two roundings.  eps <= 0 or NaN means verbatim.  The Huffman stage
 *     the paper puts after this is a call of its own on the index stream: fh_huffman_encode.
 *
 * All pointers are device pointers; x, values, out 4-byte aligned, totals and workspace 8-byte
 * aligned.  Stream sizes depend on the data, so the encoder wants room for the worst case:
 * info_cap >= fh_sparse_info_bytes(), values_cap >= maps*h*w elements, indices_cap >=
 * fh_sparse_index_bytes(); what was used is in totals (device memory, valid once the stream
 * has reached it).  The decoder is given the valid prefix of each stream; blocks that would
 * reach past it are zero-filled rather than read.  maps*h*w <= 2^31.  workspace:
 * fh_sparse_workspace_bytes() bytes of scratch.  Nothing is allocated or synchronised. */
size_t    fh_sparse_info_bytes(int64_t maps, int64_t h, int64_t w, int32_t n);
size_t    fh_sparse_index_bytes(int64_t maps, int64_t h, int64_t w, int32_t n);
size_t    fh_sparse_workspace_bytes(int64_t maps, int64_t h, int64_t w, int32_t n);
fh_status fh_sparse_encode(const void *x, fh_dtype dtype, int64_t maps, int64_t h, int64_t w, int32_t n, float tau,
                           float eps, void *info, size_t info_cap, void *values, size_t values_cap,
                           void *indices, size_t indices_cap, void *totals,
                           void *workspace, size_t workspace_cap, void *stream);
fh_status fh_sparse_decode(const void *info, const void *values, size_t values_bytes,
                           const void *indices, size_t indices_bytes, fh_dtype dtype,
                           int64_t maps, int64_t h, int64_t w, int32_t n, float eps,
                           void *out, size_t out_cap, void *workspace, size_t workspace_cap, void *stream);

/* The same for several tensors, as a plan classifies every compressible activation of a model:
 * each kind of kernel is launched once per run of up to fh_classify_batch_capacity() items of
 * one dtype, so small tensors do not each pay five launches.  All items are checked before the
 * first launch; results are identical to calling fh_classify_channels item by item.  The
 * items' outputs and workspaces must not overlap. */
typedef struct fh_classify_item {
    const void *x;          int32_t x_dtype;   int32_t reserved;    /* fh_dtype; 0 */
    int64_t     outer, channels, inner;
    double      k_sigma;    int64_t min_outliers;
    void       *workspace;  size_t workspace_cap;
    void       *stats;      void *counts;      void *mask;
} fh_classify_item;
fh_status fh_classify_channels_batch(const fh_classify_item *items, int32_t count, void *stream);
int32_t   fh_classify_batch_capacity(void);

/* The same for several sets of maps (the kept channels of every layer of a model): each pass is
 * launched once per run of up to fh_sparse_batch_capacity() items that share dtype and window.
 * All items are checked before the first launch; results are identical to the single calls.
 * The items' buffers must not overlap. */
typedef struct fh_sparse_encode_item {
    const void *x;        int32_t dtype;    int32_t n;             /* fh_dtype; window 2 | 4 | 8 */
    int64_t     maps, h, w;
    float       tau, eps;
    void       *info;     size_t info_cap;
    void       *values;   size_t values_cap;
    void       *indices;  size_t indices_cap;
    void       *totals;
    void       *workspace; size_t workspace_cap;
} fh_sparse_encode_item;
typedef struct fh_sparse_decode_item {
    const void *info;
    const void *values;   size_t values_bytes;
    const void *indices;  size_t indices_bytes;
    int32_t     dtype;    int32_t n;
    int64_t     maps, h, w;
    float       eps;      int32_t reserved;                        /* 0 */
    void       *out;      size_t out_cap;
    void       *workspace; size_t workspace_cap;
} fh_sparse_decode_item;
fh_status fh_sparse_encode_batch(const fh_sparse_encode_item *items, int32_t count, void *stream);
fh_status fh_sparse_decode_batch(const fh_sparse_decode_item *items, int32_t count, void *stream);
int32_t   fh_sparse_batch_capacity(void);

/* ---- Huffman coding of a byte stream -----------------------------------------------------------
 * Section 4.4.1 ends the predictive form of dense blocks with an entropy stage: the
 * quantisation codes are encoded with Huffman coding, and restoring starts with Huffman
 * decoding.  These two calls code any device byte buffer (for instance the index stream
 * fh_sparse_encode writes with eps > 0, whose code bytes cluster around 128).  The paper names
 * the coder only; the definition used:
 *
 *   - code lengths: Huffman's algorithm on the histogram of the n bytes -- the used byte values
 *     sorted by (count, value), two queues, a leaf preferred to an internal node of equal
 *     weight; unused values get length 0, a single used value length 1; while the longest code
 *     exceeds 24 bits every non-zero count c becomes (c + 1) >> 1 and the construction is
 *     repeated;
 *   - codes: canonical, by increasing (length, value);
 *   - stream: 256 length bytes; then uint32 offsets[chunks + 1], chunks = ceil(n / 256); then
 *     the payload, 32-bit words: the codes of chunk c (symbols 256 c ...) start at word
 *     offsets[c], first bit first from bit 31 of a word downwards, zero-padded to a whole word;
 *     offsets[chunks] = words in all;
 *   - totals: uint64[2] = {stream bytes used, payload bits};
 *   - decoding restores the bytes exactly.
 *
 * All pointers are device pointers, 16-byte aligned (totals 8); n < 2^32.  The encoder wants
 * stream_cap >= fh_huffman_stream_bytes(n) (the worst case) and fh_huffman_workspace_bytes(n)
 * bytes of scratch; what was used is in totals once the stream has reached it.  The decoder is
 * given the valid prefix of the stream (at least the lengths and the offsets, else
 * FH_ERR_BUFFER_TOO_SMALL); words past it read as zero.  Nothing is allocated or synchronised. */
size_t    fh_huffman_stream_bytes(uint64_t n);
size_t    fh_huffman_workspace_bytes(uint64_t n);
fh_status fh_huffman_encode(const void *bytes, uint64_t n, void *stream_out, size_t stream_cap, void *totals,
                            void *workspace, size_t workspace_cap, void *stream);
fh_status fh_huffman_decode(const void *stream_in, size_t stream_bytes, uint64_t n, void *out, size_t out_cap,
                            void *stream);

/* The same two calls for several byte buffers: every pass is launched once per run of up to
 * fh_huffman_batch_capacity() items (the code construction, a single workgroup's work per
 * buffer, then runs for all of them side by side).  Everything is checked before the first
 * launch; results identical to the single calls.
 *
 * n_device: NULL, or a device pointer (8-byte aligned) to a uint64 that holds the symbol count
 * by the time the stream reaches the call -- for a buffer whose length is itself the output of
 * an earlier call on the same stream (the index-byte total of fh_sparse_encode), so that the
 * whole chain can be enqueued without the host reading anything back.  `n` is then an upper
 * bound: buffers, capacities and launches are sized for it, and the count used is
 * min(*n_device, n).  The decoder's stream_bytes may then be the capacity of the stream buffer
 * (at least the size the encoder reported). */
typedef struct fh_huffman_encode_item {
    const void *bytes;      uint64_t n;
    void       *stream_out; size_t stream_cap;
    void       *totals;
    void       *workspace;  size_t workspace_cap;
    const void *n_device;
} fh_huffman_encode_item;
typedef struct fh_huffman_decode_item {
    const void *stream_in;  size_t stream_bytes;
    uint64_t    n;
    void       *out;        size_t out_cap;
    const void *n_device;
} fh_huffman_decode_item;
fh_status fh_huffman_encode_batch(const fh_huffman_encode_item *items, int32_t count, void *stream);
fh_status fh_huffman_decode_batch(const fh_huffman_decode_item *items, int32_t count, void *stream);
int32_t   fh_huffman_batch_capacity(void);

/* ---- the channel-wise mix compressor as one call each way ------------------------------------------
 * Section 4.4.1 describes ONE compressor -- classify channels by the three-sigma rule, quantise
 * the normal ones, store the salient ones block-wise (sparse blocks as CSR, dense blocks by
 * Lorenzo prediction within an error bound, their codes Huffman-coded) -- and Algorithm 1 knows
 * two actions, compress and decompress.  These calls enqueue that whole chain, built from the
 * calls above, on one stream without the host reading anything back:
 *
 *   fh_mix_compress    fh_classify_channels -> slots as fh_channel_slots numbers them -> the raw
 *                      store cleared (rows of unused slots are zero) -> fh_compress_mixed ->
 *                      fh_sparse_encode of the raw store viewed as `maps` maps of h x w ->
 *                      (entropy = 1) fh_huffman_encode of the index stream;
 *   fh_mix_decompress  (entropy = 1) fh_huffman_decode -> fh_sparse_decode -> fh_decompress_mixed.
 *
 * Results are identical to making those calls one by one with the same parameters.  The
 * caller owns two device buffers per tensor, both 256-byte aligned: `store`, which holds the
 * stored form from compress until decompress, and `workspace`, scratch that either call may
 * overwrite and that is free again once the call's work has run.  fh_mix_layout says how large
 * they must be (sizes for the worst case: how much of the value, index and Huffman streams is
 * in use depends on the data) and where each part lies:
 *   store      header (uint64[8]: [0..3] the sparse stage's totals {values, index bytes, sparse
 *              blocks, dense blocks}, [4..5] the Huffman stage's totals {stream bytes, payload
 *              bits}, [6] bytes the stored form occupies -- header, codes, meta and, when
 *              channels are kept, slots, info bytes, the values in use and the index or Huffman
 *              stream in use --, [7] raw-store rows in use), slots, packed, meta, info, values,
 *              then indices (entropy = 0) or the Huffman stream (entropy = 1);
 *   workspace  stats, counts, mask (as fh_classify_channels writes them), the classification's
 *              partial sums, the raw store, the sparse stage's scratch, and with entropy = 1 the
 *              plain index stream and the Huffman stage's scratch.
 * maps * h * w must equal outer * raw_channels * inner (feature maps: maps = outer *
 * raw_channels, h * w = inner; [tokens][hidden]: one map of h = tokens, w = raw_channels); with
 * raw_channels == 0 the chain is the classification followed by the plain quantiser and maps, h,
 * w, window, tau, eps and entropy are ignored.  At most 2^31 elements per tensor.  decompress
 * reads the same fields as compress (shape, parameters, store, workspace) plus out, out_dtype,
 * out_cap.  The batched calls run every stage once for all items (in runs of that stage's
 * batch capacity); everything is checked before the first launch; nothing is allocated on the
 * device or synchronised. */
typedef struct fh_mix_item {
    const void *x;          int32_t x_dtype;   int32_t out_dtype;   /* fh_dtype */
    int64_t     outer, channels, inner;
    int64_t     maps, h, w;                     /* the raw store as feature maps */
    fh_params   quant;                          /* quantiser of the normal channels */
    double      k_sigma;    int64_t min_outliers;                   /* classification */
    int64_t     raw_channels;                   /* rows of the raw store: salient channels beyond it are quantised */
    int32_t     window;     int32_t entropy;    /* pooling window 2 | 4 | 8; 1: Huffman-code the index stream */
    float       tau, eps;                       /* sparsity threshold; error bound of dense blocks (<= 0: verbatim) */
    int64_t     reserved;                       /* 0 */
    void       *store;      size_t store_cap;
    void       *workspace;  size_t workspace_cap;
    void       *out;        size_t out_cap;
} fh_mix_item;
typedef struct fh_mix_regions {
    size_t store_bytes, workspace_bytes;
    /* offsets into store (indices is 0 and unused when entropy = 1, huffman when entropy = 0) */
    size_t header, slots, packed, meta, info, values, indices, huffman;
    /* offsets into workspace */
    size_t stats, counts, mask, classify_ws, raw, sparse_ws, indices_ws, huffman_ws;
    /* sizes of the parts: exact for slots, packed, meta, info, raw; capacities for the streams */
    size_t slots_bytes, packed_bytes, meta_bytes, info_bytes, values_cap, indices_cap, huffman_cap, raw_bytes,
           classify_ws_bytes, sparse_ws_bytes, huffman_ws_bytes;
} fh_mix_regions;
fh_status fh_mix_layout(const fh_mix_item *item, fh_mix_regions *regions);   /* host only; reads shape and parameters */
fh_status fh_mix_compress(const fh_mix_item *item, void *stream);
fh_status fh_mix_decompress(const fh_mix_item *item, void *stream);
fh_status fh_mix_compress_batch(const fh_mix_item *items, int32_t count, void *stream);
fh_status fh_mix_decompress_batch(const fh_mix_item *items, int32_t count, void *stream);

const char *fh_status_string(fh_status s);

#ifdef __cplusplus
}
#endif
#endif /* FEDHYBRID_H */
