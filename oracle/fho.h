/*
 * fho.h -- CPU oracle for the group quantiser that FedHybrid applies to normal
 * (non-salient) channels of a saved activation (paper Section 4.4.1, "Channel-wise
 * Mix Compression": normal channels are quantised with the conventional linear
 * scale; Section 3, "Activation compression": compress in the forward pass,
 * decompress in the backward pass).
 *
 * THIS IS TEST INFRASTRUCTURE.  It is a plain, slow, single-threaded, scalar C
 * implementation whose only job is to say what the right answer is.  Nothing in
 * the product path may include, link or call it; only the tests, the smoke check
 * and the benchmark's CPU-baseline leg do.  It shares no code, header, table or
 * constant generator with the HIP implementation.
 *
 * All pointers are HOST pointers.  All floating-point work is IEEE-754 binary32,
 * round-to-nearest-even, no fused contraction except the one explicit fmaf in
 * decompression, no flush-to-zero (build with -ffp-contract=off).  The quantisation
 * decision is an integer decided by floating point, so it is taken in the
 * precision the kernels use (binary32) rather than in binary64.
 *
 * The paper names the quantiser but prints no formula, bit width, rounding rule or
 * storage layout for it; the definition implemented here is written out in the
 * comment of each function in fho.c.
 */
#ifndef FHO_H
#define FHO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { FHO_F32 = 0, FHO_BF16 = 1 };
enum { FHO_ROUND_NEAREST = 0, FHO_ROUND_STOCHASTIC = 1 };

/* Philox4x32-10 block function (Salmon, Moraes, Dror, Shaw: "Parallel random
 * numbers: as easy as 1, 2, 3", SC'11, Section 3.3 and Table 2). */
void fho_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]);

/* The 16 random bits that stochastic rounding spends on element `index` of the
 * tensor `tensor_id` under `seed`. */
uint32_t fho_random16(uint64_t seed, uint64_t tensor_id, uint64_t index);

/* ceil(numel*bits/8) rounded up to a multiple of 16; 8 bytes per group. */
size_t fho_packed_bytes(int64_t numel, int bits);
size_t fho_meta_bytes(int64_t numel, int group_size);

/* Forward side.  x: numel elements of `dtype` (bf16 as uint16 bit patterns).
 * packed: fho_packed_bytes() bytes, fully written (padding zero).
 * meta: 2 floats per group, {scale, zero}.  Returns 0, or -1 on a bad argument. */
int fho_compress(const void *x, int dtype, int64_t numel, int group_size, int bits,
                 int rounding, uint64_t seed, uint64_t tensor_id,
                 uint8_t *packed, float *meta);

/* Backward side.  out: numel elements of `out_dtype`. */
int fho_decompress(const uint8_t *packed, const float *meta, int64_t numel,
                   int group_size, int bits, int out_dtype, void *out);

/* The unpacked code of every element (one byte each), for tests that look at codes. */
int fho_unpack_codes(const uint8_t *packed, int64_t numel, int bits, uint8_t *codes);

/* ---- channel classification (fho_classify.c; Section 4.4.1: 3-sigma rule, salient vs
 *      normal channels) ---- */

/* Pairwise (balanced binary tree, natural order, zero padded) binary64 sums of x and x*x. */
void fho_pairwise_moments(const void *x, int dtype, int64_t numel, double *s1_out, double *s2_out);

/* Tensor viewed as [outer][channels][inner].  stats = {mean, variance, threshold, numel};
 * counts[channels] = outliers per channel; mask[channels] = 1 for salient channels
 * (count >= min_outliers).  Returns 0, or -1 on a bad argument. */
int fho_classify_channels(const void *x, int dtype, int64_t outer, int64_t channels, int64_t inner,
                          double k_sigma, int64_t min_outliers,
                          double stats[4], uint32_t *counts, uint8_t *mask);

/* ---- salient channels routed around the quantiser (fho_mixed.c; Section 4.4.1: only normal
 *      channels are quantised; salient channels are kept verbatim here) ---- */

/* slots[c] = 0, 1, 2, ... for salient channels in channel order while fewer than raw_channels
 * are in use, -1 for every other channel.  Returns the number of slots used, or -1. */
int64_t fho_channel_slots(const uint8_t *mask, int64_t channels, int64_t raw_channels, int16_t *slots);

/* Tensor viewed as [outer][channels][inner].  raw: [outer][raw_channels][inner] elements of
 * `dtype`; rows of unused slots are left untouched.  packed / meta as in fho_compress. */
int fho_compress_mixed(const void *x, int dtype, int64_t outer, int64_t channels, int64_t inner,
                       const int16_t *slots, int64_t raw_channels,
                       int group_size, int bits, int rounding, uint64_t seed, uint64_t tensor_id,
                       uint8_t *packed, float *meta, void *raw);

int fho_decompress_mixed(const uint8_t *packed, const float *meta, const void *raw, int raw_dtype,
                         int64_t outer, int64_t channels, int64_t inner,
                         const int16_t *slots, int64_t raw_channels,
                         int group_size, int bits, int out_dtype, void *out);

/* ---- sparse-block storage of salient-channel feature maps (fho_sparse.c; Section 4.4.1:
 *      non-zero mask, n x n average pooling against a threshold tau, sparse blocks as CSR) ---- */

/* maps * ceil(h/n) * ceil(w/n), or -1. */
int64_t fho_sparse_blocks(int64_t maps, int64_t h, int64_t w, int n);

/* x: [maps][h][w] elements of dtype.  info: one byte per block.  values: room for maps*h*w
 * elements.  indices: room for blocks*(n+1) + maps*h*w bytes.  totals = {values written, index
 * bytes written, sparse blocks, dense blocks}.  eps > 0: dense blocks are stored by Lorenzo
 * prediction with error bound eps (outliers intact) instead of verbatim.  Returns 0, or -1 on
 * a bad argument. */
int fho_sparse_encode(const void *x, int dtype, int64_t maps, int64_t h, int64_t w, int n, float tau, float eps,
                      uint8_t *info, void *values, uint8_t *indices, uint64_t totals[4]);

/* out: [maps][h][w].  Returns 0, -1 on a bad argument, -2 on an inconsistent stream. */
int fho_sparse_decode(const uint8_t *info, const void *values, const uint8_t *indices, int dtype,
                      int64_t maps, int64_t h, int64_t w, int n, float eps, void *out);

/* ---- Huffman coding of a byte stream (fho_huffman.c; Section 4.4.1: the quantisation codes of
 *      the predictive form are encoded with Huffman coding, and restored by Huffman decoding) ----
 * Code lengths: Huffman's algorithm on the byte histogram (leaves sorted by (count, symbol),
 * two queues, a leaf preferred to an internal node of equal weight); unused symbols have
 * length 0, a single used symbol length 1; while the longest code exceeds 24 bits every
 * non-zero count c becomes (c + 1) >> 1 and the construction is repeated.  Codes: canonical, by
 * increasing (length, symbol).  Stream: len[256] bytes, then uint32 offsets[chunks + 1]
 * (chunks of 256 symbols; offsets in 32-bit words into the payload), then the payload: each
 * chunk's codes written first bit first from bit 31 of its first word downwards, zero-padded
 * to a whole word. */
void   fho_huffman_lengths(const uint64_t hist[256], uint8_t len[256]);
void   fho_huffman_codes(const uint8_t len[256], uint32_t code[256]);
size_t fho_huffman_stream_bytes(uint64_t n);        /* room the encoder wants for n symbols */
/* totals = {stream bytes used, payload bits}.  Returns 0, or -1 on a bad argument. */
int    fho_huffman_encode(const uint8_t *in, uint64_t n, uint8_t *stream, uint64_t totals[2]);
/* Returns 0, -1 on a bad argument, -2 on a stream that does not decode to n symbols. */
int    fho_huffman_decode(const uint8_t *stream, uint64_t stream_bytes, uint64_t n, uint8_t *out);

#ifdef __cplusplus
}
#endif
#endif /* FHO_H */
