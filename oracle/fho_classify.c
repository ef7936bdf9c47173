/*
 * fho_classify.c -- CPU oracle for the channel classification step of FedHybrid's
 * Channel-wise Mix Compression (paper Section 4.4.1): outliers are identified with the
 * empirical 3-sigma rule, and channels are classified into outlier-rich (salient) and
 * normal ones; normal channels go to the quantiser (fho.c).
 *
 * THIS IS TEST INFRASTRUCTURE (see fho.h).  Plain scalar C, host pointers.
 *
 * The paper gives the rule's name only.  The definition implemented here:
 *
 *   view      the tensor is [outer][channels][inner], row-major (NCHW: outer = N,
 *             inner = H*W; a [tokens][hidden] activation: inner = 1).
 *   moments   S1 = sum x, S2 = sum x*x over ALL elements, in binary64.  x*x is exact
 *             in binary64 (24-bit significands).  Sums are PAIRWISE: the sequence, in
 *             element order and padded with zeros to a power of two, is reduced by a
 *             balanced binary tree, s[i] = s[2i] + s[2i+1] level by level.  (This fixes
 *             the rounding of every partial sum while leaving a parallel machine free
 *             to form it in any blocking aligned to powers of two.)
 *   spread    mean = S1 / N (a total of -0.0, which only an all-negative-zero tensor gives and
 *             whose sign would depend on how far the sequence is padded, counts as +0.0),
 *             variance = max(S2 / N - mean*mean, 0),
 *             threshold = (k*k) * variance        -- no square root is taken.
 *   outlier   element x is an outlier iff d*d > threshold with d = (double)x - mean,
 *             i.e. |x - mean| > k*sigma up to the rounding of these binary64 steps.
 *   count     count[c] = number of outliers over the outer*inner elements of channel c.
 *   classify  salient[c] = (count[c] >= min_outliers), min_outliers >= 1.
 *
 * The parameters the paper omits (k, defaulting to 3 by the rule's name, and how many
 * outliers make a channel "outlier-rich") are inputs.
 */
#include "fho.h"

#include <string.h>

static double elem_as_double(const void *x, int dtype, int64_t i)
{
    if (dtype == FHO_F32) return (double)((const float *)x)[i];
    uint32_t bits = (uint32_t)((const uint16_t *)x)[i] << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

/* Pairwise sums of x and x*x.  The tree is walked with one pending partial per level:
 * element i completes, at every level whose bit of i is set, the node whose left half
 * is pending there.  What is still pending at the end are left halves whose right half
 * is all padding (zeros), so they rise unchanged and join the next pending level above. */
void fho_pairwise_moments(const void *x, int dtype, int64_t numel, double *s1_out, double *s2_out)
{
    double p1[64], p2[64];
    int have[64];
    memset(have, 0, sizeof have);
    for (int64_t i = 0; i < numel; ++i) {
        double v = elem_as_double(x, dtype, i);
        double a = v, b = v * v;
        int level = 0;
        while ((i >> level) & 1) {
            a = p1[level] + a;
            b = p2[level] + b;
            have[level] = 0;
            ++level;
        }
        p1[level] = a;
        p2[level] = b;
        have[level] = 1;
    }
    double a = 0.0, b = 0.0;
    int any = 0;
    for (int level = 0; level < 64; ++level) {
        if (!have[level]) continue;
        if (!any) { a = p1[level]; b = p2[level]; any = 1; }
        else { a = p1[level] + a; b = p2[level] + b; }
    }
    *s1_out = a;
    *s2_out = b;
}

/* stats: {mean, variance, threshold, numel}.  counts: channels x uint32.  mask: channels x uint8. */
int fho_classify_channels(const void *x, int dtype, int64_t outer, int64_t channels, int64_t inner,
                          double k_sigma, int64_t min_outliers,
                          double stats[4], uint32_t *counts, uint8_t *mask)
{
    if (outer < 0 || channels < 1 || inner < 1 || min_outliers < 1 || !(k_sigma > 0.0)) return -1;
    if (dtype != FHO_F32 && dtype != FHO_BF16) return -1;
    const int64_t numel = outer * channels * inner;
    memset(counts, 0, (size_t)channels * sizeof *counts);
    memset(mask, 0, (size_t)channels);
    stats[0] = stats[1] = stats[2] = 0.0;
    stats[3] = (double)numel;
    if (numel == 0) return 0;

    double s1, s2;
    fho_pairwise_moments(x, dtype, numel, &s1, &s2);
    const double n = (double)numel;
    const double mean = (s1 + 0.0) / n;            /* a total of -0.0 counts as +0.0 */
    const double mean_sq = mean * mean;
    double variance = s2 / n - mean_sq;
    if (!(variance > 0.0)) variance = 0.0;
    const double threshold = (k_sigma * k_sigma) * variance;
    stats[0] = mean;
    stats[1] = variance;
    stats[2] = threshold;

    for (int64_t o = 0; o < outer; ++o)
        for (int64_t c = 0; c < channels; ++c)
            for (int64_t j = 0; j < inner; ++j) {
                double d = elem_as_double(x, dtype, (o * channels + c) * inner + j) - mean;
                if (d * d > threshold) counts[c] += 1u;
            }
    for (int64_t c = 0; c < channels; ++c)
        mask[c] = (int64_t)counts[c] >= min_outliers ? 1 : 0;
    return 0;
}
