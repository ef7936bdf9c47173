/*
 * fho_mixed.c -- CPU oracle for routing salient channels around the quantiser
 * (paper Section 4.4.1, "Channel-wise Mix Compression": channels are split into
 * outlier-rich (salient) and normal ones; only normal channels, whose values are
 * concentrated, go through the linear-scale quantiser, so that outliers do not stretch
 * its range).
 *
 * THIS IS TEST INFRASTRUCTURE (see fho.h).  Plain scalar C, host pointers.
 *
 * The paper stores salient channels by a sparse / predictive scheme of its own; here
 * they are kept verbatim ("raw") beside the quantised stream.  The definition:
 *
 *   view      the tensor is [outer][channels][inner], row-major; element i belongs to
 *             channel c(i) = (i / inner) mod channels, sample o(i) = i / (inner*channels),
 *             position j(i) = i mod inner.
 *   slots     slots[c] is -1 for a normal channel, else the row (0 <= slot < raw_channels)
 *             of the raw store that keeps channel c.  fho_channel_slots() derives it from a
 *             salient mask: salient channels get slots 0, 1, 2, ... in channel order; once
 *             raw_channels slots are used up the remaining salient channels are treated as
 *             normal.  A slot outside [0, raw_channels) also means normal.
 *   raw       raw is [outer][raw_channels][inner] in the input's dtype; an element of a
 *             kept channel is copied bit for bit to raw[(o*raw_channels + slot)*inner + j].
 *             Rows of unused slots are not written.
 *   quantise  groups are runs of group_size consecutive elements of the flattened tensor,
 *             exactly as in fho_compress.  Within a group, min and max are taken over the
 *             NORMAL elements only; a group without normal elements has scale = zero = 0.
 *             Everything else (degenerate range, scale, inverse, rounding, the random bits
 *             of element i, bit packing, padding) is as in fho_compress.  Elements of kept
 *             channels get code 0.
 *   restore   a normal element is fmaf(code, scale, zero) as in fho_decompress; an element
 *             of a kept channel is its raw value converted to the output dtype (same dtype:
 *             the same bits; bf16 -> f32: exact widening; f32 -> bf16: nearest even).
 */
#include "fho.h"

#include <math.h>
#include <string.h>

static float mixed_load(const void *x, int dtype, int64_t i)
{
    if (dtype == FHO_F32) return ((const float *)x)[i];
    uint32_t bits = (uint32_t)((const uint16_t *)x)[i] << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return f;
}

static uint16_t mixed_to_bf16(float f)
{
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

int64_t fho_channel_slots(const uint8_t *mask, int64_t channels, int64_t raw_channels, int16_t *slots)
{
    if (channels < 1 || channels > 16384 || raw_channels < 0 || raw_channels > channels) return -1;
    if (!mask || !slots) return -1;
    int64_t used = 0;
    for (int64_t c = 0; c < channels; ++c) {
        if (mask[c] != 0 && used < raw_channels) slots[c] = (int16_t)used++;
        else slots[c] = -1;
    }
    return used;
}

/* the raw-store row of channel c, or -1 */
static int64_t kept_slot(const int16_t *slots, int64_t c, int64_t raw_channels)
{
    int64_t s = slots[c];
    return (s >= 0 && s < raw_channels) ? s : -1;
}

static int mixed_args_ok(int64_t outer, int64_t channels, int64_t inner, int64_t raw_channels,
                         int group_size, int bits)
{
    if (outer < 0 || channels < 1 || channels > 16384 || inner < 1) return 0;
    if (raw_channels < 0 || raw_channels > channels) return 0;
    if (group_size != 64 && group_size != 128 && group_size != 256) return 0;
    if (bits != 2 && bits != 4 && bits != 8) return 0;
    return 1;
}

int fho_compress_mixed(const void *x, int dtype, int64_t outer, int64_t channels, int64_t inner,
                       const int16_t *slots, int64_t raw_channels,
                       int group_size, int bits, int rounding, uint64_t seed, uint64_t tensor_id,
                       uint8_t *packed, float *meta, void *raw)
{
    if (!mixed_args_ok(outer, channels, inner, raw_channels, group_size, bits)) return -1;
    if (dtype != FHO_F32 && dtype != FHO_BF16) return -1;
    if (rounding != FHO_ROUND_NEAREST && rounding != FHO_ROUND_STOCHASTIC) return -1;
    const int64_t numel = outer * channels * inner;
    if (numel == 0) return 0;
    if (!x || !slots || !packed || !meta || (raw_channels > 0 && !raw)) return -1;

    const float Lf = (float)((1 << bits) - 1);
    const float tiny = 0x1p-100f;
    memset(packed, 0, fho_packed_bytes(numel, bits));

    /* salient channels: verbatim copies */
    for (int64_t i = 0; i < numel; ++i) {
        int64_t run = i / inner, j = i % inner, c = run % channels, o = run / channels;
        int64_t s = kept_slot(slots, c, raw_channels);
        if (s < 0) continue;
        int64_t dst = (o * raw_channels + s) * inner + j;
        if (dtype == FHO_F32) ((uint32_t *)raw)[dst] = ((const uint32_t *)x)[i];
        else ((uint16_t *)raw)[dst] = ((const uint16_t *)x)[i];
    }

    /* normal channels: the group quantiser, blind to the elements of kept channels */
    int64_t g = 0;
    for (int64_t start = 0; start < numel; start += group_size, ++g) {
        int64_t end = start + group_size < numel ? start + group_size : numel;
        int have = 0;
        float mn = 0.0f, mx = 0.0f;
        for (int64_t i = start; i < end; ++i) {
            if (kept_slot(slots, (i / inner) % channels, raw_channels) >= 0) continue;
            float v = mixed_load(x, dtype, i);
            if (!have) { mn = mx = v; have = 1; }
            if (v < mn) mn = v;
            if (v > mx) mx = v;
        }
        if (!have) { meta[2 * g] = 0.0f; meta[2 * g + 1] = 0.0f; continue; }
        float range = mx - mn;
        int degenerate = range < tiny;
        float scale = degenerate ? 0.0f : range / Lf;
        float inv = degenerate ? 0.0f : Lf / range;
        meta[2 * g + 0] = scale;
        meta[2 * g + 1] = mn + 0.0f;
        if (degenerate) continue;
        for (int64_t i = start; i < end; ++i) {
            if (kept_slot(slots, (i / inner) % channels, raw_channels) >= 0) continue;
            float q = (mixed_load(x, dtype, i) - mn) * inv;
            if (q < 0.0f) q = 0.0f;
            if (q > Lf) q = Lf;
            uint32_t code;
            if (rounding == FHO_ROUND_NEAREST) {
                code = (uint32_t)rintf(q);
            } else {
                float k = floorf(q);
                float f = q - k;
                float u = (float)fho_random16(seed, tensor_id, (uint64_t)i) * 0x1p-16f;
                code = (uint32_t)k + (u < f ? 1u : 0u);
            }
            uint64_t bitpos = (uint64_t)i * (uint64_t)bits;
            packed[bitpos >> 3] |= (uint8_t)(code << (bitpos & 7u));
        }
    }
    return 0;
}

int fho_decompress_mixed(const uint8_t *packed, const float *meta, const void *raw, int raw_dtype,
                         int64_t outer, int64_t channels, int64_t inner,
                         const int16_t *slots, int64_t raw_channels,
                         int group_size, int bits, int out_dtype, void *out)
{
    if (!mixed_args_ok(outer, channels, inner, raw_channels, group_size, bits)) return -1;
    if (raw_dtype != FHO_F32 && raw_dtype != FHO_BF16) return -1;
    if (out_dtype != FHO_F32 && out_dtype != FHO_BF16) return -1;
    const int64_t numel = outer * channels * inner;
    if (numel == 0) return 0;
    if (!packed || !meta || !slots || !out || (raw_channels > 0 && !raw)) return -1;

    const uint32_t code_mask = (1u << bits) - 1u;
    for (int64_t i = 0; i < numel; ++i) {
        int64_t run = i / inner, j = i % inner, c = run % channels, o = run / channels;
        int64_t s = kept_slot(slots, c, raw_channels);
        if (s >= 0) {
            int64_t src = (o * raw_channels + s) * inner + j;
            if (raw_dtype == out_dtype) {
                if (out_dtype == FHO_F32) ((uint32_t *)out)[i] = ((const uint32_t *)raw)[src];
                else ((uint16_t *)out)[i] = ((const uint16_t *)raw)[src];
            } else if (out_dtype == FHO_F32) {
                ((float *)out)[i] = mixed_load(raw, FHO_BF16, src);
            } else {
                ((uint16_t *)out)[i] = mixed_to_bf16(((const float *)raw)[src]);
            }
            continue;
        }
        uint64_t bitpos = (uint64_t)i * (uint64_t)bits;
        uint32_t code = ((uint32_t)packed[bitpos >> 3] >> (bitpos & 7u)) & code_mask;
        int64_t g = i / group_size;
        float v = fmaf((float)code, meta[2 * g], meta[2 * g + 1]);
        if (out_dtype == FHO_F32) ((float *)out)[i] = v;
        else ((uint16_t *)out)[i] = mixed_to_bf16(v);
    }
    return 0;
}
