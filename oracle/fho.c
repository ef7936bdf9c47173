/*
 * fho.c -- CPU oracle (test infrastructure; see fho.h).  Plain scalar C, one
 * element at a time, no blocking, no vector intrinsics, no threads.
 *
 * The encoding, step by step (paper Section 4.4.1 names a linear-scale quantiser
 * for normal channels and requires that zeros survive decompression; Section 3
 * fixes the forward/backward roles; every parameter the paper leaves open is an
 * input):
 *
 *   groups    consecutive runs of G elements of the flattened tensor; the last
 *             one may be short and uses its real elements only.
 *   range     mn = min, mx = max of the group; range = mx - mn; L = 2^B - 1.
 *   meta      zero = mn + 0.0f (so that -0.0 is stored as +0.0);
 *             range < 2^-100 (constant, all-zero, vanishing)  -> scale = 0;
 *             otherwise scale = range / L and inv = L / range.
 *   quantise  q = clamp((x - mn) * inv, 0, L);
 *             nearest:    code = rint(q), ties to even;
 *             stochastic: code = floor(q) + [u < q - floor(q)], u = h / 2^16,
 *                         h = 16 random bits owned by the element.
 *   pack      element i sits in bits [(i*B) mod 8, +B) of byte floor(i*B/8).
 *   restore   x^ = fmaf(code, scale, zero); bf16 output rounds that to nearest even.
 */
#include "fho.h"

#include <math.h>
#include <string.h>

/* ---- Philox4x32-10 (SC'11 paper, Section 3.3: the round maps (c0,c1,c2,c3) to
 *      (hi(M1*c2)^c1^k0, lo(M1*c2), hi(M0*c0)^c3^k1, lo(M0*c0)); the key is bumped
 *      by the Weyl constants before every round but the first; ten rounds). ---- */

void fho_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    const uint64_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;
    const uint32_t W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int r = 0; r < 10; ++r) {
        if (r > 0) { k0 += W0; k1 += W1; }
        uint64_t p0 = M0 * (uint64_t)c0;
        uint64_t p1 = M1 * (uint64_t)c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* Random bits of one element.  One Philox block serves 8 consecutive elements:
 * key = the 64-bit seed, counter = (block index b = i/8 as 64 bits, tensor id as
 * 64 bits).  Element i reads output word (i mod 8)/2, low half-word when i is
 * even, high half-word when odd.  The bits are a function of (seed, tensor id, i)
 * alone, which is what "keyed by (seed, tensor id, element index)" asks for. */
uint32_t fho_random16(uint64_t seed, uint64_t tensor_id, uint64_t index)
{
    uint64_t b = index >> 3;
    uint32_t ctr[4] = { (uint32_t)b, (uint32_t)(b >> 32),
                        (uint32_t)tensor_id, (uint32_t)(tensor_id >> 32) };
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint32_t w[4];
    fho_philox4x32_10(ctr, key, w);
    uint32_t word = w[(index & 7u) >> 1];
    return (index & 1u) ? (word >> 16) : (word & 0xFFFFu);
}

size_t fho_packed_bytes(int64_t numel, int bits)
{
    if (numel <= 0) return 0;
    uint64_t raw = ((uint64_t)numel * (uint64_t)bits + 7u) / 8u;
    return (size_t)((raw + 15u) / 16u * 16u);
}

size_t fho_meta_bytes(int64_t numel, int group_size)
{
    if (numel <= 0) return 0;
    return (size_t)(8u * (((uint64_t)numel + (uint64_t)group_size - 1u) / (uint64_t)group_size));
}

/* bf16 <-> fp32.  Widening appends sixteen zero bits (exact).  Narrowing rounds to
 * nearest, ties to even, on the bit pattern (finite inputs). */
static float load_elem(const void *x, int dtype, int64_t i)
{
    if (dtype == FHO_F32) return ((const float *)x)[i];
    uint32_t bits = (uint32_t)((const uint16_t *)x)[i] << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return f;
}

static uint16_t narrow_bf16(float f)
{
    uint32_t bits;
    memcpy(&bits, &f, sizeof bits);
    if ((bits & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((bits >> 16) | 0x40u); /* NaN stays NaN */
    uint32_t keep = bits >> 16;
    uint32_t drop = bits & 0xFFFFu;
    if (drop > 0x8000u || (drop == 0x8000u && (keep & 1u))) keep += 1u;
    return (uint16_t)keep;
}

static int args_ok(int64_t numel, int group_size, int bits)
{
    return numel >= 0 && group_size >= 1 && (bits == 2 || bits == 4 || bits == 8);
}

int fho_compress(const void *x, int dtype, int64_t numel, int group_size, int bits,
                 int rounding, uint64_t seed, uint64_t tensor_id,
                 uint8_t *packed, float *meta)
{
    if (!args_ok(numel, group_size, bits)) return -1;
    if (dtype != FHO_F32 && dtype != FHO_BF16) return -1;
    if (rounding != FHO_ROUND_NEAREST && rounding != FHO_ROUND_STOCHASTIC) return -1;
    if (numel == 0) return 0;
    if (!x || !packed || !meta) return -1;

    const int levels = (1 << bits) - 1;            /* L */
    const float Lf = (float)levels;
    const float tiny = 0x1p-100f;
    memset(packed, 0, fho_packed_bytes(numel, bits));

    int64_t g = 0;
    for (int64_t start = 0; start < numel; start += group_size, ++g) {
        int64_t end = start + group_size < numel ? start + group_size : numel;

        float mn = load_elem(x, dtype, start), mx = mn;
        for (int64_t i = start + 1; i < end; ++i) {
            float v = load_elem(x, dtype, i);
            if (v < mn) mn = v;
            if (v > mx) mx = v;
        }
        float range = mx - mn;
        float zero = mn + 0.0f;
        int degenerate = range < tiny;
        float scale = degenerate ? 0.0f : range / Lf;
        float inv = degenerate ? 0.0f : Lf / range;
        meta[2 * g + 0] = scale;
        meta[2 * g + 1] = zero;
        if (degenerate) continue;                  /* all codes 0: bytes already zero */

        for (int64_t i = start; i < end; ++i) {
            float t = load_elem(x, dtype, i) - mn;
            float q = t * inv;
            if (q < 0.0f) q = 0.0f;
            if (q > Lf) q = Lf;
            uint32_t code;
            if (rounding == FHO_ROUND_NEAREST) {
                code = (uint32_t)rintf(q);         /* default rounding mode: ties to even */
            } else {
                float k = floorf(q);
                float f = q - k;                   /* exact */
                float u = (float)fho_random16(seed, tensor_id, (uint64_t)i) * 0x1p-16f;
                code = (uint32_t)k + (u < f ? 1u : 0u);
            }
            uint64_t bitpos = (uint64_t)i * (uint64_t)bits;
            packed[bitpos >> 3] |= (uint8_t)(code << (bitpos & 7u));
        }
    }
    return 0;
}

int fho_unpack_codes(const uint8_t *packed, int64_t numel, int bits, uint8_t *codes)
{
    if (!args_ok(numel, 1, bits)) return -1;
    const uint32_t mask = (1u << bits) - 1u;
    for (int64_t i = 0; i < numel; ++i) {
        uint64_t bitpos = (uint64_t)i * (uint64_t)bits;
        codes[i] = (uint8_t)((packed[bitpos >> 3] >> (bitpos & 7u)) & mask);
    }
    return 0;
}

int fho_decompress(const uint8_t *packed, const float *meta, int64_t numel,
                   int group_size, int bits, int out_dtype, void *out)
{
    if (!args_ok(numel, group_size, bits)) return -1;
    if (out_dtype != FHO_F32 && out_dtype != FHO_BF16) return -1;
    if (numel == 0) return 0;
    if (!packed || !meta || !out) return -1;
    const uint32_t mask = (1u << bits) - 1u;
    for (int64_t i = 0; i < numel; ++i) {
        int64_t g = i / group_size;
        uint64_t bitpos = (uint64_t)i * (uint64_t)bits;
        uint32_t code = (packed[bitpos >> 3] >> (bitpos & 7u)) & mask;
        float v = fmaf((float)code, meta[2 * g + 0], meta[2 * g + 1]);
        if (out_dtype == FHO_F32) ((float *)out)[i] = v;
        else ((uint16_t *)out)[i] = narrow_bf16(v);
    }
    return 0;
}
