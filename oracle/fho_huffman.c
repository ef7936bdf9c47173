/* CPU oracle for the entropy stage of the predictive form (FedHybrid Section 4.4.1: the
 * quantisation codes are encoded with Huffman coding; restoring starts with Huffman
 * decoding).  TEST INFRASTRUCTURE ONLY: plain loops, one symbol at a time; shares nothing
 * with the HIP path.  The paper names the coder and nothing else; everything below the name
 * (tie-breaking, length limit, canonical codes, chunked layout) is the reading stated in
 * fho.h, chosen so that the result is unique. */
#include "fho.h"

#include <stdlib.h>
#include <string.h>

#define CHUNK 256u
#define MAXLEN 24

typedef struct { uint64_t weight; int symbol; } leaf_t;

static int leaf_order(const void *a, const void *b)
{
    const leaf_t *x = (const leaf_t *)a, *y = (const leaf_t *)b;
    if (x->weight != y->weight) return x->weight < y->weight ? -1 : 1;
    return x->symbol - y->symbol;
}

/* depth of every used symbol in the Huffman tree of the counts c; returns the largest */
static int tree_depths(const uint64_t c[256], uint8_t len[256])
{
    leaf_t leaf[256];
    int m = 0;
    memset(len, 0, 256);
    for (int s = 0; s < 256; ++s)
        if (c[s]) { leaf[m].weight = c[s]; leaf[m].symbol = s; ++m; }
    if (m == 0) return 0;
    if (m == 1) { len[leaf[0].symbol] = 1; return 1; }
    qsort(leaf, (size_t)m, sizeof leaf[0], leaf_order);
    /* nodes 0..m-1: the leaves in sorted order; m..2m-2: internal nodes in the order they are made */
    uint64_t weight[511];
    int parent[511], depth[511];
    for (int i = 0; i < m; ++i) weight[i] = leaf[i].weight;
    int next_leaf = 0, next_internal = m, made = m;
    while (made < 2 * m - 1) {
        int pick[2];
        for (int k = 0; k < 2; ++k) {
            const int have_leaf = next_leaf < m, have_internal = next_internal < made;
            if (have_leaf && (!have_internal || weight[next_leaf] <= weight[next_internal])) pick[k] = next_leaf++;
            else pick[k] = next_internal++;
        }
        weight[made] = weight[pick[0]] + weight[pick[1]];
        parent[pick[0]] = parent[pick[1]] = made;
        ++made;
    }
    depth[2 * m - 2] = 0;
    int deepest = 0;
    for (int i = 2 * m - 3; i >= 0; --i) depth[i] = depth[parent[i]] + 1;      /* a parent is made after its children */
    for (int i = 0; i < m; ++i) {
        len[leaf[i].symbol] = (uint8_t)depth[i];
        if (depth[i] > deepest) deepest = depth[i];
    }
    return deepest;
}

void fho_huffman_lengths(const uint64_t hist[256], uint8_t len[256])
{
    uint64_t c[256];
    memcpy(c, hist, sizeof c);
    while (tree_depths(c, len) > MAXLEN)
        for (int s = 0; s < 256; ++s)
            if (c[s]) c[s] = (c[s] + 1) >> 1;
}

void fho_huffman_codes(const uint8_t len[256], uint32_t code[256])
{
    uint32_t count[MAXLEN + 2] = {0}, next[MAXLEN + 2] = {0};
    for (int s = 0; s < 256; ++s)
        if (len[s] >= 1 && len[s] <= MAXLEN) ++count[len[s]];
    for (int l = 2; l <= MAXLEN; ++l) next[l] = (next[l - 1] + count[l - 1]) << 1;
    for (int s = 0; s < 256; ++s)
        code[s] = (len[s] >= 1 && len[s] <= MAXLEN) ? next[len[s]]++ : 0u;
}

static uint64_t chunks_of(uint64_t n) { return (n + CHUNK - 1) / CHUNK; }

size_t fho_huffman_stream_bytes(uint64_t n)
{
    /* a chunk holds at most 256 codes of 24 bits = 192 words */
    return (size_t)(256u + 4u * (chunks_of(n) + 1u) + 4u * 192u * chunks_of(n));
}

static void put_u32(uint8_t *p, uint32_t v) { memcpy(p, &v, 4); }
static uint32_t get_u32(const uint8_t *p) { uint32_t v; memcpy(&v, p, 4); return v; }

int fho_huffman_encode(const uint8_t *in, uint64_t n, uint8_t *stream, uint64_t totals[2])
{
    if (!stream || !totals || (n > 0 && !in) || n >= ((uint64_t)1 << 32)) return -1;
    uint64_t hist[256] = {0};
    for (uint64_t i = 0; i < n; ++i) ++hist[in[i]];
    uint8_t len[256];
    uint32_t code[256];
    fho_huffman_lengths(hist, len);
    fho_huffman_codes(len, code);
    memcpy(stream, len, 256);
    const uint64_t chunks = chunks_of(n);
    uint8_t *offsets = stream + 256, *payload = offsets + 4 * (chunks + 1);
    uint64_t word = 0, bits_total = 0;
    for (uint64_t c = 0; c < chunks; ++c) {
        put_u32(offsets + 4 * c, (uint32_t)word);
        const uint64_t end = (c + 1) * CHUNK < n ? (c + 1) * CHUNK : n;
        uint32_t acc = 0;
        int filled = 0;                                   /* bits of acc in use, from bit 31 downwards */
        for (uint64_t i = c * CHUNK; i < end; ++i) {
            const int l = len[in[i]];
            for (int b = l - 1; b >= 0; --b) {            /* one bit at a time, first bit first */
                acc |= ((code[in[i]] >> b) & 1u) << (31 - filled);
                if (++filled == 32) { put_u32(payload + 4 * word++, acc); acc = 0; filled = 0; }
            }
            bits_total += (uint64_t)l;
        }
        if (filled) put_u32(payload + 4 * word++, acc);
    }
    put_u32(offsets + 4 * chunks, (uint32_t)word);
    totals[0] = 256u + 4u * (chunks + 1u) + 4u * word;
    totals[1] = bits_total;
    return 0;
}

int fho_huffman_decode(const uint8_t *stream, uint64_t stream_bytes, uint64_t n, uint8_t *out)
{
    if (!stream || (n > 0 && !out) || n >= ((uint64_t)1 << 32)) return -1;
    const uint64_t chunks = chunks_of(n);
    if (stream_bytes < 256u + 4u * (chunks + 1u)) return -2;
    const uint8_t *len = stream, *offsets = stream + 256, *payload = offsets + 4 * (chunks + 1);
    const uint64_t words = (stream_bytes - 256u - 4u * (chunks + 1u)) / 4u;
    /* canonical decoding tables: symbols by (length, symbol); first code and count of every length */
    uint32_t count[MAXLEN + 2] = {0}, first[MAXLEN + 2] = {0}, start[MAXLEN + 2] = {0};
    uint8_t sorted[256];
    for (int s = 0; s < 256; ++s) {
        if (len[s] > MAXLEN) return -2;
        if (len[s]) ++count[len[s]];
    }
    for (int l = 2; l <= MAXLEN; ++l) first[l] = (first[l - 1] + count[l - 1]) << 1;
    for (int l = 2; l <= MAXLEN; ++l) start[l] = start[l - 1] + count[l - 1];
    {
        uint32_t fill[MAXLEN + 2];
        memcpy(fill, start, sizeof fill);
        for (int s = 0; s < 256; ++s)
            if (len[s]) sorted[fill[len[s]]++] = (uint8_t)s;
    }
    for (uint64_t c = 0; c < chunks; ++c) {
        uint64_t bit = (uint64_t)get_u32(offsets + 4 * c) * 32u;
        const uint64_t end = (c + 1) * CHUNK < n ? (c + 1) * CHUNK : n;
        for (uint64_t i = c * CHUNK; i < end; ++i) {
            uint32_t code = 0;
            int l = 0, found = 0;
            while (l < MAXLEN && !found) {
                if (bit / 32u >= words) return -2;
                code = (code << 1) | ((get_u32(payload + 4 * (bit / 32u)) >> (31u - bit % 32u)) & 1u);
                ++bit;
                ++l;
                if (count[l] && code >= first[l] && code - first[l] < count[l]) {
                    out[i] = sorted[start[l] + code - first[l]];
                    found = 1;
                }
            }
            if (!found) return -2;
        }
    }
    return 0;
}
