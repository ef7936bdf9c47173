"""The whole channel-wise mix compressor (Section 4.4.1, first sentence to last) as a
composition of the oracle's stages, in the section's order: three-sigma classification, slots
for the salient channels, quantisation of the normal channels with the salient ones in a raw
store (unused rows zero), the raw store's maps as sparse / predicted blocks, Huffman coding of
the index stream; and back.  Test infrastructure: calls only `oracle`."""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

import oracle


@dataclass
class Stored:
    stats: np.ndarray
    counts: np.ndarray
    mask: np.ndarray
    slots: np.ndarray
    used: int
    packed: np.ndarray
    meta: np.ndarray
    raw: np.ndarray                 # what the sparse stage was given
    info: np.ndarray
    values: np.ndarray
    indices: np.ndarray
    totals: np.ndarray
    huffman: np.ndarray             # the coded index stream (empty without the entropy stage)
    payload_bits: int
    stored_bytes: int


def mix_compress(x, outer, C, inner, raw_channels, G, B, rounding, seed, tid, k_sigma, min_outliers,
                 maps, h, w, window, tau, eps, entropy, dtype="f32") -> Stored:
    stats, counts, mask = oracle.classify_channels(x, outer, C, inner, k_sigma, min_outliers, dtype=dtype)
    slots, used = oracle.channel_slots(mask, raw_channels)
    packed, meta, raw = oracle.compress_mixed(x, outer, C, inner, slots, raw_channels, G, B, rounding, seed, tid,
                                              dtype=dtype, raw_fill=0)
    esize = 4 if dtype == "f32" else 2
    stored = 64 + packed.size + meta.size * 4
    if raw.size:
        info, values, indices, totals = oracle.sparse_encode(raw, maps, h, w, window, tau, dtype=dtype, eps=eps)
        stored += 2 * C + info.size + values.size * esize
        if entropy:
            huff, bits = oracle.huffman_encode(indices)
            stored += huff.size
        else:
            huff, bits = np.zeros(0, np.uint8), 0
            stored += indices.size
    else:
        info, values, indices = np.zeros(0, np.uint8), raw[:0], np.zeros(0, np.uint8)
        totals, huff, bits = np.zeros(4, np.uint64), np.zeros(0, np.uint8), 0
    return Stored(stats, counts, mask, slots, used, packed, meta, raw, info, values, indices, totals, huff, bits, stored)


def mix_decompress(st: Stored, outer, C, inner, raw_channels, G, B, maps, h, w, window, eps, entropy,
                   dtype="f32", out_dtype="f32") -> np.ndarray:
    if st.raw.size:
        indices = oracle.huffman_decode(st.huffman, st.indices.size) if entropy else st.indices
        raw = oracle.sparse_decode(st.info, st.values, indices, maps, h, w, window, dtype=dtype, eps=eps)
    else:
        raw = st.raw
    return oracle.decompress_mixed(st.packed, st.meta, raw, outer, C, inner, st.slots, raw_channels, G, B,
                                   raw_dtype=dtype, out_dtype=out_dtype)
