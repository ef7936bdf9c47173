"""Pins for the oracle's Huffman stage (Section 4.4.1: the quantisation codes of the predictive
form are encoded with Huffman coding; restoring begins with Huffman decoding).  The paper names
the coder only, so the pins are what the mathematics fixes: the textbook example (Cormen,
Leiserson, Rivest, Stein, "Introduction to Algorithms", section 16.3: frequencies 45, 13, 12,
16, 9, 5 give lengths 1, 3, 3, 3, 4, 4), optimality against an independent heap-based
construction, Kraft's equality, prefix-freeness, the entropy bound, a stream worked out by
hand, and the lossless round trip."""
from __future__ import annotations

import heapq
import itertools

import numpy as np
import pytest

import oracle


def _hist(data):
    return np.bincount(np.asarray(data, dtype=np.uint8), minlength=256).astype(np.uint64)


def _heap_cost(hist):
    """Cost (sum of count * length) of an optimal prefix code, by the heap construction."""
    heap = [int(c) for c in hist if c]
    if len(heap) == 1:
        return heap[0]
    heapq.heapify(heap)
    cost = 0
    while len(heap) > 1:
        a, b = heapq.heappop(heap), heapq.heappop(heap)
        cost += a + b
        heapq.heappush(heap, a + b)
    return cost


def test_textbook_example():
    h = np.zeros(256, np.uint64)
    for s, c in zip(b"abcdef", (45, 13, 12, 16, 9, 5)):
        h[s] = c
    l = oracle.huffman_lengths(h)
    assert [int(l[s]) for s in b"abcdef"] == [1, 3, 3, 3, 4, 4]
    assert int(l.astype(np.int64).sum()) == 18                   # every other symbol has no code
    codes = oracle.huffman_codes(l)
    assert [int(codes[s]) for s in b"abcdef"] == [0b0, 0b100, 0b101, 0b110, 0b1110, 0b1111]


def test_a_stream_worked_out_by_hand():
    # counts a5 b2 r2 c1 d1; leaves by (count, symbol): c d b r a.  c+d = 2; the tie between the
    # leaf b (2) and that node goes to the leaf: b+r = 4; then 2+4 = 6; then a+6.
    # lengths a1 b3 c3 d3 r3; canonical codes a=0 b=100 c=101 d=110 r=111.
    data = np.frombuffer(b"abracadabra", np.uint8)
    l = oracle.huffman_lengths(_hist(data))
    assert {chr(s): int(l[s]) for s in b"abcdr"} == {"a": 1, "b": 3, "c": 3, "d": 3, "r": 3}
    stream, bits = oracle.huffman_encode(data)
    assert bits == 23 and stream.size == 256 + 4 * 2 + 4
    assert np.array_equal(stream[:256], l)
    assert stream[256:264].view(np.uint32).tolist() == [0, 1]     # one chunk, one word
    # 0 100 111 0 101 0 110 0 100 111 0, first bit in bit 31
    assert int(stream[264:268].view(np.uint32)[0]) == int("0100" "1110" "1010" "1100" "1001" "110" + "0" * 9, 2)
    assert bytes(oracle.huffman_decode(stream, data.size)) == b"abracadabra"


def test_equal_counts_are_ordered_by_symbol():
    # three symbols, equal counts: the two smallest symbols are merged first, the largest gets the short code
    l = oracle.huffman_lengths(_hist(np.frombuffer(b"xyzzyx", np.uint8)))
    assert {chr(s): int(l[s]) for s in b"xyz"} == {"x": 2, "y": 2, "z": 1}
    l = oracle.huffman_lengths(_hist(np.arange(5, dtype=np.uint8)))           # 0..4 once each
    assert l[:5].tolist() == [3, 3, 2, 2, 2]          # 0+1 -> 2; 2+3 -> 2 (leaves before the node); 4+(0+1); ...


@pytest.mark.parametrize("seed", range(12))
def test_cost_is_optimal_and_the_code_is_complete(seed):
    rng = np.random.default_rng(seed)
    used = int(rng.integers(2, 257))
    h = np.zeros(256, np.uint64)
    syms = rng.choice(256, used, replace=False)
    kind = seed % 3
    h[syms] = (rng.integers(1, 50, used) if kind == 0 else
               (rng.pareto(0.7, used) * 10 + 1).astype(np.uint64) if kind == 1 else
               np.full(used, 7))                                   # many ties
    l = oracle.huffman_lengths(h).astype(np.int64)
    assert (l[h == 0] == 0).all() and (l[h > 0] >= 1).all() and l.max() <= 24
    assert int((h.astype(np.int64) * l).sum()) == _heap_cost(h)
    assert sum(2.0 ** -int(x) for x in l[l > 0]) == 1.0            # Kraft's equality: no wasted code
    # prefix-free and canonical
    codes = oracle.huffman_codes(l.astype(np.uint8))
    words = sorted((format(int(codes[s]), f"0{int(l[s])}b"), s) for s in range(256) if l[s])
    for (a, _), (b, _) in zip(words, words[1:]):
        assert not b.startswith(a)
    order = sorted((int(l[s]), s) for s in range(256) if l[s])
    values = [int(codes[s]) << (24 - int(l[s])) for _, s in order]
    assert values == sorted(values) and len(set(values)) == len(values)


def test_average_length_is_within_one_bit_of_the_entropy():
    rng = np.random.default_rng(5)
    data = np.clip(np.rint(rng.normal(128, 3.0, 200000)), 0, 255).astype(np.uint8)   # like prediction errors
    h = _hist(data)
    p = h[h > 0] / data.size
    entropy = float(-(p * np.log2(p)).sum())
    stream, bits = oracle.huffman_encode(data)
    assert entropy <= bits / data.size < entropy + 1
    assert stream.size < data.size / 2
    assert np.array_equal(oracle.huffman_decode(stream, data.size), data)


@pytest.mark.parametrize("n", [0, 1, 2, 255, 256, 257, 511, 512, 513, 70000])
def test_round_trip_over_chunk_boundaries(n):
    rng = np.random.default_rng(n)
    data = rng.integers(0, 256, n).astype(np.uint8) if n % 2 else (rng.geometric(0.3, n) % 256).astype(np.uint8)
    stream, bits = oracle.huffman_encode(data)
    chunks = (n + 255) // 256
    offsets = stream[256:256 + 4 * (chunks + 1)].view(np.uint32)
    l = stream[:256].astype(np.int64)
    assert bits == int(l[data].sum())
    # every chunk starts on a word and is as long as its codes need
    for c in range(chunks):
        need = int(l[data[c * 256:(c + 1) * 256]].sum())
        assert int(offsets[c + 1]) - int(offsets[c]) == (need + 31) // 32
    assert stream.size == 256 + 4 * (chunks + 1) + 4 * int(offsets[-1] if chunks else 0)
    assert np.array_equal(oracle.huffman_decode(stream, n), data)


def test_one_symbol_and_two_symbols():
    data = np.full(1000, 200, np.uint8)
    stream, bits = oracle.huffman_encode(data)
    assert bits == 1000 and stream[200] == 1 and int(stream[:256].astype(np.int64).sum()) == 1
    assert np.array_equal(oracle.huffman_decode(stream, 1000), data)
    data[::3] = 7
    stream, bits = oracle.huffman_encode(data)
    assert bits == 1000 and stream[7] == 1 and stream[200] == 1
    assert np.array_equal(oracle.huffman_decode(stream, 1000), data)


def test_codes_longer_than_24_bits_are_avoided_by_halving_the_counts():
    fib = [1, 1]
    while len(fib) < 34:
        fib.append(fib[-1] + fib[-2])
    h = np.zeros(256, np.uint64)
    h[10:10 + len(fib)] = fib                                      # the tree of these counts is a 33-deep comb
    l = oracle.huffman_lengths(h).astype(np.int64)
    assert l.max() <= 24 and (l[10:44] >= 1).all()
    assert sum(2.0 ** -int(x) for x in l[l > 0]) == 1.0
    # the same counts halved (rounding up) until the comb is short enough give the same lengths
    c = h.copy()
    rounds = 0
    while True:
        plain = oracle.huffman_lengths(c)
        if _heap_cost(c) == int((c.astype(np.int64) * plain.astype(np.int64)).sum()):
            break                                                  # no halving happened inside: optimal for c
        c[c > 0] = (c[c > 0] + 1) >> 1
        rounds += 1
    assert rounds >= 1 and np.array_equal(plain, l)
    # and data whose own histogram is such a comb (27 deep) still comes back, with the limited lengths
    data = np.repeat(np.arange(10, 38, dtype=np.uint8), fib[:28])
    stream, _ = oracle.huffman_encode(data)
    assert stream[:256].max() <= 24 and np.array_equal(stream[:256], oracle.huffman_lengths(_hist(data)))
    assert np.array_equal(oracle.huffman_decode(stream, data.size), data)


def test_a_truncated_stream_is_refused():
    data = (np.arange(5000) % 251).astype(np.uint8)
    stream, _ = oracle.huffman_encode(data)
    with pytest.raises(ValueError):
        oracle.huffman_decode(stream[:-4], data.size)
    with pytest.raises(ValueError):
        oracle.huffman_decode(stream[:200], data.size)


def test_room_the_encoder_asks_for_is_the_worst_case_of_the_layout():
    """fho_huffman_stream_bytes: 256 length bytes, one offset per chunk of 256 symbols plus one,
    and for every chunk 256 symbols of the longest code the limit allows (24 bits = 192 words).
    Pinned by the layout's arithmetic and by streams that come as close to the bound as data can:
    uniform bytes (8 bits per symbol) and the comb whose rarest symbols carry 24-bit codes."""
    size = oracle.lib().fho_huffman_stream_bytes
    for n in (0, 1, 255, 256, 257, 4096, 65_537, 10 ** 6 + 3):
        chunks = -(-n // 256)
        assert size(n) == 256 + 4 * (chunks + 1) + 4 * (256 * 24 // 32) * chunks
    rng = np.random.default_rng(0)
    uniform = rng.integers(0, 256, 70_001).astype(np.uint8)
    fib = [1, 1]
    while len(fib) < 28:
        fib.append(fib[-1] + fib[-2])
    comb = np.repeat(np.arange(10, 38, dtype=np.uint8), fib)
    rare_first = comb[np.argsort(np.repeat(fib, fib), kind="stable")]      # the long codes crowd the first chunks
    for data in (uniform, comb, rare_first, np.zeros(300, np.uint8)):
        stream, bits = oracle.huffman_encode(data)
        assert stream.size <= size(data.size)
        lengths = stream[:256].astype(np.int64)
        chunk_bits = [int(lengths[data[c:c + 256]].sum()) for c in range(0, data.size, 256)]
        assert max(chunk_bits) <= 256 * 24 and bits == sum(chunk_bits)
        assert stream.size == 256 + 4 * (len(chunk_bits) + 1) + 4 * sum(-(-b // 32) for b in chunk_bits)
