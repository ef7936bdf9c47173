"""Pins of the oracle chain (tests/oracle_chain.py), the composition the GPU chain is compared
with: what Section 4.4.1 promises of the whole compressor must hold end to end -- outliers in
salient channels no longer stretch the normal channels' quantisation range, salient channels
come back within the error bound (exactly without one), zeros survive, and the stored size is
the sum of its parts."""
from __future__ import annotations

import numpy as np
import pytest

import oracle
import oracle_chain as OC
from paper_2510_11400_amd import workloads as W


def _run(eps, entropy, raw_channels=4, B=4):
    outer, C, inner = 8, 32, 196
    x, planted = W.outlier_channel_tensor(outer, C, inner, seed=3, dist="relu", salient_fraction=0.1, hit_fraction=0.1)
    args = (outer, C, inner, raw_channels, 128, B)
    st = OC.mix_compress(x, *args, "nearest", 0, 0, 3.0, 15, outer * raw_channels, 14, 14, 4, 0.5, eps, entropy)
    back = OC.mix_decompress(st, *args, outer * raw_channels, 14, 14, 4, eps, entropy)
    return x.reshape(outer, C, inner), back.reshape(outer, C, inner), st, planted


@pytest.mark.parametrize("entropy", [0, 1])
@pytest.mark.parametrize("eps", [0.0, 0.02])
def test_whole_chain_round_trip(eps, entropy):
    x, back, st, planted = _run(eps, entropy)
    kept = np.flatnonzero(st.slots >= 0)
    assert set(kept) <= set(np.flatnonzero(st.mask)) and 0 < kept.size <= 4
    assert set(kept) <= set(planted)                       # what the three-sigma rule finds are the planted channels
    normal = np.setdiff1d(np.arange(x.shape[1]), kept)
    # salient channels: exact without a bound, within it otherwise (outliers intact)
    err = np.abs(back[:, kept] - x[:, kept])
    assert err.max() == 0.0 if eps == 0.0 else err.max() <= eps * (1 + 1e-6) + np.abs(x[:, kept]).max() * 2.0 ** -22
    # zeros of kept channels survive exactly (the paper's requirement)
    assert np.all(back[:, kept][x[:, kept] == 0.0] == 0.0)
    # normal channels: the error is that of groups whose range holds no 81x outlier
    plain_p, plain_m = oracle.compress(x.reshape(-1), 128, 4, "nearest", 0, 0)
    plain = oracle.decompress(plain_p, plain_m, x.size, 128, 4).reshape(x.shape)
    e_mix = np.abs(back[:, normal] - x[:, normal]).max()
    e_plain = np.abs(plain[:, normal] - x[:, normal]).max()
    assert e_mix <= np.abs(x[:, normal]).max() / 15 / 2 * 1.01
    unkept_planted = np.setdiff1d(planted, kept)
    if unkept_planted.size == 0:
        assert e_mix < e_plain / 4                         # the plain quantiser's groups straddle the outliers
    # the entropy stage changes sizes, not values; the stored size is the sum of its parts
    parts = 64 + st.packed.size + st.meta.size * 4 + 2 * 32 + st.info.size + st.values.size * 4
    parts += st.huffman.size if entropy else st.indices.size
    assert st.stored_bytes == parts
    if entropy:
        assert st.huffman.size > 0 and st.payload_bits <= 8 * st.indices.size + 8


def test_nothing_kept_equals_the_plain_quantiser():
    outer, C, inner = 8, 32, 196
    x, _ = W.outlier_channel_tensor(outer, C, inner, seed=3, dist="relu")
    st = OC.mix_compress(x, outer, C, inner, 0, 128, 4, "stochastic", 5, 9, 3.0, 15, 0, 0, 0, 4, 0.5, 0.02, 1)
    p, m = oracle.compress(x, 128, 4, "stochastic", 5, 9)
    assert np.array_equal(st.packed, p) and np.array_equal(st.meta.view(np.uint32), m.view(np.uint32))
    assert st.stored_bytes == 64 + p.size + m.size * 4 and st.used == 0
    back = OC.mix_decompress(st, outer, C, inner, 0, 128, 4, 0, 0, 0, 4, 0.02, 1)
    assert np.array_equal(back.view(np.uint32), oracle.decompress(p, m, x.size, 128, 4).view(np.uint32))
