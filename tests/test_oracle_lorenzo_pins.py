"""Pins for the oracle's error-bounded predictive form of dense blocks (Section 4.4.1: in dense
blocks each element is predicted from its neighbours by the Lorenzo predictor, prediction
errors within the bound are quantised, outliers are kept intact, prediction uses decompressed
values).  The paper's equations for this step are garbled and it prints no example; the pins
are the error bound itself, the textbook property of the first-order Lorenzo predictor
(it reproduces a + b*r + c*col exactly), exact lattice data, a vectorised numpy twin built
from second differences and cumulative sums, and outliers surviving bit for bit."""
from __future__ import annotations

import numpy as np
import pytest

import oracle
from paper_2510_11400_amd import workloads as W

f32 = np.float32


def _blocks(a2d, n):
    """Non-overlapping n x n blocks of a [h][w] array, block-row-major, each row-major."""
    h, w = a2d.shape
    return [a2d[r:r + n, c:c + n] for r in range(0, h, n) for c in range(0, w, n)]


def _lattice_np(x, eps):
    two = f32(eps) + f32(eps)
    t = (x.astype(f32) / two).astype(f32)
    ok = np.abs(t) < f32(2.0 ** 22)
    q = np.where(ok, np.rint(np.where(ok, t, 0)), 0).astype(np.int64)
    return q, ok, two


def _second_difference(q):
    """d = q - left - up + diag with zeros outside the block."""
    z = np.zeros((q.shape[0] + 1, q.shape[1] + 1), dtype=np.int64)
    z[1:, 1:] = q
    return z[1:, 1:] - z[1:, :-1] - z[:-1, 1:] + z[:-1, :-1]


def _dense_everything(x, maps, h, w, n, eps, dtype="f32"):
    """Encode with tau < 0, so that every block takes the dense form."""
    return oracle.sparse_encode(x, maps, h, w, n, -1.0, dtype=dtype, eps=eps)


@pytest.mark.parametrize("n", [2, 4, 8])
@pytest.mark.parametrize("eps", [1e-3, 0.05, 0.5])
def test_restored_values_are_within_the_error_bound_and_outliers_are_intact(n, eps):
    maps, h, w = 5, 27, 22
    x = W.salient_feature_maps(maps, h, w, seed=n, zero_level=-0.5)          # few zeros: smooth positive field
    info, v, idx, t = _dense_everything(x, maps, h, w, n, eps)
    y = oracle.sparse_decode(info, v, idx, maps, h, w, n, eps=eps)
    err = np.abs(y.astype(np.float64) - x.astype(np.float64))
    bound = eps * (1 + 1e-6) + np.abs(x.astype(np.float64)) * 2.0 ** -22      # the division's and the product's rounding
    assert (err <= bound).all()
    # what the value stream holds are elements of x, in order, and they come back bit for bit
    exact = y.view(np.uint32) == x.view(np.uint32)
    assert exact.sum() >= v.size
    assert t[0] == v.size == int((info & 0x7F).sum()) and t[1] == idx.size == maps * h * w and t[2] == 0
    # and the bound is not vacuous: most elements are not exact at the coarser settings
    if eps >= 0.05:
        assert (~exact).mean() > 0.3


@pytest.mark.parametrize("n", [2, 4, 8])
def test_first_order_lorenzo_reproduces_planes_exactly(n):
    """On lattice data q = a + b*r + c*col every interior prediction is exact: code 128.  The
    first row and column of a block predict from zeros outside the block, so they carry the
    slope (or the value itself)."""
    eps = 0.25                                                              # lattice step 0.5: exact in binary32
    h = w = 2 * n
    r, c = np.meshgrid(np.arange(h), np.arange(w), indexing="ij")
    q = 3 + 2 * (r % n) - 1 * (c % n)                                        # the same plane in every block
    x = (q * 0.5).astype(f32).reshape(-1)
    info, v, idx, t = _dense_everything(x, 1, h, w, n, eps)
    assert v.size == 0 and (info == 0x80).all()                              # no outlier anywhere
    codes = idx.reshape(4, n, n)
    for blk in codes:
        assert (blk[1:, 1:] == 128).all()
        assert blk[0, 0] == 128 + 3
        assert (blk[0, 1:] == 128 - 1).all() and (blk[1:, 0] == 128 + 2).all()
    y = oracle.sparse_decode(info, v, idx, 1, h, w, n, eps=eps)
    assert np.array_equal(y, x)                                              # lattice data comes back exactly


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("n,eps", [(2, 0.01), (4, 0.02), (8, 0.1), (4, 1e-4)])
def test_against_second_differences_and_cumulative_sums(dtype, n, eps):
    maps, h, w = 3, 21, 30
    x = W.salient_feature_maps(maps, h, w, seed=7 + n, zero_level=0.0, dtype=dtype)
    xf = x if dtype == "f32" else (x.astype(np.uint32) << 16).view(f32)
    xf = xf.copy()
    info, v, idx, t = _dense_everything(x, maps, h, w, n, eps, dtype=dtype)
    y = oracle.sparse_decode(info, v, idx, maps, h, w, n, dtype=dtype, eps=eps)
    yf = y if dtype == "f32" else (y.astype(np.uint32) << 16).view(f32)
    nv = ni = 0
    b = 0
    for m in range(maps):
        for blk, out in zip(_blocks(xf.reshape(maps, h, w)[m], n), _blocks(yf.reshape(maps, h, w)[m], n)):
            q, ok, two = _lattice_np(blk, eps)
            d = _second_difference(q)
            outlier = ~ok | (d <= -128) | (d >= 128)
            want_codes = np.where(outlier, 0, d + 128).astype(np.uint8)
            got_codes = idx[ni:ni + blk.size].reshape(blk.shape)
            assert np.array_equal(got_codes, want_codes)
            assert info[b] == (0x80 | int(outlier.sum()))
            got_out = v[nv:nv + int(outlier.sum())]
            raw = x.reshape(maps, h, w)[m]
            # outliers: the original bits, row-major
            r0 = (b % (-(-h // n) * -(-w // n))) // -(-w // n) * n
            c0 = (b % -(-w // n)) * n
            assert np.array_equal(got_out, raw[r0:r0 + n, c0:c0 + n][outlier])
            # restore: cumulative sums of the second differences give the lattice back
            assert np.array_equal(np.cumsum(np.cumsum(d, axis=0), axis=1), q)
            want = (q.astype(f32) * two).astype(f32)
            if dtype == "bf16":
                u = want.view(np.uint32).astype(np.uint64)
                want = (((u + 0x7FFF + ((u >> 16) & 1)) >> 16).astype(np.uint32) << 16).view(f32)
            want = np.where(outlier, blk, want)
            assert np.array_equal(out.view(np.uint32), want.view(np.uint32))
            nv += int(outlier.sum())
            ni += blk.size
            b += 1
    assert nv == v.size and ni == idx.size


def test_values_without_a_lattice_point_are_outliers_and_predict_as_zero():
    eps = 1e-3
    x = np.full(16, 0.5, f32)
    x[5] = 3e7                      # |x / 2eps| >= 2^22
    x[10] = np.inf
    info, v, idx, _ = _dense_everything(x, 1, 4, 4, 4, eps)
    codes = idx.reshape(4, 4)
    assert codes[1, 1] == 0 and codes[2, 2] == 0
    # neighbours predict from a lattice value of 0 there: q = 250 everywhere else
    q = np.full((4, 4), 250)
    q[1, 1] = q[2, 2] = 0
    d = _second_difference(q)
    want = np.where((np.abs(d) >= 128) | (q == 0), 0, d + 128)
    assert np.array_equal(codes, want.astype(np.uint8))
    # the value stream: every element whose code is 0, row-major, original bits
    assert np.array_equal(v.view(np.uint32), x[(want == 0).reshape(-1)].view(np.uint32))
    y = oracle.sparse_decode(info, v, idx, 1, 4, 4, 4, eps=eps)
    assert y[5] == x[5] and y[10] == x[10] and np.abs(y[[0, 1, 15]] - 0.5).max() <= eps


def test_sparse_blocks_are_untouched_by_the_error_bound_and_eps_zero_is_verbatim():
    maps, h, w, n = 4, 28, 28, 4
    x = W.salient_feature_maps(maps, h, w, seed=3)
    info0, v0, idx0, t0 = oracle.sparse_encode(x, maps, h, w, n, 0.5)
    info1, v1, idx1, t1 = oracle.sparse_encode(x, maps, h, w, n, 0.5, eps=0.02)
    sparse = (info0 & 0x80) == 0
    assert np.array_equal(sparse, (info1 & 0x80) == 0) and np.array_equal(info0[sparse], info1[sparse])
    assert t0[2] == t1[2] and t0[3] == t1[3]
    y = oracle.sparse_decode(info1, v1, idx1, maps, h, w, n, eps=0.02)
    # elements of sparse blocks are exact, elements of dense blocks within the bound
    BH = BW = 7
    blk_of = (np.arange(h)[:, None] // n) * BW + (np.arange(w)[None, :] // n)
    in_sparse = sparse.reshape(maps, BH * BW)[:, blk_of.reshape(-1)].reshape(maps, h, w).reshape(-1)
    assert np.array_equal(y[in_sparse], x[in_sparse])
    assert np.abs(y - x).max() <= 0.02 * (1 + 1e-5) + np.abs(x).max() * 2.0 ** -22
    assert v1.size < v0.size                                                 # dense blocks now cost bytes, not floats
    for bad in (0.0, -1.0, float("nan")):
        i2, v2, x2, t2 = oracle.sparse_encode(x, maps, h, w, n, 0.5, eps=bad)
        assert np.array_equal(i2, info0) and np.array_equal(v2, v0) and np.array_equal(x2, idx0)


def test_decoder_rejects_an_outlier_count_that_does_not_match_the_codes():
    x = W.salient_feature_maps(1, 8, 8, seed=1, zero_level=-1.0)
    info, v, idx, _ = _dense_everything(x, 1, 8, 8, 4, 0.05)
    bad = info.copy()
    bad[0] = 0x80 | ((info[0] & 0x7F) + 1)
    with pytest.raises(ValueError):
        oracle.sparse_decode(bad, np.concatenate([v, v[:1]]), idx, 1, 8, 8, 4, eps=0.05)


def test_a_value_without_a_lattice_point_is_an_outlier_even_where_the_prediction_error_is_small():
    # all zeros but two elements: their lattice value is taken as 0, so every prediction error
    # is 0 -- they must still go to the value stream, and their neighbours must stay coded
    eps = 0.5                                               # lattice step 1
    x = np.zeros(64, f32)
    x[27] = 5.0e6                                           # 2^22 <= |x / step| < 2^23: no lattice point
    x[45] = -np.inf
    info, v, idx, _ = _dense_everything(x, 1, 8, 8, 8, eps)
    want = np.full(64, 128, np.uint8)
    want[[27, 45]] = 0
    assert np.array_equal(idx, want) and info.tolist() == [0x80 | 2]
    assert np.array_equal(v.view(np.uint32), x[[27, 45]].view(np.uint32))
    y = oracle.sparse_decode(info, v, idx, 1, 8, 8, 8, eps=eps)
    assert np.array_equal(y.view(np.uint32), x.view(np.uint32))
    # just below the limit the value is on the lattice and its neighbours feel it
    x[27] = 4.0e6
    info, v, idx, _ = _dense_everything(x, 1, 8, 8, 8, eps)
    assert (idx.reshape(8, 8)[3:5, 3:5] == 0).all()         # itself, right, below, diagonal: |d| = 4e6


def test_the_lattice_ends_just_below_two_to_the_22_steps():
    eps = 0.5
    for value, on_lattice in ((2.0 ** 22, False), (2.0 ** 22 - 1, True), (-(2.0 ** 22), False)):
        x = np.zeros(16, f32)
        x[5] = value
        info, v, idx, _ = _dense_everything(x, 1, 4, 4, 4, eps)
        neighbours_coded = (idx.reshape(4, 4)[1, 2] != 0) and (idx.reshape(4, 4)[2, 1] != 0)
        assert neighbours_coded == (not on_lattice)
        assert info[0] == (0x80 | (4 if on_lattice else 1))
