"""Pins for the oracle of the sparse-block storage of salient-channel maps (Section 4.4.1:
binary non-zero mask, mean filtering by n x n average pooling against a threshold tau, sparse
blocks in Compressed Sparse Row format, zeros preserved).  The paper prints no worked example;
the pins are library routines that implement the same textbook objects (scipy's CSR, torch's
average pooling), hand-written tiny cases, stream bookkeeping and the lossless round trip."""
from __future__ import annotations

import numpy as np
import pytest
import scipy.sparse as sp

import oracle
from paper_2510_11400_amd import workloads as W

f32 = np.float32


def _walk(info, values, indices, maps, h, w, n):
    """Cut the two streams back into per-block pieces with running offsets."""
    BH, BW = -(-h // n), -(-w // n)
    nv = ni = 0
    out = []
    b = 0
    for m in range(maps):
        for bi in range(BH):
            for bj in range(BW):
                rows, cols = min(n, h - bi * n), min(n, w - bj * n)
                count = int(info[b] & 0x7F)
                if info[b] & 0x80:
                    out.append(("dense", m, bi, bj, rows, cols, values[nv:nv + count], None, None))
                    nv += count
                else:
                    rp = indices[ni:ni + rows + 1]
                    col = indices[ni + rows + 1:ni + rows + 1 + count]
                    out.append(("sparse", m, bi, bj, rows, cols, values[nv:nv + count], rp, col))
                    nv += count
                    ni += rows + 1 + count
                b += 1
    assert nv == len(values) and ni == len(indices)
    return out


def _maps(maps, h, w, seed, zero_level=0.3, dtype="f32"):
    return W.salient_feature_maps(maps, h, w, seed=seed, zero_level=zero_level, dtype=dtype)


def test_a_hand_written_map():
    # 3 x 5 map, n = 2: blocks (rows x cols) 2x2 2x2 2x1 / 1x2 1x2 1x1
    x = np.array([[0, 7, 0, 0, 9],
                  [0, 0, 0, 3, 0],
                  [5, 6, 0, 0, 0]], dtype=f32)
    info, v, idx, t = oracle.sparse_encode(x.reshape(-1), 1, 3, 5, 2, 0.5)
    # densities: 1/4, 1/4, 1/2 | 2/2, 0/2, 0/1 -> all sparse except the 1x2 block [5, 6]
    assert info.tolist() == [1, 1, 1, 0x80 | 2, 0, 0]
    assert v.tolist() == [7, 3, 9, 5, 6]
    assert idx.tolist() == [0, 1, 1, 1,      # block 0: row_ptr 0,1,1; col 1
                            0, 0, 1, 1,      # block 1: row_ptr 0,0,1; col 1 (the 3 sits at column 3 = 1 in the block)
                            0, 1, 1, 0,      # block 2 (one column): row_ptr 0,1,1; col 0
                            0, 0,            # block 4: one row, empty
                            0, 0]            # block 5: one row, empty
    assert t.tolist() == [5, 16, 5, 1]
    y = oracle.sparse_decode(info, v, idx, 1, 3, 5, 2)
    assert np.array_equal(y.reshape(3, 5), x)


@pytest.mark.parametrize("n", [2, 4, 8])
@pytest.mark.parametrize("h,w", [(8, 8), (7, 7), (14, 14), (28, 28), (13, 29), (1, 1), (1, 40), (33, 2)])
def test_sparse_blocks_are_scipys_csr_of_the_block(n, h, w):
    maps = 3
    x = _maps(maps, h, w, seed=h * 100 + w + n)
    info, v, idx, _ = oracle.sparse_encode(x, maps, h, w, n, 0.6)
    x3 = x.reshape(maps, h, w)
    kinds = set()
    for kind, m, bi, bj, rows, cols, vals, rp, col in _walk(info, v, idx, maps, h, w, n):
        block = x3[m, bi * n:bi * n + rows, bj * n:bj * n + cols]
        assert block.shape == (rows, cols)
        kinds.add(kind)
        if kind == "dense":
            assert np.array_equal(vals, block.reshape(-1))
        else:
            ref = sp.csr_matrix(block)
            ref.sort_indices()
            assert np.array_equal(rp, ref.indptr) and np.array_equal(col, ref.indices)
            assert np.array_equal(vals, ref.data)
    if h * w >= 28 * 28:
        assert kinds == {"dense", "sparse"}


@pytest.mark.parametrize("n", [2, 4, 8])
@pytest.mark.parametrize("tau", [0.0, 0.2, 0.3, 0.5, 0.75, 1.0])
def test_the_split_is_average_pooling_of_the_nonzero_mask_against_tau(n, tau):
    torch = pytest.importorskip("torch")
    maps, h, w = 4, 27, 22                                  # edge blocks of several shapes
    x = _maps(maps, h, w, seed=n)
    info, _, _, totals = oracle.sparse_encode(x, maps, h, w, n, tau)
    mask = torch.from_numpy((x.reshape(maps, 1, h, w) != 0).astype(f32))
    density = torch.nn.functional.avg_pool2d(mask, n, stride=n, ceil_mode=True, count_include_pad=False)
    sparse = (density <= f32(tau)).numpy().reshape(-1)
    assert np.array_equal((info & 0x80) == 0, sparse)
    assert totals[2] == sparse.sum() and totals[3] == (~sparse).sum()
    # counts: non-zeros for sparse blocks, area for dense ones
    nnz = torch.nn.functional.avg_pool2d(mask, n, stride=n, ceil_mode=True, divisor_override=1).numpy().reshape(-1)
    area = torch.nn.functional.avg_pool2d(torch.ones_like(mask), n, stride=n, ceil_mode=True,
                                          divisor_override=1).numpy().reshape(-1)
    assert np.array_equal(info & 0x7F, np.where(sparse, nnz, area).astype(np.uint8))


def test_threshold_extremes():
    maps, h, w, n = 2, 20, 20, 4
    x = _maps(maps, h, w, seed=9)
    x3 = x.reshape(maps, h, w)
    # tau < 0: nothing is sparse, the value stream is the input in block order
    info, v, idx, t = oracle.sparse_encode(x, maps, h, w, n, -1.0)
    assert (info == (0x80 | 16)).all() and idx.size == 0 and t.tolist() == [maps * h * w, 0, 0, 50]
    blocks = x3.reshape(maps, 5, 4, 5, 4).transpose(0, 1, 3, 2, 4).reshape(-1)
    assert np.array_equal(v, blocks)
    # tau = 0: exactly the all-zero blocks are sparse and they store no value
    info, v, idx, t = oracle.sparse_encode(x, maps, h, w, n, 0.0)
    zero_block = ~(x3.reshape(maps, 5, 4, 5, 4) != 0).any(axis=(2, 4)).reshape(-1)
    assert np.array_equal((info & 0x80) == 0, zero_block) and (info[zero_block] == 0).all()
    assert idx.size == 5 * zero_block.sum()                 # row_ptr only: n + 1 zeros each
    # tau >= 1: everything is sparse, the value stream holds exactly the non-zeros
    info, v, idx, t = oracle.sparse_encode(x, maps, h, w, n, 1.0)
    assert ((info & 0x80) == 0).all() and v.size == np.count_nonzero(x) and t[3] == 0
    assert idx.size == 50 * 5 + v.size
    # NaN threshold: no comparison holds, so nothing is sparse
    info, _, _, t = oracle.sparse_encode(x, maps, h, w, n, float("nan"))
    assert t[2] == 0


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("n", [2, 4, 8])
def test_round_trip_is_lossless_including_negative_zero(dtype, n):
    rng = np.random.default_rng(n)
    for (maps, h, w) in ((1, 1, 1), (2, 5, 3), (3, 16, 16), (5, 14, 14), (2, 57, 31), (1, 112, 112)):
        x = _maps(maps, h, w, seed=maps + h, dtype=dtype)
        neg = rng.integers(0, x.size, max(1, x.size // 50))
        if dtype == "f32":
            x[neg] = -0.0
            x[rng.integers(0, x.size, 3)] = -2.5             # negative values are values too
        else:
            x[neg] = 0x8000
        for tau in (0.0, 0.4, 1.0):
            info, v, idx, t = oracle.sparse_encode(x, maps, h, w, n, tau, dtype=dtype)
            y = oracle.sparse_decode(info, v, idx, maps, h, w, n, dtype=dtype)
            assert np.array_equal(y.view(np.uint8), x.view(np.uint8))
            assert t[0] == v.size and t[1] == idx.size and t[2] + t[3] == info.size


def test_stream_sizes_follow_from_the_block_table():
    maps, h, w, n = 7, 30, 19, 4
    x = _maps(maps, h, w, seed=2, zero_level=0.8)
    info, v, idx, t = oracle.sparse_encode(x, maps, h, w, n, 0.5)
    pieces = _walk(info, v, idx, maps, h, w, n)             # asserts both streams are consumed exactly
    assert len(pieces) == oracle.sparse_blocks(maps, h, w, n) == maps * 8 * 5
    assert t[0] == sum(len(p[6]) for p in pieces)
    assert t[1] == sum(p[4] + 1 + len(p[6]) for p in pieces if p[0] == "sparse")
    # sparser input stores less
    dense_in = _maps(maps, h, w, seed=2, zero_level=-0.5)
    _, v2, idx2, _ = oracle.sparse_encode(dense_in, maps, h, w, n, 0.5)
    assert v.size < v2.size


def test_rejects_bad_arguments_and_inconsistent_streams():
    x = np.zeros(2 * 4 * 4, f32)
    for bad_n in (1, 3, 16):
        with pytest.raises(ValueError):
            oracle.sparse_encode(x, 2, 4, 4, bad_n, 0.5)
    with pytest.raises(ValueError):
        oracle.sparse_encode(x, 2, 4, 5, 2, 0.5)            # size mismatch
    info, v, idx, t = oracle.sparse_encode(np.zeros(0, f32), 0, 4, 4, 2, 0.5)
    assert info.size == 0 and t.tolist() == [0, 0, 0, 0]
    x = _maps(1, 8, 8, seed=1)
    info, v, idx, _ = oracle.sparse_encode(x, 1, 8, 8, 4, 1.0)
    broken = idx.copy()
    broken[0] = 3                                           # row_ptr[0] must be 0
    with pytest.raises(ValueError):
        oracle.sparse_decode(info, v, broken, 1, 8, 8, 4)
