"""Pins for the oracle of salient-channel routing (Section 4.4.1, Channel-wise Mix
Compression: only normal channels go through the linear-scale quantiser, so that outliers
do not stretch its range; salient channels are kept verbatim by this library).  The paper
prints no worked example; the pins are reductions to the already pinned plain quantiser,
explicit index arithmetic, error bounds that only hold when salient values are excluded
from the statistics, brute force on tiny tensors, and an independent numpy twin."""
from __future__ import annotations

import numpy as np
import pytest

import oracle
from np_quantiser import compress_mixed_np, compress_np
from paper_2510_11400_amd import workloads as W

f32 = np.float32


def _bf16_bits(x32):
    u = x32.view(np.uint32).astype(np.uint64)
    return ((u + 0x7FFF + ((u >> 16) & 1)) >> 16).astype(np.uint16)


def _widen(b16):
    return (b16.astype(np.uint32) << 16).view(np.float32)


# ---- slots -------------------------------------------------------------------------------

def test_slots_number_salient_channels_in_order_and_stop_at_the_cap():
    mask = np.array([0, 1, 1, 0, 0, 1, 0, 1, 1, 0], dtype=np.uint8)
    slots, used = oracle.channel_slots(mask, 10)
    assert used == 5 and slots.tolist() == [-1, 0, 1, -1, -1, 2, -1, 3, 4, -1]
    slots, used = oracle.channel_slots(mask, 3)          # the last two salient channels do not fit
    assert used == 3 and slots.tolist() == [-1, 0, 1, -1, -1, 2, -1, -1, -1, -1]
    slots, used = oracle.channel_slots(mask, 0)
    assert used == 0 and (slots == -1).all()
    slots, used = oracle.channel_slots(np.ones(7, np.uint8) * 200, 7)      # any non-zero byte is salient
    assert used == 7 and slots.tolist() == list(range(7))


@pytest.mark.parametrize("seed", range(6))
def test_slots_match_a_cumulative_count(seed):
    rng = np.random.default_rng(seed)
    C = int(rng.integers(1, 3000))
    mask = (rng.random(C) < rng.choice([0.0, 0.02, 0.5, 1.0])).astype(np.uint8)
    cap = int(rng.integers(0, C + 1))
    slots, used = oracle.channel_slots(mask, cap)
    m64 = mask.astype(np.int64)
    rank = np.cumsum(m64) - m64                           # salient channels before c
    want = np.where((mask == 1) & (rank < cap), rank, -1)
    assert used == min(int(mask.sum()), cap)
    assert (slots == want).all()


def test_slots_reject_bad_arguments():
    with pytest.raises(ValueError):
        oracle.channel_slots(np.zeros(4, np.uint8), 5)    # more raw rows than channels
    with pytest.raises(ValueError):
        oracle.channel_slots(np.zeros(4, np.uint8), -1)
    with pytest.raises(ValueError):
        oracle.channel_slots(np.zeros(16385, np.uint8), 1)


# ---- reductions to the plain quantiser -----------------------------------------------------

@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("G,B,rounding", [(64, 2, "stochastic"), (128, 4, "nearest"), (256, 8, "stochastic")])
def test_without_salient_channels_it_is_the_plain_quantiser(dtype, G, B, rounding):
    rng = np.random.default_rng(G + B)
    outer, C, inner = 3, 37, 29
    x = rng.standard_normal(outer * C * inner).astype(f32)
    xin = x if dtype == "f32" else _bf16_bits(x)
    slots = np.full(C, -1, np.int16)
    p, m, raw = oracle.compress_mixed(xin, outer, C, inner, slots, 0, G, B, rounding, 11, 5, dtype=dtype)
    p0, m0 = oracle.compress(xin, G, B, rounding, 11, 5, dtype=dtype)
    assert raw.size == 0 and (p == p0).all() and (m.view(np.uint32) == m0.view(np.uint32)).all()
    for od in ("f32", "bf16"):
        y = oracle.decompress_mixed(p, m, raw, outer, C, inner, slots, 0, G, B, raw_dtype=dtype, out_dtype=od)
        y0 = oracle.decompress(p0, m0, x.size, G, B, out_dtype=od)
        assert (y.view(np.uint8) == y0.view(np.uint8)).all()
    # slots that point outside the raw store mean "normal" too
    wild = np.full(C, 9, np.int16)
    p1, m1, _ = oracle.compress_mixed(xin, outer, C, inner, wild, 4, G, B, rounding, 11, 5, dtype=dtype)
    assert (p1 == p0).all() and (m1.view(np.uint32) == m0.view(np.uint32)).all()


@pytest.mark.parametrize("G,B,rounding", [(64, 4, "nearest"), (128, 2, "stochastic"), (256, 8, "nearest")])
def test_groups_inside_one_channel_are_either_plain_or_empty(G, B, rounding):
    """inner is a multiple of the group size, so no group mixes channels: a group of a normal
    channel carries exactly the bytes the plain quantiser gives it (same element indices,
    hence the same random bits), a group of a kept channel is all zero."""
    rng = np.random.default_rng(B)
    outer, C, inner = 2, 9, 2 * G
    x = (rng.standard_normal(outer * C * inner) * rng.choice([0.1, 1, 30], outer * C * inner)).astype(f32)
    mask = np.zeros(C, np.uint8)
    mask[[1, 4, 8]] = 1
    slots, used = oracle.channel_slots(mask, 3)
    p, m, raw = oracle.compress_mixed(x, outer, C, inner, slots, 3, G, B, rounding, 77, 3)
    p0, m0 = oracle.compress(x, G, B, rounding, 77, 3)
    gpr = inner // G                                      # groups per channel run
    bpg = G * B // 8                                      # code bytes per group
    for g in range(outer * C * gpr):
        c = (g // gpr) % C
        got = p[g * bpg:(g + 1) * bpg]
        if mask[c]:
            assert not got.any() and m[g, 0] == 0 and m[g, 1] == 0
        else:
            assert (got == p0[g * bpg:(g + 1) * bpg]).all()
            assert (m[g].view(np.uint32) == m0[g].view(np.uint32)).all()


# ---- the raw store ------------------------------------------------------------------------

@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("outer,C,inner", [(4, 10, 7), (3, 16, 1), (1, 5, 300), (5, 1, 13)])
def test_raw_store_holds_the_kept_channels_bit_for_bit(dtype, outer, C, inner):
    rng = np.random.default_rng(outer * 100 + C)
    x = rng.standard_normal(outer * C * inner).astype(f32)
    x[rng.integers(0, x.size, 5)] = -0.0                  # sign of zero must survive
    xin = x if dtype == "f32" else _bf16_bits(x)
    mask = (rng.random(C) < 0.4).astype(np.uint8)
    mask[0] = 1
    cap = int(mask.sum()) + 1 if int(mask.sum()) < C else C   # one spare row when there is room
    slots, used = oracle.channel_slots(mask, cap)
    fill = 0x5A5A if dtype == "bf16" else f32(123.25)
    _, _, raw = oracle.compress_mixed(xin, outer, C, inner, slots, cap, 64, 4, dtype=dtype, raw_fill=fill)
    raw3 = raw.reshape(outer, cap, inner)
    x3 = xin.reshape(outer, C, inner)
    kept = np.flatnonzero(mask)
    itemview = np.uint32 if dtype == "f32" else np.uint16
    assert (raw3[:, :used, :].view(itemview) == x3[:, kept, :].view(itemview)).all()
    if cap > used:                                        # spare rows were not touched
        assert (raw3[:, used:, :] == fill).all()


# ---- what the routing is for: outliers no longer stretch the range ---------------------------

@pytest.mark.parametrize("inner,rounding", [(1, "nearest"), (1, "stochastic"), (49, "nearest"), (256, "stochastic")])
def test_normal_elements_keep_the_error_bound_of_their_own_range(inner, rounding):
    rng = np.random.default_rng(inner)
    outer, C, G, B = (64, 96, 64, 4) if inner == 1 else (3, 24, 64, 4)
    x = rng.uniform(-1, 1, outer * C * inner).astype(f32)
    x3 = x.reshape(outer, C, inner)
    sal = np.array([3, 10, 17])
    x3[:, sal, :] *= f32(1000.0)                          # outlier-rich channels
    mask = np.zeros(C, np.uint8)
    mask[sal] = 1
    slots, used = oracle.channel_slots(mask, 3)
    p, m, raw = oracle.compress_mixed(x, outer, C, inner, slots, 3, G, B, rounding, 5, 9)
    y = oracle.decompress_mixed(p, m, raw, outer, C, inner, slots, 3, G, B)
    y3 = y.reshape(outer, C, inner)
    # kept channels come back exactly
    assert (y3[:, sal, :].view(np.uint32) == x3[:, sal, :].view(np.uint32)).all()
    # normal values lie in [-1, 1]: the range of any group is at most 2, so the step is at most
    # 2/15 -- with the outliers inside the statistics it would be near 2000/15
    normal = np.ones(C, bool)
    normal[sal] = False
    err = np.abs(y3[:, normal, :].astype(np.float64) - x3[:, normal, :].astype(np.float64))
    step = 2.0 / 15
    assert err.max() <= (step / 2 if rounding == "nearest" else step) * (1 + 1e-5)
    assert m[:, 0].max() <= f32(step) * f32(1 + 1e-6)


def test_group_statistics_by_brute_force_on_tiny_tensors():
    rng = np.random.default_rng(1)
    G, B = 64, 8
    for trial in range(30):
        outer, C, inner = int(rng.integers(1, 5)), int(rng.integers(1, 40)), int(rng.integers(1, 9))
        n = outer * C * inner
        x = rng.standard_normal(n).astype(f32)
        mask = (rng.random(C) < 0.3).astype(np.uint8)
        cap = int(rng.integers(0, C + 1))
        slots, used = oracle.channel_slots(mask, cap)
        p, m, raw = oracle.compress_mixed(x, outer, C, inner, slots, cap, G, B)
        codes = oracle.unpack_codes(p, n, B)
        for g in range((n + G - 1) // G):
            vals = []
            for i in range(g * G, min(n, (g + 1) * G)):
                c = (i // inner) % C
                if slots[c] >= 0:
                    assert codes[i] == 0
                else:
                    vals.append(x[i])
            if not vals:
                assert m[g, 0] == 0 and m[g, 1] == 0
                continue
            mn, mx = min(vals), max(vals)
            assert m[g, 1] == mn + f32(0)
            rngf = f32(mx) - f32(mn)
            assert m[g, 0] == (f32(0) if rngf < f32(2.0 ** -100) else f32(rngf / f32(255)))
        # the extreme normal elements of a non-degenerate group get codes 0 and L
        for g in range((n + G - 1) // G):
            idx = [i for i in range(g * G, min(n, (g + 1) * G)) if slots[(i // inner) % C] < 0]
            if len(idx) >= 2 and m[g, 0] > 0:
                v = x[idx]
                assert codes[idx[int(np.argmin(v))]] == 0 and codes[idx[int(np.argmax(v))]] == 255


# ---- the independent numpy twin --------------------------------------------------------------

@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("outer,C,inner,G,B,rounding", [
    (16, 64, 1, 64, 2, "stochastic"),
    (7, 33, 1, 128, 4, "nearest"),
    (2, 12, 49, 64, 8, "stochastic"),
    (3, 5, 196, 256, 4, "stochastic"),
    (1, 3, 1000, 128, 2, "nearest"),
    (5, 17, 6, 64, 8, "nearest"),
])
def test_against_the_numpy_twin(dtype, outer, C, inner, G, B, rounding):
    rng = np.random.default_rng(outer * 31 + C)
    n = outer * C * inner
    x = (rng.standard_normal(n) * rng.choice([0.01, 1, 50], n)).astype(f32)
    if dtype == "bf16":
        xin = _bf16_bits(x)
        x = _widen(xin)
    else:
        xin = x
    mask = (rng.random(C) < 0.25).astype(np.uint8)
    cap = max(1, int(mask.sum()) - 1)                     # one salient channel too many for the store
    slots, used = oracle.channel_slots(mask, cap)
    p, m, raw = oracle.compress_mixed(xin, outer, C, inner, slots, cap, G, B, rounding, 1234, 42, dtype=dtype)
    pn, mn_, codes = compress_mixed_np(x, outer, C, inner, slots >= 0, G, B, rounding, 1234, 42)
    assert (p == pn).all()
    assert (m.view(np.uint32) == mn_.view(np.uint32)).all()
    # restore: kept channels from the raw store, the rest as the plain inverse gives it
    y = oracle.decompress_mixed(p, m, raw, outer, C, inner, slots, cap, G, B, raw_dtype=dtype, out_dtype="f32")
    plain = oracle.decompress(p, m, n, G, B, out_dtype="f32")
    kept_elem = np.broadcast_to((slots >= 0)[None, :, None], (outer, C, inner)).reshape(n)
    want = np.where(kept_elem, x, plain)
    assert (y.view(np.uint32) == want.view(np.uint32)).all()


def test_restore_converts_raw_values_to_the_output_dtype():
    rng = np.random.default_rng(8)
    outer, C, inner = 2, 6, 40
    x = rng.standard_normal(outer * C * inner).astype(f32)
    mask = np.array([1, 0, 0, 1, 0, 0], np.uint8)
    slots, _ = oracle.channel_slots(mask, 2)
    kept_elem = np.broadcast_to((slots >= 0)[None, :, None], (outer, C, inner)).reshape(-1)
    # f32 raw -> bf16 out: nearest even
    p, m, raw = oracle.compress_mixed(x, outer, C, inner, slots, 2, 64, 8)
    y = oracle.decompress_mixed(p, m, raw, outer, C, inner, slots, 2, 64, 8, raw_dtype="f32", out_dtype="bf16")
    assert (y[kept_elem] == _bf16_bits(x)[kept_elem]).all()
    # bf16 raw -> f32 out: exact widening
    xb = _bf16_bits(x)
    p, m, raw = oracle.compress_mixed(xb, outer, C, inner, slots, 2, 64, 8, dtype="bf16")
    y = oracle.decompress_mixed(p, m, raw, outer, C, inner, slots, 2, 64, 8, raw_dtype="bf16", out_dtype="f32")
    assert (y[kept_elem].view(np.uint32) == _widen(xb)[kept_elem].view(np.uint32)).all()


def test_planted_outlier_channels_end_to_end_with_the_classifier():
    """classify -> slots -> mixed round trip on the generator the GPU tests use."""
    outer, C, inner = 4, 32, 64
    x, planted = W.outlier_channel_tensor(outer, C, inner, seed=3, dist="gauss")
    _, _, mask = oracle.classify_channels(x, outer, C, inner, 3.0, 8)
    assert set(np.flatnonzero(mask)) == set(int(c) for c in planted)
    slots, used = oracle.channel_slots(mask, len(planted))
    p, m, raw = oracle.compress_mixed(x, outer, C, inner, slots, used, 64, 4)
    y = oracle.decompress_mixed(p, m, raw, outer, C, inner, slots, used, 64, 4)
    x3, y3 = x.reshape(outer, C, inner), y.reshape(outer, C, inner)
    assert (y3[:, planted, :] == x3[:, planted, :]).all()
    plain = oracle.decompress(*oracle.compress(x, 64, 4), x.size, 64, 4).reshape(outer, C, inner)
    normal = np.setdiff1d(np.arange(C), planted)
    assert np.abs(y3[:, normal] - x3[:, normal]).max() <= np.abs(plain[:, normal] - x3[:, normal]).max()


def test_rejects_bad_arguments():
    x = np.zeros(2 * 4 * 8, f32)
    slots = np.full(4, -1, np.int16)
    with pytest.raises(ValueError):
        oracle.compress_mixed(x, 2, 4, 8, slots, 5, 64, 4)          # raw_channels > channels
    with pytest.raises(ValueError):
        oracle.compress_mixed(x, 2, 4, 8, slots, 0, 32, 4)          # group size
    with pytest.raises(ValueError):
        oracle.compress_mixed(x, 2, 4, 8, slots, 0, 64, 3)          # bits
    p, m, raw = oracle.compress_mixed(np.zeros(0, f32), 0, 4, 8, slots, 2, 64, 4)   # empty tensor
    assert p.size == 0 and m.size == 0 and raw.size == 0


def test_zero_point_of_a_group_whose_normal_minimum_is_negative_zero_is_positive_zero():
    outer, C, inner = 1, 2, 64
    x = np.zeros(outer * C * inner, f32)
    x[:64] = -5.0                                         # channel 0, kept: far below everything else
    x[64:128] = np.linspace(0, 1, 64, dtype=f32)
    x[64] = -0.0                                          # the normal minimum
    slots = np.array([0, -1], np.int16)
    for G in (64, 128):                                   # G = 128: one group holding both channels
        p, m, raw = oracle.compress_mixed(x, outer, C, inner, slots, 1, G, 8)
        g = 64 // G
        assert m[g, 1].view(np.uint32) == 0               # +0.0, not -0.0 (and not -5)
        assert m[g, 0] == f32(1.0) / f32(255)
