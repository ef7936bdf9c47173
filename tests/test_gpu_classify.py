"""Parity of the HIP channel classification with the CPU oracle (Section 4.4.1: outliers
by the three-sigma rule, channels sorted into salient and normal).  Bar: mean, variance
and threshold bit-exact (binary64, pairwise sums in a fixed tree), outlier counts and the
salient mask exact."""
from __future__ import annotations

import numpy as np
import pytest

import oracle
from paper_2510_11400_amd import workloads as W

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu
f32 = np.float32


@pytest.fixture(scope="module")
def api():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a visible MI355X")
    from paper_2510_11400_amd import api as _api
    return _api


def _device(x, dtype):
    t = torch.from_numpy(x.view(np.int16) if dtype == "bf16" else x).cuda()
    return t.view(torch.bfloat16) if dtype == "bf16" else t


def _check(api, x, outer, C, inner, k=3.0, min_out=1, dtype="f32", name=""):
    print(f"[classify] {name} {dtype} [{outer}][{C}][{inner}] k={k} min={min_out}", flush=True)
    stats, counts, mask = oracle.classify_channels(x, outer, C, inner, k, min_out, dtype=dtype)
    gs, gc, gm = api.fh_classify_channels(_device(x, dtype), outer, C, inner, k, min_out)
    torch.cuda.synchronize()
    gs, gc, gm = gs.cpu().numpy(), gc.cpu().numpy().view(np.uint32), gm.cpu().numpy()
    assert np.array_equal(gs.view(np.uint64), stats.view(np.uint64)), f"{name}: stats {gs} vs oracle {stats}"
    assert np.array_equal(gc, counts), f"{name}: counts differ at {np.flatnonzero(gc != counts)[:8]}"
    assert np.array_equal(gm, mask), f"{name}: mask differs"
    return counts, mask


SHAPES = [(1, 1, 1), (1, 3, 5), (2, 7, 49), (4, 16, 196), (3, 5, 1000), (8, 64, 1024), (32, 64, 49),
          (1, 2, 40000), (2, 3, 70001), (300, 768, 1), (17, 3072, 1), (5, 16384, 3), (64, 128, 7 * 7),
          (2, 1, 1024), (1, 1, 1025), (1, 1, 4096 * 3 + 17)]


@pytest.mark.parametrize("shape", SHAPES)
def test_shapes_and_layouts(api, shape):
    outer, C, inner = shape
    x, planted = W.outlier_channel_tensor(outer, C, inner, seed=outer + inner, salient_fraction=0.1)
    _check(api, x, outer, C, inner, 3.0, max(1, outer * inner // 40), name="shape")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("k", [1.0, 2.0, 3.0, 4.5])
def test_thresholds_and_dtypes(api, dtype, k):
    x, _ = W.outlier_channel_tensor(24, 96, 28 * 28, seed=int(k * 10), dist="relu", dtype=dtype,
                                    magnitude=81.0 if dtype == "f32" else 347.0)
    for min_out in (1, 50, 10 ** 6):
        _check(api, x, 24, 96, 28 * 28, k, min_out, dtype=dtype, name="k")


def test_planted_channels_are_the_salient_ones(api):
    outer, C, inner = 32, 256, 14 * 14
    x, planted = W.outlier_channel_tensor(outer, C, inner, seed=7, salient_fraction=0.04, hit_fraction=0.05)
    counts, mask = _check(api, x, outer, C, inner, 3.0, outer * inner // 100, name="planted")
    assert set(np.flatnonzero(mask)) == set(int(c) for c in planted)


def test_degenerate_inputs(api):
    for value in (0.0, -3.25):
        x = np.full(6 * 10 * 50, value, dtype=f32)
        counts, mask = _check(api, x, 6, 10, 50, name="constant")
        assert not counts.any() and not mask.any()
    for n in (1, 5, 1024, 1500):                             # negative zeros of any length
        _check(api, np.full(n, -0.0, dtype=f32), 1, 1, n, name="negative zeros")
    # empty outer: outputs are zeroed, nothing is read
    gs, gc, gm = api.fh_classify_channels(torch.empty(0, device="cuda"), 0, 12, 9)
    torch.cuda.synchronize()
    assert gs.cpu().tolist() == [0.0, 0.0, 0.0, 0.0] and not gc.cpu().numpy().any() and not gm.cpu().numpy().any()


def test_workspace_and_outputs_can_be_reused_between_calls(api):
    outer, C, inner = 16, 40, 333
    n = outer * C * inner
    ws = torch.empty(api.classify_workspace_bytes(n), dtype=torch.uint8, device="cuda")
    stats = torch.empty(4, dtype=torch.float64, device="cuda")
    counts = torch.full((C,), 12345, dtype=torch.int32, device="cuda")      # stale values must vanish
    mask = torch.full((C,), 7, dtype=torch.uint8, device="cuda")
    for seed in (1, 2, 3):
        x, _ = W.outlier_channel_tensor(outer, C, inner, seed=seed)
        want = oracle.classify_channels(x, outer, C, inner, 3.0, 20)
        api.fh_classify_channels(_device(x, "f32"), outer, C, inner, 3.0, 20, workspace=ws, stats=stats,
                                 counts=counts, mask=mask)
        torch.cuda.synchronize()
        assert np.array_equal(stats.cpu().numpy().view(np.uint64), want[0].view(np.uint64))
        assert np.array_equal(counts.cpu().numpy().view(np.uint32), want[1])
        assert np.array_equal(mask.cpu().numpy(), want[2])


@pytest.mark.timeout(600)
def test_paper_sized_activation_set(api):
    # the five per-sample shapes of the paper's local-engine ablation, at batch 64
    for i, (C, h, w) in enumerate(W.ABLATION_SHAPES):
        x, planted = W.outlier_channel_tensor(64, C, h * w, seed=100 + i, dist="relu")
        counts, mask = _check(api, x, 64, C, h * w, 3.0, 64 * h * w // 100, name="ablation")
        assert set(int(c) for c in planted) <= set(np.flatnonzero(mask))


# ---- the batched call --------------------------------------------------------------------------

def test_batched_call_matches_the_oracle_for_every_item(api):
    """More items than one launch holds, both dtypes (so several runs), an empty tensor, a tensor
    whose partial sums need a second tree level, very different channel counts."""
    shapes = [(4, 16, 196, "f32"), (2, 7, 49, "f32"), (300, 768, 1, "bf16"), (0, 12, 9, "f32"), (1, 3, 1_100_000, "f32"),
              (5, 16384, 3, "f32"), (64, 32, 49, "bf16")] + [(3, 5 + i, 100 + 7 * i, "f32") for i in range(14)]
    entries, host = [], []
    for i, (outer, C, inner, dtype) in enumerate(shapes):
        x, _ = W.outlier_channel_tensor(max(outer, 1), C, inner, seed=100 + i, salient_fraction=0.1, dtype=dtype)
        x = x[: outer * C * inner]
        host.append(x)
        k, mo = (3.0, max(1, outer * inner // 50)) if i % 2 == 0 else (2.0, 3)
        entries.append(api.ClassifyEntry(_device(x, dtype) if x.size else torch.empty(0, device="cuda"),
                                         outer, C, inner, k, mo))
    assert len(entries) > api.classify_batch_capacity()
    batch = api.ClassifyBatch(entries)
    print(f"[classify] batch of {len(entries)} tensors", flush=True)
    api.fh_classify_channels_batch(batch)
    torch.cuda.synchronize()
    for i, ((outer, C, inner, dtype), x, e) in enumerate(zip(shapes, host, entries)):
        stats, counts, mask = oracle.classify_channels(x, outer, C, inner, e.k_sigma, e.min_outliers, dtype=dtype)
        assert np.array_equal(e.stats.cpu().numpy().view(np.uint64), stats.view(np.uint64)), f"item {i}: stats"
        assert np.array_equal(e.counts.cpu().numpy().view(np.uint32), counts), f"item {i}: counts"
        assert np.array_equal(e.mask.cpu().numpy(), mask), f"item {i}: mask"
    # a second call on the same batch (buffers reused) gives the same answers
    api.fh_classify_channels_batch(batch)
    torch.cuda.synchronize()
    for (outer, C, inner, dtype), x, e in zip(shapes, host, entries):
        _, counts, _ = oracle.classify_channels(x, outer, C, inner, e.k_sigma, e.min_outliers, dtype=dtype)
        assert np.array_equal(e.counts.cpu().numpy().view(np.uint32), counts)


def test_batched_call_on_the_full_size_set(api):
    shapes = ((64, 32, 112 * 112), (64, 96, 112 * 112), (64, 144, 56 * 56), (64, 192, 28 * 28), (64, 384, 14 * 14))
    entries, host = [], []
    for i, (outer, C, inner) in enumerate(shapes):
        x, _ = W.outlier_channel_tensor(outer, C, inner, seed=i, dist="relu")
        host.append(x)
        entries.append(api.ClassifyEntry(torch.from_numpy(x).cuda(), outer, C, inner, 3.0, outer * inner // 100))
    api.fh_classify_channels_batch(api.ClassifyBatch(entries))
    torch.cuda.synchronize()
    for (outer, C, inner), x, e in zip(shapes, host, entries):
        stats, counts, mask = oracle.classify_channels(x, outer, C, inner, 3.0, outer * inner // 100)
        assert np.array_equal(e.stats.cpu().numpy().view(np.uint64), stats.view(np.uint64))
        assert np.array_equal(e.counts.cpu().numpy().view(np.uint32), counts)
        assert np.array_equal(e.mask.cpu().numpy(), mask)
