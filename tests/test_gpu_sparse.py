"""Parity of the HIP sparse-block storage with the CPU oracle (Section 4.4.1: non-zero mask,
n x n average pooling against tau, sparse blocks in CSR form, zeros preserved).  Bar: the info
bytes, both streams up to the reported totals, the totals and the restored maps all bit-exact."""
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


def _host(t, dtype):
    t = t.cpu()
    return t.view(torch.int16).numpy().view(np.uint16) if dtype == "bf16" else t.numpy()


def _bits(a):
    return a.view(np.uint32) if a.dtype == np.float32 else a


def _check(api, x, maps, h, w, n, tau, dtype="f32", name="", eps=0.0):
    print(f"[sparse] {name} {dtype} [{maps}][{h}][{w}] n={n} tau={tau} eps={eps}", flush=True)
    info, v, idx, totals = oracle.sparse_encode(x, maps, h, w, n, tau, dtype=dtype, eps=eps)
    dx = _device(x, dtype)
    b = api.fh_sparse_encode(dx, maps, h, w, n, tau, eps=eps)
    torch.cuda.synchronize()
    gt = b.totals.cpu().numpy().view(np.uint64)
    assert np.array_equal(gt, totals), f"{name}: totals {gt} vs {totals}"
    nb = oracle.sparse_blocks(maps, h, w, n)
    assert np.array_equal(b.info.cpu().numpy()[:nb], info), f"{name}: info bytes differ"
    gv = _host(b.values, dtype)[:int(totals[0])]
    assert np.array_equal(_bits(gv), _bits(v)), f"{name}: value stream differs"
    gi = b.indices.cpu().numpy()[:int(totals[1])]
    assert np.array_equal(gi, idx), f"{name}: index stream differs"
    out = api.fh_sparse_decode(b.info, b.values[:int(totals[0])], b.indices[:int(totals[1])], maps, h, w, n, eps=eps)
    torch.cuda.synchronize()
    want = x if not eps > 0 else oracle.sparse_decode(info, v, idx, maps, h, w, n, dtype=dtype, eps=eps)
    assert np.array_equal(_bits(_host(out, dtype)), _bits(want)), f"{name}: restored maps differ"
    return totals


SHAPES = [(1, 1, 1), (3, 7, 7), (8, 14, 14), (5, 28, 28), (2, 56, 56), (4, 13, 29), (1, 1, 700), (2, 300, 1),
          (600, 7, 7), (3, 57, 31), (1, 112, 112), (257, 9, 10)]


@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("n", [2, 4, 8])
def test_shapes_and_windows(api, shape, n):
    maps, h, w = shape
    x = W.salient_feature_maps(maps, h, w, seed=h + w + n)
    _check(api, x, maps, h, w, n, 0.5, name="shape")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("tau", [-1.0, 0.0, 0.2, 0.3, 0.75, 1.0, float("nan")])
def test_thresholds_and_dtypes(api, dtype, tau):
    maps, h, w = 24, 27, 22
    x = W.salient_feature_maps(maps, h, w, seed=int(0 if tau != tau else abs(tau) * 10) + 3, dtype=dtype)
    rng = np.random.default_rng(1)
    x[rng.integers(0, x.size, 40)] = 0x8000 if dtype == "bf16" else -0.0       # negative zeros are values
    for n in (2, 4, 8):
        t = _check(api, x, maps, h, w, n, tau, dtype=dtype, name="tau")
        if tau != tau or tau < 0:
            assert t[2] == 0
        if tau >= 1:
            assert t[3] == 0


def test_all_zero_and_all_dense_maps(api):
    z = np.zeros(6 * 20 * 20, f32)
    t = _check(api, z, 6, 20, 20, 4, 0.5, name="zeros")
    assert t.tolist() == [0, 150 * 5, 150, 0]
    d = np.arange(1, 6 * 20 * 20 + 1, dtype=f32)
    t = _check(api, d, 6, 20, 20, 4, 0.5, name="dense")
    assert t.tolist() == [2400, 0, 0, 150]
    t = _check(api, d, 6, 20, 20, 4, 1.0, name="dense stored as CSR")
    assert t.tolist() == [2400, 150 * 5 + 2400, 150, 0]


def test_more_groups_than_the_write_pass_adds_up_itself(api):
    # beyond 2048 groups of 256 tiles the scan kernel runs between the passes
    maps, h, w, n = 9000, 16, 16, 2                         # 576000 tiles -> 2250 groups
    x = W.salient_feature_maps(maps, h, w, seed=77)
    _check(api, x, maps, h, w, n, 0.5, name="scan kernel")


def test_many_rows_of_the_scan_kernel(api):
    # a row of the scan kernel covers 512 groups; this set needs 17, the last one ragged
    maps, h, w, n = 700, 112, 112, 2                        # 2 195 200 tiles -> 8575 groups
    x = W.salient_feature_maps(maps, h, w, seed=78)
    _check(api, x, maps, h, w, n, 0.5, name="scan rounds")
    _check(api, x, maps, h, w, n, 0.5, name="scan rounds, predictive", eps=0.05)


def test_full_size_salient_channels_of_a_layer(api):
    # 4 kept channels of the 112 x 112 expanded feature map at batch 64
    maps, h, w = 64 * 4, 112, 112
    for dtype in ("f32", "bf16"):
        x = W.salient_feature_maps(maps, h, w, seed=5, dtype=dtype)
        _check(api, x, maps, h, w, 8, 0.5, dtype=dtype, name="layer")


def test_buffers_can_be_reused_and_empty_input_is_fine(api):
    maps, h, w, n = 10, 30, 30, 4
    bufs = api.alloc_sparse(maps, h, w, n, torch.float32, "cuda")
    for seed in (1, 2):
        x = W.salient_feature_maps(maps, h, w, seed=seed, zero_level=0.2 * seed)
        info, v, idx, totals = oracle.sparse_encode(x, maps, h, w, n, 0.4)
        api.fh_sparse_encode(torch.from_numpy(x).cuda(), maps, h, w, n, 0.4, buffers=bufs)
        torch.cuda.synchronize()
        assert np.array_equal(bufs.totals.cpu().numpy().view(np.uint64), totals)
        assert np.array_equal(bufs.values.cpu().numpy()[:int(totals[0])].view(np.uint32), v.view(np.uint32))
    b = api.fh_sparse_encode(torch.empty(0, device="cuda"), 0, 5, 5, 4, 0.5)
    torch.cuda.synchronize()
    assert b.totals.cpu().tolist() == [0, 0, 0, 0]


def test_decoder_stays_inside_truncated_or_foreign_streams(api):
    """The decoder bounds every read by the sizes it is given: a block whose slice would leave a
    stream is zero-filled, entries pointing outside a block are dropped.  The kernels run to
    completion; only the restored values are (defined) garbage."""
    maps, h, w, n = 8, 24, 24, 4
    x = W.salient_feature_maps(maps, h, w, seed=3)
    b = api.fh_sparse_encode(torch.from_numpy(x).cuda(), maps, h, w, n, 0.5)
    torch.cuda.synchronize()
    nv, ni = (int(v) for v in b.totals.cpu().tolist()[:2])
    # truncated streams: the blocks that still fit come back exactly, the others as zeros
    out = api.fh_sparse_decode(b.info, b.values[:nv // 2], b.indices[:ni // 2], maps, h, w, n)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    same = got == x
    assert same[: x.size // 4].all() and ((got == 0) | same).all() and not same.all()
    # foreign info bytes (random): must simply finish
    junk = torch.randint(0, 256, (b.info.numel(),), dtype=torch.uint8, device="cuda")
    out = api.fh_sparse_decode(junk, b.values[:nv], b.indices[:ni], maps, h, w, n)
    torch.cuda.synchronize()
    assert out.numel() == x.size
    # foreign index bytes
    junk_idx = torch.randint(0, 256, (ni,), dtype=torch.uint8, device="cuda")
    out = api.fh_sparse_decode(b.info, b.values[:nv], junk_idx, maps, h, w, n)
    torch.cuda.synchronize()
    assert out.numel() == x.size


def test_salient_channels_end_to_end(api):
    """mixed compress -> sparse storage of the raw store -> back -> mixed restore, against the
    oracle's mixed round trip (the sparse stage is lossless, so it must not show)."""
    outer, C, hh, ww = 8, 48, 28, 28
    inner = hh * ww
    x, planted = W.outlier_channel_tensor(outer, C, inner, seed=21, dist="relu", salient_fraction=0.08)
    mask = np.zeros(C, np.uint8)
    mask[planted] = 1
    cap = len(planted)
    dx = torch.from_numpy(x).cuda()
    d_slots = api.fh_channel_slots(torch.from_numpy(mask).cuda(), cap)
    gp, gm, graw = api.fh_compress_mixed(dx, outer, C, inner, d_slots, cap, 128, 4, "stochastic", 4, 2)
    b = api.fh_sparse_encode(graw, outer * cap, hh, ww, 4, 0.6)
    torch.cuda.synchronize()
    nv, ni, ns, nd = (int(v) for v in b.totals.cpu().tolist())
    assert ns > 0 and nd > 0
    raw_back = api.fh_sparse_decode(b.info, b.values[:nv], b.indices[:ni], outer * cap, hh, ww, 4)
    got = api.fh_decompress_mixed(gp, gm, raw_back, outer, C, inner, d_slots, cap, 128, 4)
    torch.cuda.synchronize()
    slots, _ = oracle.channel_slots(mask, cap)
    p, m, raw = oracle.compress_mixed(x, outer, C, inner, slots, cap, 128, 4, "stochastic", 4, 2)
    want = oracle.decompress_mixed(p, m, raw, outer, C, inner, slots, cap, 128, 4)
    assert np.array_equal(got.cpu().numpy().view(np.uint32), want.view(np.uint32))
    stored = nv * 4 + ni + b.info.numel()
    assert stored < raw.nbytes                               # post-ReLU salient channels do shrink


def test_argument_errors_reach_the_caller(api):
    x = torch.zeros(2 * 8 * 8, device="cuda")
    with pytest.raises(api.FedHybridError) as e:
        api.fh_sparse_encode(x, 2, 8, 8, 3, 0.5)
    assert e.value.status == 12
    bufs = api.alloc_sparse(2, 8, 8, 4, torch.float32, "cuda")
    bufs.indices = bufs.indices[:10]
    with pytest.raises(api.FedHybridError) as e:
        api.fh_sparse_encode(x, 2, 8, 8, 4, 0.5, buffers=bufs)
    assert e.value.status == 7


# ---- dense blocks within an error bound (Lorenzo prediction, outliers intact) ------------------

@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("n", [2, 4, 8])
@pytest.mark.parametrize("eps", [1e-4, 0.02, 0.5])
def test_predictive_dense_blocks(api, dtype, n, eps):
    for (maps, h, w) in ((6, 27, 22), (3, 56, 56), (40, 7, 7)):
        x = W.salient_feature_maps(maps, h, w, seed=n + maps, zero_level=0.1, dtype=dtype)
        _check(api, x, maps, h, w, n, 0.4, dtype=dtype, name="predictive", eps=eps)
        _check(api, x, maps, h, w, n, -1.0, dtype=dtype, name="predictive, all dense", eps=eps)


def test_predictive_blocks_with_values_off_the_lattice(api):
    rng = np.random.default_rng(4)
    maps, h, w = 4, 24, 24
    x = W.salient_feature_maps(maps, h, w, seed=8, zero_level=-0.5)
    x[rng.integers(0, x.size, 30)] = np.inf
    x[rng.integers(0, x.size, 30)] = -3.0e9
    x[rng.integers(0, x.size, 30)] = np.nan
    x[rng.integers(0, x.size, 30)] = f32(2.0 ** 22 * 0.02)                  # exactly at the end of the lattice
    for n in (2, 4, 8):
        info, v, idx, totals = oracle.sparse_encode(x, maps, h, w, n, 0.3, eps=0.01)
        b = api.fh_sparse_encode(torch.from_numpy(x).cuda(), maps, h, w, n, 0.3, eps=0.01)
        torch.cuda.synchronize()
        assert np.array_equal(b.totals.cpu().numpy().view(np.uint64), totals)
        assert np.array_equal(b.info.cpu().numpy()[:info.size], info)
        assert np.array_equal(b.values.cpu().numpy()[:v.size].view(np.uint32), v.view(np.uint32))
        assert np.array_equal(b.indices.cpu().numpy()[:idx.size], idx)
        out = api.fh_sparse_decode(b.info, b.values[:v.size], b.indices[:idx.size], maps, h, w, n, eps=0.01)
        torch.cuda.synchronize()
        want = oracle.sparse_decode(info, v, idx, maps, h, w, n, eps=0.01)
        assert np.array_equal(out.cpu().numpy().view(np.uint32), want.view(np.uint32))


def test_predictive_full_size_layer_meets_the_bound(api):
    maps, h, w, n, eps = 64 * 4, 112, 112, 8, 0.05
    x = W.salient_feature_maps(maps, h, w, seed=6, zero_level=0.0)
    t = _check(api, x, maps, h, w, n, 0.4, name="predictive layer", eps=eps)
    b = api.fh_sparse_encode(torch.from_numpy(x).cuda(), maps, h, w, n, 0.4, eps=eps)
    torch.cuda.synchronize()
    nv, ni = int(t[0]), int(t[1])
    out = api.fh_sparse_decode(b.info, b.values[:nv], b.indices[:ni], maps, h, w, n, eps=eps).cpu().numpy()
    assert np.abs(out.astype(np.float64) - x).max() <= eps * (1 + 1e-6) + np.abs(x).max() * 2.0 ** -22
    assert nv * 4 + ni + b.info.numel() < 0.45 * x.nbytes                 # and it does pay


def test_predictive_decoder_stays_inside_truncated_or_foreign_streams(api):
    maps, h, w, n, eps = 8, 24, 24, 4, 0.02
    x = W.salient_feature_maps(maps, h, w, seed=3, zero_level=0.0)
    b = api.fh_sparse_encode(torch.from_numpy(x).cuda(), maps, h, w, n, 0.3, eps=eps)
    torch.cuda.synchronize()
    nv, ni = (int(v) for v in b.totals.cpu().tolist()[:2])
    for info, vals, idx in ((b.info, b.values[:nv // 2], b.indices[:ni // 2]),
                            (torch.randint(0, 256, (b.info.numel(),), dtype=torch.uint8, device="cuda"),
                             b.values[:nv], b.indices[:ni]),
                            (b.info, b.values[:nv], torch.randint(0, 256, (ni,), dtype=torch.uint8, device="cuda"))):
        out = api.fh_sparse_decode(info, vals, idx, maps, h, w, n, eps=eps)
        torch.cuda.synchronize()
        assert out.numel() == x.size


def test_the_whole_channel_wise_chain_can_be_captured_in_a_graph_and_replayed(api):
    """classify -> slots -> mixed compress -> sparse storage of the raw store -> back -> mixed
    restore, captured once and replayed on new inputs: no call allocates, clears memory with a
    memset or synchronises, so every replay must reproduce what the oracle computes."""
    outer, C, hh, ww, cap, n, tau, eps = 6, 40, 28, 28, 3, 4, 0.5, 0.02
    inner = hh * ww
    G, B = 128, 4
    dev = "cuda"
    xd = torch.empty(outer * C * inner, device=dev)
    ws = torch.empty(api.classify_workspace_bytes(xd.numel()), dtype=torch.uint8, device=dev)
    stats = torch.empty(4, dtype=torch.float64, device=dev)
    counts = torch.empty(C, dtype=torch.int32, device=dev)
    mask = torch.empty(C, dtype=torch.uint8, device=dev)
    slots = torch.empty(C, dtype=torch.int16, device=dev)
    packed, meta = api.alloc_compressed(xd.numel(), G, B, dev)
    raw = torch.zeros(outer * cap * inner, device=dev)
    bufs = api.alloc_sparse(outer * cap, hh, ww, n, torch.float32, dev)
    raw_back = torch.empty_like(raw)
    out = torch.empty_like(xd)
    min_out = outer * inner // 100

    def chain(stream):
        api.fh_classify_channels(xd, outer, C, inner, 3.0, min_out, workspace=ws, stats=stats, counts=counts,
                                 mask=mask, stream=stream)
        api.fh_channel_slots(mask, cap, slots=slots, stream=stream)
        api.fh_compress_mixed(xd, outer, C, inner, slots, cap, G, B, "stochastic", 5, 1, packed=packed, meta=meta,
                              raw=raw, stream=stream)
        api.fh_sparse_encode(raw, outer * cap, hh, ww, n, tau, buffers=bufs, stream=stream, eps=eps)
        # the valid prefixes are only known on the device: the decoder is given the whole buffers,
        # it reads no further than the info bytes say
        api.fh_sparse_decode(bufs.info, bufs.values, bufs.indices, outer * cap, hh, ww, n, out=raw_back,
                             workspace=bufs.workspace, stream=stream, eps=eps)
        api.fh_decompress_mixed(packed, meta, raw_back, outer, C, inner, slots, cap, G, B, out=out, stream=stream)

    def expected(x):
        _, _, omask = oracle.classify_channels(x, outer, C, inner, 3.0, min_out)
        oslots, used = oracle.channel_slots(omask, cap)
        p, m, oraw = oracle.compress_mixed(x, outer, C, inner, oslots, cap, G, B, "stochastic", 5, 1)
        # rows of unused slots are not written by the compressor: they keep what the buffer held
        # (zeros here), and go through the sparse stage like the others
        info, v, idx, _ = oracle.sparse_encode(oraw, outer * cap, hh, ww, n, tau, eps=eps)
        back = oracle.sparse_decode(info, v, idx, outer * cap, hh, ww, n, eps=eps)
        return oslots, p, m, oracle.decompress_mixed(p, m, back, outer, C, inner, oslots, cap, G, B)

    x0, _ = W.outlier_channel_tensor(outer, C, inner, seed=1, dist="relu", salient_fraction=0.05)
    xd.copy_(torch.from_numpy(x0))
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        chain(side)                                          # warm-up outside capture
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        chain(torch.cuda.current_stream())
    for rep in range(3):
        x, _ = W.outlier_channel_tensor(outer, C, inner, seed=10 + rep, dist="relu", salient_fraction=0.05 + 0.02 * rep)
        xd.copy_(torch.from_numpy(x))
        out.fill_(float("nan"))
        raw.zero_()
        packed.fill_(0x5A)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        oslots, p, m, want = expected(x)
        assert np.array_equal(slots.cpu().numpy(), oslots), f"replay {rep}: slots"
        assert np.array_equal(packed.cpu().numpy(), p), f"replay {rep}: codes"
        assert np.array_equal(meta.cpu().numpy().view(np.uint32), m.view(np.uint32)), f"replay {rep}: meta"
        assert np.array_equal(out.cpu().numpy().view(np.uint32), want.view(np.uint32)), f"replay {rep}: restored"


# ---- the batched calls ---------------------------------------------------------------------------

def test_batched_calls_match_the_oracle_for_every_set(api):
    """More sets than one launch holds, both dtypes and all windows (several runs), an empty set,
    a set large enough for the scan kernel, with and without an error bound."""
    specs = [(3, 28, 28, 4, "f32", 0.0), (5, 14, 14, 4, "f32", 0.02), (0, 9, 9, 4, "f32", 0.0), (2, 56, 56, 8, "f32", 0.05),
             (4, 13, 29, 2, "bf16", 0.0), (9000, 16, 16, 2, "f32", 0.0), (7, 7, 7, 8, "bf16", 0.1)]
    specs += [(2 + i, 10 + i, 12 + 2 * i, 4, "f32", 0.01 * (i % 3)) for i in range(14)]
    entries, host = [], []
    for i, (maps, h, w, n, dtype, eps) in enumerate(specs):
        x = W.salient_feature_maps(max(maps, 1), h, w, seed=50 + i, zero_level=0.2, dtype=dtype)[: maps * h * w]
        host.append(x)
        tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
        xd = _device(x, dtype) if x.size else torch.empty(0, dtype=tdt, device="cuda")
        entries.append(api.SparseEntry(maps, h, w, n, 0.45, eps, x=xd, out=torch.empty(x.size, dtype=tdt, device="cuda")))
    assert len(entries) > api.sparse_batch_capacity()
    batch = api.SparseBatch(entries)
    print(f"[sparse] batch of {len(entries)} map sets", flush=True)
    api.fh_sparse_encode_batch(batch)
    api.fh_sparse_decode_batch(batch)                         # whole buffers as streams: bounded by the info bytes
    torch.cuda.synchronize()
    for i, ((maps, h, w, n, dtype, eps), x, e) in enumerate(zip(specs, host, entries)):
        info, v, idx, totals = oracle.sparse_encode(x, maps, h, w, n, 0.45, dtype=dtype, eps=eps)
        assert np.array_equal(e.buffers.totals.cpu().numpy().view(np.uint64), totals), f"set {i}: totals"
        assert np.array_equal(e.buffers.info.cpu().numpy()[:info.size], info), f"set {i}: info"
        assert np.array_equal(_bits(_host(e.buffers.values, dtype)[:v.size]), _bits(v)), f"set {i}: values"
        assert np.array_equal(e.buffers.indices.cpu().numpy()[:idx.size], idx), f"set {i}: indices"
        want = oracle.sparse_decode(info, v, idx, maps, h, w, n, dtype=dtype, eps=eps)
        assert np.array_equal(_bits(_host(e.out, dtype)), _bits(want)), f"set {i}: restored"
