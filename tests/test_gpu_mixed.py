"""Parity of the HIP mixed path with the CPU oracle (Section 4.4.1, Channel-wise Mix
Compression: salient channels are routed around the quantiser; this library keeps them
verbatim in a raw store).  Bar: slots, code bytes, meta, the raw rows of kept channels and
the restored tensor all bit-exact; raw rows of unused slots untouched."""
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


def _tdtype(dtype):
    return torch.bfloat16 if dtype == "bf16" else torch.float32


def _bits(a):
    return a.view(np.uint32) if a.dtype == np.float32 else a


def _mask(C, fraction, seed):
    rng = np.random.default_rng(seed)
    if fraction >= 1.0:
        return np.ones(C, np.uint8)
    m = (rng.random(C) < fraction).astype(np.uint8)
    return m


def _roundtrip(api, x, outer, C, inner, mask, cap, G, B, rounding, dtype="f32", out_dtypes=("f32", "bf16"),
               seed=99, tid=7, name=""):
    print(f"[mixed] {name} {dtype} [{outer}][{C}][{inner}] kept<={cap} of {int(mask.sum())} G{G} B{B} {rounding}",
          flush=True)
    n = outer * C * inner
    slots, used = oracle.channel_slots(mask, cap)
    fill = 0x5A5A if dtype == "bf16" else f32(-777.5)
    p, m, raw = oracle.compress_mixed(x, outer, C, inner, slots, cap, G, B, rounding, seed, tid, dtype=dtype,
                                      raw_fill=fill)

    d_mask = torch.from_numpy(mask).cuda()
    d_slots = api.fh_channel_slots(d_mask, cap)
    d_raw = torch.from_numpy(np.full(outer * cap * inner, fill, dtype=x.dtype).view(np.int16)
                             if dtype == "bf16" else np.full(outer * cap * inner, fill, dtype=x.dtype)).cuda()
    if dtype == "bf16":
        d_raw = d_raw.view(torch.bfloat16)
    gp, gm, graw = api.fh_compress_mixed(_device(x, dtype), outer, C, inner, d_slots, cap, G, B, rounding, seed, tid,
                                         raw=d_raw)
    torch.cuda.synchronize()
    assert np.array_equal(d_slots.cpu().numpy(), slots), f"{name}: slots differ"
    gp_h, gm_h, graw_h = gp.cpu().numpy(), gm.cpu().numpy(), _host(graw, dtype)
    bad = np.flatnonzero(gm_h.view(np.uint32) != m.view(np.uint32))
    assert bad.size == 0, f"{name}: meta differs at {bad[:8]} ({gm_h.ravel()[bad[:4]]} vs {m.ravel()[bad[:4]]})"
    bad = np.flatnonzero(gp_h != p)
    assert bad.size == 0, f"{name}: {bad.size} code bytes differ, first at {bad[:8]}"
    bad = np.flatnonzero(_bits(graw_h) != _bits(raw))
    assert bad.size == 0, f"{name}: raw store differs at {bad[:8]}"

    for od in out_dtypes:
        want = oracle.decompress_mixed(p, m, raw, outer, C, inner, slots, cap, G, B, raw_dtype=dtype, out_dtype=od)
        got = api.fh_decompress_mixed(gp, gm, graw, outer, C, inner, d_slots, cap, G, B, out_dtype=_tdtype(od))
        torch.cuda.synchronize()
        got_h = _host(got, od)
        bad = np.flatnonzero(_bits(got_h) != _bits(want))
        assert bad.size == 0, f"{name}: restored {od} differs at {bad[:8]}"
    return slots, used


# (outer, channels, inner): one channel per element (even, odd and tiny channel counts), feature
# maps whose rows are multiples of a lane's run, odd rows, rows shorter than a lane's run,
# single channel, sizes that end inside a tile
SHAPES = [(64, 768, 1), (33, 96, 1), (50, 100, 1), (7, 12, 1), (8, 32, 56 * 56), (4, 24, 49), (3, 16, 196),
          (2, 10, 7), (6, 5, 3), (1, 1, 5000), (9, 3, 1), (1, 4, 8192), (2, 3, 4097), (5, 16384, 1), (1, 2, 1)]


@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_shapes_and_layouts(api, shape, dtype):
    outer, C, inner = shape
    x, _ = W.outlier_channel_tensor(outer, C, inner, seed=outer + inner, salient_fraction=0.1, dtype=dtype)
    mask = _mask(C, 0.15, C + inner)
    mask[0] = 1
    cap = max(1, int(mask.sum()))
    _roundtrip(api, x, outer, C, inner, mask, cap, 64, 4, "stochastic", dtype=dtype, name="shape")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_one_channel_per_element_many_channels(api, dtype):
    """inner = 1 with channel counts beyond what a workgroup requests up front (4096), an odd count, the largest
    raw store whose rows are listed (2048) and one row more (which takes the per-element path)."""
    for outer, C, cap, share in ((5, 16384, 64, 0.01), (3, 5001, 2048, 0.5), (4, 4100, 2049, 0.6), (40, 8190, 1, 0.02)):
        x, _ = W.outlier_channel_tensor(outer, C, 1, seed=C, salient_fraction=0.1, dtype=dtype)
        mask = _mask(C, share, C)
        mask[C - 1] = 1
        _roundtrip(api, x, outer, C, 1, mask, cap, 64, 4, "nearest", dtype=dtype, name="many-channels")


@pytest.mark.parametrize("G", [64, 128, 256])
@pytest.mark.parametrize("B", [2, 4, 8])
@pytest.mark.parametrize("rounding", ["nearest", "stochastic"])
def test_quantiser_parameters(api, G, B, rounding):
    for dtype, (outer, C, inner) in (("f32", (6, 40, 14 * 14)), ("bf16", (40, 264, 1))):
        x, _ = W.outlier_channel_tensor(outer, C, inner, seed=G + B, dtype=dtype)
        mask = _mask(C, 0.1, G * B)
        _roundtrip(api, x, outer, C, inner, mask, max(1, int(mask.sum())), G, B, rounding, dtype=dtype, name="params")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_store_smaller_or_larger_than_the_salient_set(api, dtype):
    outer, C, inner = 12, 48, 100
    x, _ = W.outlier_channel_tensor(outer, C, inner, seed=4, dtype=dtype)
    mask = _mask(C, 0.3, 11)
    k = int(mask.sum())
    assert k >= 4
    for cap in (0, 1, k - 1, k, min(C, k + 5), C):
        slots, used = _roundtrip(api, x, outer, C, inner, mask, cap, 128, 4, "nearest", dtype=dtype, name="cap")
        assert used == min(k, cap)


def test_no_salient_channel_is_the_plain_quantiser(api):
    outer, C, inner = 5, 24, 300
    x, _ = W.outlier_channel_tensor(outer, C, inner, seed=1)
    mask = np.zeros(C, np.uint8)
    _roundtrip(api, x, outer, C, inner, mask, 0, 64, 8, "stochastic", name="none")
    _roundtrip(api, x, outer, C, inner, mask, 3, 64, 8, "stochastic", name="none, spare rows")
    p0, m0 = oracle.compress(x, 64, 8, "stochastic", 99, 7)
    slots = torch.full((C,), -1, dtype=torch.int16, device="cuda")
    gp, gm, _ = api.fh_compress_mixed(torch.from_numpy(x).cuda(), outer, C, inner, slots, 0, 64, 8, "stochastic", 99, 7)
    torch.cuda.synchronize()
    assert np.array_equal(gp.cpu().numpy(), p0) and np.array_equal(gm.cpu().numpy().view(np.uint32), m0.view(np.uint32))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_every_channel_salient(api, dtype):
    outer, C, inner = 3, 16, 130
    x, _ = W.outlier_channel_tensor(outer, C, inner, seed=2, dtype=dtype)
    _roundtrip(api, x, outer, C, inner, np.ones(C, np.uint8), C, 64, 4, "stochastic", dtype=dtype, name="all")


def test_slots_kernel(api):
    rng = np.random.default_rng(0)
    for C in (1, 2, 15, 16, 17, 100, 1000, 1024, 4097, 16383, 16384):
        for frac in (0.0, 0.03, 0.5, 1.0):
            mask = (rng.random(C) < frac).astype(np.uint8) * rng.integers(1, 255, C).astype(np.uint8)
            for cap in sorted({0, 1, C // 2, C}):
                want, _ = oracle.channel_slots(mask, cap)
                got = api.fh_channel_slots(torch.from_numpy(mask).cuda(), cap)
                torch.cuda.synchronize()
                assert np.array_equal(got.cpu().numpy(), want), f"C={C} frac={frac} cap={cap}"


def test_classify_then_route_end_to_end(api):
    """The whole chain on the device: classification mask -> slots -> mixed round trip; planted
    channels come back exactly and the others with the error of their own range."""
    outer, C, inner = 16, 96, 28 * 28
    x, planted = W.outlier_channel_tensor(outer, C, inner, seed=12, dist="relu", salient_fraction=0.05)
    dx = torch.from_numpy(x).cuda()
    _, _, d_mask = api.fh_classify_channels(dx, outer, C, inner, 3.0, outer * inner // 100)
    cap = 8
    d_slots = api.fh_channel_slots(d_mask, cap)
    gp, gm, graw = api.fh_compress_mixed(dx, outer, C, inner, d_slots, cap, 128, 4, "nearest")
    got = api.fh_decompress_mixed(gp, gm, graw, outer, C, inner, d_slots, cap, 128, 4)
    torch.cuda.synchronize()
    mask = d_mask.cpu().numpy()
    assert set(np.flatnonzero(mask)) == set(int(c) for c in planted)
    _, _, omask = oracle.classify_channels(x, outer, C, inner, 3.0, outer * inner // 100)
    slots, _ = oracle.channel_slots(omask, cap)
    p, m, raw = oracle.compress_mixed(x, outer, C, inner, slots, cap, 128, 4)
    want = oracle.decompress_mixed(p, m, raw, outer, C, inner, slots, cap, 128, 4)
    assert np.array_equal(got.cpu().numpy().view(np.uint32), want.view(np.uint32))
    y3, x3 = want.reshape(outer, C, inner), x.reshape(outer, C, inner)
    assert np.array_equal(y3[:, planted, :], x3[:, planted, :])


@pytest.mark.parametrize("case", ["mobilenetv2", "transformer"])
def test_full_size_layers(api, case):
    if case == "mobilenetv2":                             # the largest expanded feature map at batch 64
        outer, C, inner, dtype, G, B, rounding = 64, 96, 112 * 112, "f32", 128, 4, "nearest"
    else:                                                 # one transformer activation: 16 x 512 tokens, hidden 3072
        outer, C, inner, dtype, G, B, rounding = 8192, 3072, 1, "bf16", 64, 2, "stochastic"
    x, planted = W.outlier_channel_tensor(outer, C, inner, seed=5, dtype=dtype,
                                          magnitude=81.0 if dtype == "f32" else 347.0)
    mask = np.zeros(C, np.uint8)
    mask[planted] = 1
    _roundtrip(api, x, outer, C, inner, mask, len(planted), G, B, rounding, dtype=dtype,
               out_dtypes=("f32",) if dtype == "f32" else ("bf16",), name=case)


def test_argument_errors_reach_the_caller(api):
    x = torch.zeros(2 * 8 * 64, device="cuda")
    slots = torch.full((8,), -1, dtype=torch.int16, device="cuda")
    with pytest.raises(api.FedHybridError) as e:
        api.fh_compress_mixed(x, 2, 8, 64, slots, 9, 64, 4)            # more raw rows than channels
    assert e.value.status == 11
    with pytest.raises(api.FedHybridError) as e:
        api.fh_compress_mixed(x, 2, 8, 64, slots, 2, 64, 4, raw=torch.empty(10, device="cuda"))
    assert e.value.status == 7
    with pytest.raises(api.FedHybridError) as e:
        api.fh_compress_mixed(x, 2, 8, 64, slots, 0, 64, 3)
    assert e.value.status == 4
    with pytest.raises(api.FedHybridError) as e:
        api.fh_channel_slots(torch.zeros(8, dtype=torch.uint8, device="cuda"), 9)
    assert e.value.status == 11
    # an empty tensor is fine and launches nothing
    p, m, r = api.fh_compress_mixed(torch.empty(0, device="cuda"), 0, 8, 64, slots, 2, 64, 4)
    assert p.numel() == 0 and m.numel() == 0 and r.numel() == 0


# ---- the batched calls ---------------------------------------------------------------------------

def test_batched_calls_match_the_oracle_for_every_tensor(api):
    """More tensors than one launch holds, both dtypes and several group sizes (several runs),
    an empty tensor, capacities below and above the salient count."""
    specs = [(8, 32, 196, "f32", 128, 4, "nearest"), (64, 768, 1, "bf16", 64, 2, "stochastic"), (0, 12, 9, "f32", 128, 4, "nearest"),
             (3, 16, 4097, "f32", 256, 8, "stochastic"), (5, 100, 1, "bf16", 64, 4, "nearest"), (2, 10, 7, "f32", 64, 8, "nearest")]
    specs += [(2 + i % 3, 8 + i, 50 + 13 * i, "f32", 128, 4, "stochastic") for i in range(16)]
    entries, host = [], []
    for i, (outer, C, inner, dtype, G, B, rounding) in enumerate(specs):
        x, _ = W.outlier_channel_tensor(max(outer, 1), C, inner, seed=70 + i, salient_fraction=0.1, dtype=dtype)
        x = x[: outer * C * inner]
        mask = _mask(C, 0.2, i)
        mask[0] = 1
        cap = max(1, int(mask.sum()) - (i % 2))              # every other tensor: one salient channel too many
        if i in (3, 9):
            cap = 0                                           # nothing kept: served by the plain kernels
        slots, used = oracle.channel_slots(mask, cap)
        host.append((x, slots, cap))
        tdt = _tdtype(dtype)
        xd = _device(x, dtype) if x.size else torch.empty(0, dtype=tdt, device="cuda")
        entries.append(api.MixedEntry(outer, C, inner, torch.from_numpy(slots).cuda(), cap, G, B, rounding, 3, 100 + i,
                                      x=xd, out=torch.empty(x.size, dtype=torch.float32, device="cuda")))
    assert len(entries) > api.mixed_batch_capacity()
    batch = api.MixedBatch(entries)
    print(f"[mixed] batch of {len(entries)} tensors", flush=True)
    api.fh_compress_mixed_batch(batch)
    api.fh_decompress_mixed_batch(batch)
    torch.cuda.synchronize()
    for i, ((outer, C, inner, dtype, G, B, rounding), (x, slots, cap), e) in enumerate(zip(specs, host, entries)):
        p, m, raw = oracle.compress_mixed(x, outer, C, inner, slots, cap, G, B, rounding, 3, 100 + i, dtype=dtype)
        used = int((slots >= 0).sum())
        assert np.array_equal(e.packed.cpu().numpy(), p), f"tensor {i}: codes"
        assert np.array_equal(e.meta.cpu().numpy().view(np.uint32), m.view(np.uint32)), f"tensor {i}: meta"
        got_raw = _host(e.raw, dtype).reshape(outer, cap, inner)[:, :used]
        assert np.array_equal(_bits(got_raw), _bits(raw.reshape(outer, cap, inner)[:, :used])), f"tensor {i}: raw"
        # restore with the oracle's raw store where unused rows are zero: kept rows are what matter
        want = oracle.decompress_mixed(p, m, raw, outer, C, inner, slots, cap, G, B, raw_dtype=dtype, out_dtype="f32")
        assert np.array_equal(e.out.cpu().numpy().view(np.uint32), want.view(np.uint32)), f"tensor {i}: restored"


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_rows_in_use_of_zero_takes_the_plain_code_path(api, dtype):
    """The slot numbering also reports how many raw-store rows are in use; a tensor for which that is
    zero runs the plain quantiser's code inside the mixed launches -- same bytes as the oracle's
    mixed form with nothing kept (= the plain quantiser), raw store untouched -- and a tensor that
    keeps something is unaffected by passing the count."""
    outer, C, inner = 7, 64, 600
    x, planted = W.outlier_channel_tensor(outer, C, inner, seed=4, dtype=dtype)
    xd = _device(x, dtype)
    for mask in (np.zeros(C, np.uint8), np.isin(np.arange(C), planted).astype(np.uint8)):
        print(f"[mixed] rows_in_use {dtype} salient={int(mask.sum())}", flush=True)
        used = torch.full((1,), -5, dtype=torch.int64, device="cuda")
        slots = api.fh_channel_slots(torch.from_numpy(mask).cuda(), 4, used=used)
        raw = torch.full((outer * 4 * inner,), 7.0, device="cuda").to(xd.dtype)
        gp, gm, graw = api.fh_compress_mixed(xd, outer, C, inner, slots, 4, 128, 4, "stochastic", 5, 2, raw=raw,
                                             rows_in_use=used)
        outs = [api.fh_decompress_mixed(gp, gm, graw, outer, C, inner, slots, 4, 128, 4, out_dtype=_tdtype(od),
                                        rows_in_use=used) for od in ("f32", "bf16")]
        torch.cuda.synchronize()
        want_slots, want_used = oracle.channel_slots(mask, 4)
        assert int(used.item()) == want_used and np.array_equal(slots.cpu().numpy(), want_slots)
        p, m, r = oracle.compress_mixed(x, outer, C, inner, want_slots, 4, 128, 4, "stochastic", 5, 2, dtype=dtype,
                                        raw_fill=0x40E0 if dtype == "bf16" else 7.0)      # 7.0 as bf16 bits
        assert np.array_equal(gp.cpu().numpy(), p) and np.array_equal(gm.cpu().numpy().view(np.uint32), m.view(np.uint32))
        assert np.array_equal(_bits(_host(graw, dtype)), _bits(r)), "raw store differs"
        for od, got in zip(("f32", "bf16"), outs):
            want = oracle.decompress_mixed(p, m, r, outer, C, inner, want_slots, 4, 128, 4, raw_dtype=dtype, out_dtype=od)
            assert np.array_equal(_bits(_host(got, od)), _bits(want)), f"restored {od} differs"
