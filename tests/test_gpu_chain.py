"""Parity of fh_mix_compress / fh_mix_decompress -- the whole channel-wise mix compressor of
Section 4.4.1 enqueued as one call each way -- with the composition of the oracle's stages
(tests/oracle_chain.py).  Bar: every stored part bit-exact (statistics, counts, mask, slots,
codes, meta, info bytes, the value / index / Huffman streams up to the sizes the header
reports, the header itself) and the restored tensor bit-exact."""
from __future__ import annotations

import numpy as np
import pytest

import oracle_chain as OC
from paper_2510_11400_amd import workloads as W

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def api():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a visible MI355X")
    from paper_2510_11400_amd import api as _api
    return _api


def _device(x, dtype):
    t = torch.from_numpy(x.view(np.int16) if dtype == "bf16" else x).cuda()
    return t.view(torch.bfloat16) if dtype == "bf16" else t


def _maps(outer, raw_channels, inner, hw):
    if hw is None:                                  # [tokens][hidden]: one map of tokens x kept channels
        return (1, outer, raw_channels) if raw_channels else (0, 0, 0)
    return outer * raw_channels, hw[0], hw[1]


def _entry(api, xd, case, out_dtype):
    (outer, C, inner, hw, raw_channels, G, B, rounding, window, tau, eps, entropy, dtype, min_out) = case
    maps, h, w = _maps(outer, raw_channels, inner, hw)
    n = outer * C * inner
    out = torch.empty(n, dtype=torch.bfloat16 if out_dtype == "bf16" else torch.float32, device="cuda")
    return api.MixEntry(outer, C, inner, raw_channels, G, B, rounding, seed=11, tensor_id=3, k_sigma=3.0,
                        min_outliers=min_out, maps=maps, h=h, w=w, window=window, tau=tau, eps=eps,
                        entropy=entropy, x=xd, out=out)


def _compare(api, batch, i, x, case, out_dtype):
    (outer, C, inner, hw, raw_channels, G, B, rounding, window, tau, eps, entropy, dtype, min_out) = case
    maps, h, w = _maps(outer, raw_channels, inner, hw)
    st = OC.mix_compress(x, outer, C, inner, raw_channels, G, B, rounding, 11, 3, 3.0, min_out, maps, h, w, window,
                         tau, eps, entropy, dtype=dtype)
    want = OC.mix_decompress(st, outer, C, inner, raw_channels, G, B, maps, h, w, window, eps, entropy, dtype=dtype,
                             out_dtype=out_dtype)
    part = lambda name: batch.part(i, name).cpu().numpy()
    assert np.array_equal(part("stats").view(np.uint64), st.stats.view(np.uint64)), "statistics differ"
    assert np.array_equal(part("counts").view(np.uint32), st.counts), "outlier counts differ"
    assert np.array_equal(part("mask"), st.mask), "mask differs"
    assert np.array_equal(part("slots").view(np.int16), st.slots), "slots differ"
    assert np.array_equal(part("packed"), st.packed), "codes differ"
    assert np.array_equal(part("meta").view(np.uint32), st.meta.reshape(-1).view(np.uint32)), "meta differs"
    header = batch.header(i).cpu().numpy()
    esize = 4 if dtype == "f32" else 2
    if raw_channels and outer:
        assert [int(v) for v in header[:4]] == [int(v) for v in st.totals], f"sparse totals {header[:4]} vs {st.totals}"
        assert np.array_equal(part("info"), st.info), "info bytes differ"
        assert np.array_equal(part("values")[: st.values.size * esize], st.values.view(np.uint8)), "value stream differs"
        if entropy:
            assert (int(header[4]), int(header[5])) == (st.huffman.size, st.payload_bits), "Huffman totals differ"
            assert np.array_equal(part("huffman")[: st.huffman.size], st.huffman), "Huffman stream differs"
        else:
            assert np.array_equal(part("indices")[: st.indices.size], st.indices), "index stream differs"
    assert int(header[6]) == st.stored_bytes, f"stored bytes {header[6]} vs {st.stored_bytes}"
    assert int(header[7]) == st.used, "raw-store rows in use differ"
    got = batch.entries[i].out.cpu()
    got = got.view(torch.int16).numpy().view(np.uint16) if out_dtype == "bf16" else got.numpy().view(np.uint32)
    ref = want if out_dtype == "bf16" else want.view(np.uint32)
    bad = np.flatnonzero(got != ref)
    assert bad.size == 0, f"restored tensor differs at {bad[:8]}"
    return st


#        outer  C   inner  (h, w)    raw G    B  rounding      win tau  eps   ent dtype  min_out
CASES = [
    (8,   32,  196,  (14, 14),  4, 128, 4, "nearest",     4, 0.5, 0.02, 1, "f32", 15),
    (8,   32,  196,  (14, 14),  4, 128, 4, "stochastic",  4, 0.5, 0.0,  1, "f32", 15),
    (8,   32,  196,  (14, 14),  4, 128, 4, "nearest",     4, 0.5, 0.02, 0, "f32", 15),
    (6,   48,  3136, (56, 56),  3, 256, 2, "stochastic",  8, 0.6, 0.05, 1, "f32", 180),
    (6,   48,  3136, (56, 56),  3, 64,  8, "nearest",     2, 0.3, 0.01, 1, "bf16", 180),
    (5,   40,  49,   (7, 7),    2, 64,  4, "nearest",     4, 0.5, 0.02, 1, "f32", 2),
    (300, 768, 1,    None,      32, 64, 2, "stochastic",  4, 0.5, 0.02, 1, "bf16", 3),
    (300, 768, 1,    None,      32, 64, 2, "stochastic",  4, 0.5, 0.0,  0, "f32", 3),
    (8,   32,  196,  (14, 14),  0, 128, 4, "nearest",     4, 0.5, 0.02, 1, "f32", 15),     # nothing kept: plain quantiser
    (4,   16,  1024, (32, 32),  16, 256, 4, "nearest",    4, 1.0, 0.02, 1, "f32", 1),      # every channel kept
    (0,   16,  64,   (8, 8),    2, 64,  4, "nearest",     4, 0.5, 0.02, 1, "f32", 1),      # empty tensor
]


def _input(case, seed):
    (outer, C, inner, hw, raw_channels, G, B, rounding, window, tau, eps, entropy, dtype, min_out) = case
    if outer == 0:
        return np.zeros(0, np.float32 if dtype == "f32" else np.uint16)
    x, _ = W.outlier_channel_tensor(outer, C, inner, seed=seed, dist="relu" if hw else "gauss", dtype=dtype,
                                    salient_fraction=0.08, hit_fraction=0.1)
    return x


@pytest.mark.parametrize("k", range(len(CASES)))
@pytest.mark.parametrize("out_dtype", ["f32", "bf16"])
def test_single_tensor_chain_matches_the_oracle_chain(api, k, out_dtype):
    case = CASES[k]
    print(f"[chain] case {k} {case} out={out_dtype}", flush=True)
    x = _input(case, k)
    dtype = case[12]
    xd = _device(x, dtype) if x.size else torch.empty(0, dtype=torch.float32 if dtype == "f32" else torch.bfloat16, device="cuda")
    batch = api.MixBatch([_entry(api, xd, case, out_dtype)], device=torch.device("cuda"))
    batch.entries[0].store.fill_(0xAB)
    batch.entries[0].workspace.fill_(0xCD)
    torch.cuda.synchronize()
    api.fh_mix_compress_batch(batch)
    batch.entries[0].workspace.fill_(0x5A)          # the stored form alone must carry the tensor
    api.fh_mix_decompress_batch(batch)
    torch.cuda.synchronize()
    # the classification's outputs live in the workspace: compare after a second forward call
    api.fh_mix_compress_batch(batch)
    torch.cuda.synchronize()
    st = _compare(api, batch, 0, x, case, out_dtype)
    if case[4] and case[0] and k != 9:
        assert 0 < st.used <= case[4]


def test_batched_chain_item_by_item_and_in_a_captured_graph(api):
    print("[chain] batch of all cases, eager and as a replayed graph", flush=True)
    xs = [_input(c, 100 + k) for k, c in enumerate(CASES)]
    entries = []
    for x, c in zip(xs, CASES):
        dtype = c[12]
        xd = _device(x, dtype) if x.size else torch.empty(0, dtype=torch.float32 if dtype == "f32" else torch.bfloat16, device="cuda")
        entries.append(_entry(api, xd, c, "f32"))
    batch = api.MixBatch(entries, device=torch.device("cuda"))
    api.fh_mix_compress_batch(batch)
    api.fh_mix_decompress_batch(batch)
    api.fh_mix_compress_batch(batch)
    torch.cuda.synchronize()
    for i, (x, c) in enumerate(zip(xs, CASES)):
        _compare(api, batch, i, x, c, "f32")
    # the same work captured once and replayed, with eager work and synchronisation in between
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        api.fh_mix_compress_batch(batch, side)      # warm-up on the capturing stream
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            api.fh_mix_compress_batch(batch, side)
            api.fh_mix_decompress_batch(batch, side)
            api.fh_mix_compress_batch(batch, side)
    for rep in range(3):
        for e in batch.entries:
            e.store.fill_(rep)
            e.out.fill_(float(rep))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for i, (x, c) in enumerate(zip(xs, CASES)):
            _compare(api, batch, i, x, c, "f32")


def test_chain_rejects_bad_arguments_before_any_launch(api):
    print("[chain] argument checks", flush=True)
    import ctypes
    lib = api.raw_library()
    x = torch.zeros(8 * 32 * 196, device="cuda")
    good = CASES[0]
    b = api.MixBatch([_entry(api, x, good, "f32")], device=torch.device("cuda"))
    sentinel = b.entries[0].store.fill_(7).clone()
    it = b.items[0]
    for field, value, status in (("window", 3, 12), ("entropy", 2, 12), ("maps", 31, 11), ("raw_channels", 33, 11),
                                 ("reserved", 1, 12), ("store_cap", 100, 7), ("workspace_cap", 100, 7), ("x_dtype", 4, 2),
                                 ("k_sigma", 0.0, 12), ("channels", 20000, 11)):
        old = getattr(it, field)
        setattr(it, field, value)
        assert lib.fh_mix_compress(ctypes.byref(it), None) == status, field
        setattr(it, field, old)
    torch.cuda.synchronize()
    assert torch.equal(b.entries[0].store, sentinel)


def test_chain_on_tensors_without_salient_channels(api):
    """Most layers have no outlier-rich channel: the slot numbering reports zero rows in use and the
    routed quantiser takes the plain code path on the device; everything still equals the oracle chain."""
    print("[chain] nothing salient", flush=True)
    for dtype, case in (("f32", (6, 48, 784, (28, 28), 3, 128, 4, "stochastic", 4, 0.5, 0.02, 1, "f32", 10 ** 6)),
                        ("bf16", (200, 512, 1, None, 32, 64, 2, "stochastic", 4, 0.5, 0.02, 1, "bf16", 10 ** 6))):
        x = _input(case, 77)
        batch = api.MixBatch([_entry(api, _device(x, dtype), case, dtype)], device=torch.device("cuda"))
        api.fh_mix_compress_batch(batch)
        api.fh_mix_decompress_batch(batch)
        api.fh_mix_compress_batch(batch)
        torch.cuda.synchronize()
        st = _compare(api, batch, 0, x, case, dtype)
        assert st.used == 0 and not st.mask.any()


@pytest.mark.parametrize("which", ["mobilenetv2", "transformer"])
def test_full_size_set_in_one_batch_as_it_is_timed(api, which):
    """The two activation sets of `bench.py --op chain [--config 4]`, each through one batched call each way -- the
    launch configuration that is timed -- and every tensor, whole, against the oracle chain: the MobileNetV2-style
    set at batch 64 (0.57 GB of fp32; G128, 4-bit, nearest) and the transformer set (12 layers of [8192][768] and
    [8192][3072] bf16, 0.75 GB; G64, 2-bit, stochastic), outliers planted in 4 % of the channels, room for 1/16 of
    the channels in the raw store, window 4, tau 0.5, error bound 0.02, Huffman stage."""
    from concurrent.futures import ThreadPoolExecutor
    if which == "mobilenetv2":
        shapes = ((64, 32, 112 * 112, (112, 112)), (64, 96, 112 * 112, (112, 112)), (64, 144, 56 * 56, (56, 56)),
                  (64, 192, 28 * 28, (28, 28)), (64, 384, 14 * 14, (14, 14)))
        G, B, rounding, dtype, dist = 128, 4, "nearest", "f32", ("relu", "relu")
    else:
        shapes = tuple(s for _ in range(12) for s in ((16 * 512, 768, 1, None), (16 * 512, 3072, 1, None)))
        G, B, rounding, dtype, dist = 64, 2, "stochastic", "bf16", ("gauss", "gelu")
    cases, xs, entries = [], [], []
    for i, (outer, C, inner, hw) in enumerate(shapes):
        print(f"[chain] full size, {which}: tensor {i} [{outer}][{C}][{inner}]", flush=True)
        x, _ = W.outlier_channel_tensor(outer, C, inner, seed=i, dist=dist[i % 2], dtype=dtype)
        case = (outer, C, inner, hw, max(1, C // 16), G, B, rounding, 4, 0.5, 0.02, 1, dtype, max(1, outer * inner // 100))
        cases.append(case)
        xs.append(x)
        entries.append(_entry(api, _device(x, dtype), case, dtype))
    batch = api.MixBatch(entries, device=torch.device("cuda"))
    api.fh_mix_compress_batch(batch)
    api.fh_mix_decompress_batch(batch)
    api.fh_mix_compress_batch(batch)                # the classification's outputs live in the workspace
    torch.cuda.synchronize()
    print("[chain] full size: oracle chain on every tensor", flush=True)
    with ThreadPoolExecutor(max_workers=8) as pool:   # the oracle's C routines run without the interpreter lock
        kept = list(pool.map(lambda i: _compare(api, batch, i, xs[i], cases[i], dtype).used, range(len(cases))))
    assert all(0 < k <= c[4] for k, c in zip(kept, cases)), kept
