"""The saved-tensor hooks on the GPU (Section 3: activations are compressed in the forward
pass and decompressed during backpropagation): what backward sees is bit for bit the
oracle's round trip of what forward saved, parameters stay exact, and the recorded purge /
regain costs give the MPS of compression (Section 4.3)."""
from __future__ import annotations

import numpy as np
import pytest

import oracle

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu
f32 = np.float32


@pytest.fixture(scope="module")
def hooks():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a visible MI355X")
    from paper_2510_11400_amd import hooks as _hooks
    return _hooks


def _oracle_roundtrip(x_host, G, B, rounding, seed, tid, dtype):
    if dtype == "bf16":
        bits = x_host.view(torch.int16).numpy().view(np.uint16).reshape(-1)
        p, m = oracle.compress(bits, G, B, rounding, seed, tid, dtype="bf16")
        y = oracle.decompress(p, m, bits.size, G, B, out_dtype="bf16")
        return torch.from_numpy(y.view(np.int16)).view(torch.bfloat16).reshape(x_host.shape)
    flat = x_host.numpy().reshape(-1)
    p, m = oracle.compress(flat, G, B, rounding, seed, tid)
    return torch.from_numpy(oracle.decompress(p, m, flat.size, G, B)).reshape(x_host.shape)


class _Probe(torch.autograd.Function):
    """Saves its input and hands whatever backward gets back to the test."""
    seen = []

    @staticmethod
    def forward(ctx, x):
        ctx.save_for_backward(x)
        return x * 1.0

    @staticmethod
    def backward(ctx, g):
        (x,) = ctx.saved_tensors
        _Probe.seen.append(x.detach().clone())
        return g


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("G,B,rounding", [(256, 4, "nearest"), (64, 2, "stochastic"), (128, 8, "stochastic")])
def test_backward_sees_the_oracles_round_trip(hooks, dtype, G, B, rounding):
    print(f"[hooks] probe {dtype} G{G} B{B} {rounding}", flush=True)
    torch.manual_seed(G + B)
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    shapes = [(32, 24, 14, 14), (16, 512, 77), (5000,)]
    _Probe.seen.clear()
    xs = [torch.randn(s, device="cuda").to(tdt).requires_grad_(True) for s in shapes]
    ctx = hooks.SavedActivations(G, B, rounding, seed=17, min_numel=1, first_tensor_id=40)
    with ctx:
        total = sum(_Probe.apply(x).float().sum() for x in xs)
    total.backward()
    torch.cuda.synchronize()
    assert ctx.next_tensor_id == 43
    for k, x in enumerate(xs):                             # backward visits them in reverse
        got = _Probe.seen[len(xs) - 1 - k].cpu()
        want = _oracle_roundtrip(x.detach().cpu(), G, B, rounding, 17, 40 + k, dtype)
        assert got.shape == x.shape and got.dtype == x.dtype
        view = torch.int32 if dtype == "f32" else torch.int16
        assert torch.equal(got.view(view), want.view(view)), f"tensor {k}"


def test_non_contiguous_and_small_tensors_and_parameters(hooks):
    _Probe.seen.clear()
    base = torch.randn(64, 96, device="cuda")
    x = base.t().requires_grad_(True)                      # non-contiguous view
    small = torch.randn(10, device="cuda", requires_grad=True)
    w = torch.nn.Parameter(torch.randn(96, 64, device="cuda"))
    ctx = hooks.SavedActivations(64, 8, min_numel=1000, record=True, exclude=[w])
    with ctx:
        y = _Probe.apply(x).sum() + _Probe.apply(small).sum() + _Probe.apply(w).sum()
    y.backward()
    torch.cuda.synchronize()
    assert len(ctx.records) == 1                           # only x was compressed
    seen_w, seen_small, seen_x = _Probe.seen
    assert torch.equal(seen_w, w.detach()) and torch.equal(seen_small, small.detach())
    want = _oracle_roundtrip(x.detach().contiguous().cpu(), 64, 8, "nearest", 0, 0, "f32")
    assert torch.equal(seen_x.cpu().view(torch.int32), want.view(torch.int32))


def test_linear_layer_gradient_uses_the_restored_activation(hooks):
    torch.manual_seed(3)
    x = torch.randn(256, 512, device="cuda")
    lin = torch.nn.Linear(512, 128, bias=False).cuda()
    gy = torch.randn(256, 128, device="cuda")
    with hooks.SavedActivations(128, 4, "stochastic", seed=5, min_numel=1, exclude=lin.parameters()):
        y = lin(x)
    y.backward(gy)
    x_hat = _oracle_roundtrip(x.cpu(), 128, 4, "stochastic", 5, 0, "f32").cuda()
    want = gy.t() @ x_hat                                  # dL/dW = gy^T x_saved
    assert torch.allclose(lin.weight.grad, want, rtol=1e-4, atol=1e-4)
    exact = gy.t() @ x
    assert not torch.allclose(lin.weight.grad, exact, rtol=1e-4, atol=1e-4)   # it really used the lossy copy


def test_recorded_costs_give_the_mps_of_compression(hooks):
    x = torch.randn(64, 96, 56, 56, device="cuda", requires_grad=True)
    ctx = hooks.SavedActivations(256, 4, record=True)
    _Probe.seen.clear()
    with ctx:
        y = _Probe.apply(x).sum()
    y.backward()
    torch.cuda.synchronize()
    (rec,) = ctx.records
    n = x.numel()
    assert rec.input_bytes == 4 * n and rec.stored_bytes == n // 2 + 8 * (n // 256)
    assert rec.saved_bytes == rec.input_bytes - rec.stored_bytes
    assert 0 < rec.purge_cost < 0.05 and 0 < rec.regain_cost < 0.05
    flt = 0.010
    assert rec.mps_compress(flt) == hooks.mps(rec.saved_bytes, flt, rec.purge_cost, rec.regain_cost)


def test_a_small_network_trains_through_the_hooks(hooks):
    torch.manual_seed(0)
    net = torch.nn.Sequential(torch.nn.Linear(256, 512), torch.nn.ReLU(), torch.nn.Linear(512, 512), torch.nn.ReLU(),
                              torch.nn.Linear(512, 10)).cuda()
    x = torch.randn(512, 256, device="cuda")
    target = torch.randint(0, 10, (512,), device="cuda")
    loss_fn = torch.nn.CrossEntropyLoss()
    loss_fn(net(x), target).backward()
    ref = [p.grad.clone() for p in net.parameters()]
    net.zero_grad()
    ctx = hooks.SavedActivations(256, 8, min_numel=4096, record=True, exclude=net.parameters())
    with ctx:
        loss = loss_fn(net(x), target)
    loss.backward()
    torch.cuda.synchronize()
    assert len(ctx.records) >= 3
    # 8-bit activations.  The error is dominated by ReLU masks taken from the restored tensor:
    # nearest rounding flushes the ~0.5 % smallest positive activations to zero, and dropping a
    # fraction f of the terms of a gradient sum costs about sqrt(f) of its norm.
    for g, p in zip(ref, net.parameters()):
        rel = (p.grad - g).norm() / g.norm()
        cos = torch.nn.functional.cosine_similarity(p.grad.flatten(), g.flatten(), dim=0)
        assert rel < 0.2 and cos > 0.98, (float(rel), float(cos))


# ---- the channel-wise mix inside the hooks (Section 4.4.1) ------------------------------------------

def _oracle_channel_wise(x_host, outer, C, inner, G, B, rounding, seed, tid, dtype, k_sigma, share, raw_share):
    bits = x_host.view(torch.int16).numpy().view(np.uint16).reshape(-1) if dtype == "bf16" else x_host.numpy().reshape(-1)
    min_outliers = max(1, int(outer * inner * share))
    _, _, mask = oracle.classify_channels(bits, outer, C, inner, k_sigma, min_outliers, dtype=dtype)
    cap = max(1, min(C, int(C * raw_share + 0.5)))
    slots, used = oracle.channel_slots(mask, cap)
    p, m, raw = oracle.compress_mixed(bits, outer, C, inner, slots, cap, G, B, rounding, seed, tid, dtype=dtype)
    y = oracle.decompress_mixed(p, m, raw, outer, C, inner, slots, cap, G, B, raw_dtype=dtype, out_dtype=dtype)
    if dtype == "bf16":
        return torch.from_numpy(y.view(np.int16)).view(torch.bfloat16).reshape(x_host.shape), used
    return torch.from_numpy(y).reshape(x_host.shape), used


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape,channel_dim", [((24, 48, 14, 14), 1), ((6, 200, 768), -1), ((40, 96), 1)])
def test_channel_wise_hooks_give_backward_the_oracles_chain(hooks, dtype, shape, channel_dim):
    """classify -> slots -> mixed compress in the pack hook, mixed restore in the unpack hook:
    bit for bit the oracle's chain, and the planted channels come back exactly."""
    from paper_2510_11400_amd import workloads as W
    print(f"[hooks] channel-wise {dtype} {shape} dim {channel_dim}", flush=True)
    d = channel_dim % len(shape)
    outer = int(np.prod(shape[:d])) if d else 1
    C = shape[d]
    inner = int(np.prod(shape[d + 1:])) if d + 1 < len(shape) else 1
    x_np, planted = W.outlier_channel_tensor(outer, C, inner, seed=C, dist="gauss", salient_fraction=0.05, dtype=dtype)
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    x_host = (torch.from_numpy(x_np.view(np.int16)).view(torch.bfloat16) if dtype == "bf16" else torch.from_numpy(x_np)).reshape(shape)
    x = x_host.cuda().requires_grad_(True)
    G, B, rounding, seed = 64, 4, "stochastic", 5
    _Probe.seen.clear()
    ctx = hooks.SavedActivations(G, B, rounding, seed=seed, min_numel=1, first_tensor_id=9, channel_dim=channel_dim,
                                 record=True)
    with ctx:
        y = _Probe.apply(x)
    y.sum().backward()
    torch.cuda.synchronize()
    want, used = _oracle_channel_wise(x_host, outer, C, inner, G, B, rounding, seed, 9, dtype, 3.0, 0.01, 1.0 / 16.0)
    got = _Probe.seen[0].cpu()
    assert got.shape == x_host.shape and got.dtype == tdt
    same = got.view(torch.int16 if dtype == "bf16" else torch.int32) == want.view(torch.int16 if dtype == "bf16" else torch.int32)
    assert bool(same.all())
    moved = [slice(None)] * len(shape)
    kept_exact = 0
    for c in planted:                                          # the planted channels were found, got a row, and are exact
        moved[d] = int(c)
        kept_exact += bool((got[tuple(moved)] == x_host[tuple(moved)]).all())
    assert used == len(planted) and kept_exact == len(planted)
    assert ctx.records[0].stored_bytes < ctx.records[0].input_bytes


def test_channel_wise_hooks_shrink_the_error_of_the_normal_channels(hooks):
    """With 81x outliers in a few channels the plain quantiser's error follows the outliers'
    range; with those channels kept aside it follows the normal channels' own range."""
    from paper_2510_11400_amd import workloads as W
    outer, C, inner = 32, 64, 400
    x_np, planted = W.outlier_channel_tensor(outer, C, inner, seed=3, dist="gauss", salient_fraction=0.05, magnitude=81.0)
    x_host = torch.from_numpy(x_np).reshape(outer, C, inner)
    normal = np.setdiff1d(np.arange(C), planted)
    errs = {}
    for name, kw in (("plain", {}), ("channel-wise", {"channel_dim": 1})):
        _Probe.seen.clear()
        x = x_host.cuda().requires_grad_(True)
        with hooks.SavedActivations(256, 4, "nearest", min_numel=1, **kw):
            y = _Probe.apply(x)
        y.sum().backward()
        torch.cuda.synchronize()
        got = _Probe.seen[0].cpu()
        errs[name] = float((got[:, normal] - x_host[:, normal]).abs().max())
    print(f"[hooks] max error on normal channels: {errs}", flush=True)
    assert errs["channel-wise"] < errs["plain"] / 8


def test_a_contiguous_view_at_an_odd_storage_offset_is_compressed_from_a_copy(hooks):
    """The kernels want 16-byte aligned tensors; a saved view that starts 4 bytes into its storage is
    contiguous but not aligned, and must neither raise inside the forward pass nor change the result."""
    _Probe.seen.clear()
    base = torch.randn(1 + 64 * 96, device="cuda")
    x = base[1:].view(64, 96).requires_grad_(True)
    assert x.is_contiguous() and x.data_ptr() % 16 != 0
    ctx = hooks.SavedActivations(64, 8, min_numel=1, record=True)
    with ctx:
        y = _Probe.apply(x).sum()
    y.backward()
    torch.cuda.synchronize()
    assert len(ctx.records) == 1
    want = _oracle_roundtrip(x.detach().cpu().contiguous(), 64, 8, "nearest", 0, 0, "f32")
    assert torch.equal(_Probe.seen[0].cpu().view(torch.int32), want.view(torch.int32))


@pytest.mark.parametrize("channel_wise", [False, True])
@pytest.mark.parametrize("batch_bytes", [1, 300_000, 1 << 30])
def test_tensors_compressed_in_batches_give_the_same_bytes(hooks, channel_wise, batch_bytes):
    """batch_bytes > 0: the pack hook only notes a tensor; the batch goes through the batched entry points
    when it is full (1: every tensor at once; 300 kB: every few), when the context ends (1 GiB), or when
    a tensor is needed back first.  What backward sees is the oracle's result for each tensor's own id."""
    from paper_2510_11400_amd import workloads as W
    print(f"[hooks] batches of {batch_bytes} bytes, channel-wise {channel_wise}", flush=True)
    shapes = [(6, 40, 10, 10), (50, 96), (3, 16, 33), (9000,), (12, 24, 7, 7), (64, 128)]
    G, B, rounding, seed = 64, 4, "stochastic", 21
    hosts = []
    for k, shp in enumerate(shapes):
        if len(shp) >= 2:
            outer, C, inner = shp[0], shp[1], int(np.prod(shp[2:])) if len(shp) > 2 else 1
            x_np, _ = W.outlier_channel_tensor(outer, C, inner, seed=k, dist="gauss", salient_fraction=0.1)
        else:
            x_np = np.random.default_rng(k).standard_normal(shp[0]).astype(np.float32)
        hosts.append(torch.from_numpy(x_np).reshape(shp))
    _Probe.seen.clear()
    xs = [h.cuda().requires_grad_(True) for h in hosts]
    kw = {"channel_dim": 1} if channel_wise else {}
    ctx = hooks.SavedActivations(G, B, rounding, seed=seed, min_numel=1, first_tensor_id=3, batch_bytes=batch_bytes,
                                 record=True, **kw)
    with ctx:
        total = sum(_Probe.apply(x).sum() for x in xs[:4])
        if batch_bytes == 300_000:
            early = torch.autograd.grad(_Probe.apply(xs[4]).sum(), xs[4])[0]     # needed back before its batch is full
            assert early.shape == xs[4].shape
            first_seen = _Probe.seen.pop()
        else:
            total = total + _Probe.apply(xs[4]).sum()
            first_seen = None
        total = total + _Probe.apply(xs[5]).sum()
    total.backward()
    torch.cuda.synchronize()
    assert ctx.next_tensor_id == 3 + len(xs) and not ctx._pending
    seen = {}
    order = [5, 3, 2, 1, 0] if first_seen is not None else [5, 4, 3, 2, 1, 0]           # backward visits them in reverse
    for k, got in zip(order, _Probe.seen):
        seen[k] = got
    if first_seen is not None:
        seen[4] = first_seen
    for k, h in enumerate(hosts):
        shp = shapes[k]
        if channel_wise:
            outer, C, inner = (shp[0], shp[1], int(np.prod(shp[2:])) if len(shp) > 2 else 1) if len(shp) >= 2 else (1, shp[0], 1)
            want, _ = _oracle_channel_wise(h, outer, C, inner, G, B, rounding, seed, 3 + k, "f32", 3.0, 0.01, 1.0 / 16.0)
        else:
            want = _oracle_roundtrip(h, G, B, rounding, seed, 3 + k, "f32")
        assert torch.equal(seen[k].cpu().view(torch.int32), want.view(torch.int32)), f"tensor {k}"
    assert len(ctx.records) == len(xs) and all(r.purge_cost is not None and r.purge_cost >= 0 for r in ctx.records)
