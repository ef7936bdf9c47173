"""The binding's temporaries on a side stream: fh_classify_channels, fh_sparse_decode and
fh_huffman_encode allocate their scratch themselves when the caller passes none, launch on the
caller's stream and drop the tensor on return.  With allocation churn on the default stream
right behind such a call the results must still equal the oracle's (the scratch block must not
be handed out again while the side stream's kernels use it)."""
from __future__ import annotations

import numpy as np
import pytest

import oracle
from paper_2510_11400_amd import workloads as W

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def api():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a visible MI355X")
    from paper_2510_11400_amd import api as _api
    return _api


def _churn(nbytes, rounds=6):
    """Allocate, fill and drop blocks of the scratch's size on the current (default) stream."""
    for k in range(rounds):
        t = torch.empty(max(16, nbytes), dtype=torch.uint8, device="cuda")
        t.fill_(0xA5 ^ k)
        del t


def test_classify_on_side_stream_with_churn(api):
    print("[side-stream] classify", flush=True)
    outer, C, inner = 48, 96, 56 * 56
    x, _ = W.outlier_channel_tensor(outer, C, inner, seed=5, dist="relu")
    stats, counts, mask = oracle.classify_channels(x, outer, C, inner, 3.0, outer * inner // 100)
    xd = torch.from_numpy(x).cuda()
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    nbytes = api.classify_workspace_bytes(x.size)
    for _ in range(3):
        gs, gc, gm = api.fh_classify_channels(xd, outer, C, inner, 3.0, outer * inner // 100, stream=side)
        _churn(nbytes)
        side.synchronize()
        torch.cuda.synchronize()
        assert np.array_equal(gs.cpu().numpy().view(np.uint64), stats.view(np.uint64))
        assert np.array_equal(gc.cpu().numpy().view(np.uint32), counts)
        assert np.array_equal(gm.cpu().numpy(), mask)


def test_sparse_decode_on_side_stream_with_churn(api):
    print("[side-stream] sparse decode", flush=True)
    maps, h, w, n = 700, 56, 56, 4
    x = W.salient_feature_maps(maps, h, w, seed=3)
    xd = torch.from_numpy(x).cuda()
    bufs = api.fh_sparse_encode(xd, maps, h, w, n, 0.5)
    torch.cuda.synchronize()
    nv, ni = int(bufs.totals[0]), int(bufs.totals[1])
    side = torch.cuda.Stream()
    nbytes = api.sparse_workspace_bytes(maps, h, w, n)
    for _ in range(3):
        out = torch.empty(x.size, dtype=torch.float32, device="cuda")
        torch.cuda.synchronize()
        api.fh_sparse_decode(bufs.info, bufs.values[:nv], bufs.indices[:ni], maps, h, w, n, out=out, stream=side)
        _churn(nbytes)
        side.synchronize()
        torch.cuda.synchronize()
        assert np.array_equal(out.cpu().numpy().view(np.uint32), x.reshape(-1).view(np.uint32))


def test_huffman_encode_on_side_stream_with_churn(api):
    print("[side-stream] huffman encode", flush=True)
    rng = np.random.default_rng(11)
    data = np.clip(np.rint(rng.normal(128.0, 6.0, 3_000_001)), 0, 255).astype(np.uint8)
    want, bits = oracle.huffman_encode(data)
    d = torch.from_numpy(data).cuda()
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    nbytes = api.huffman_workspace_bytes(data.size)
    for _ in range(3):
        stream_out, totals = api.fh_huffman_encode(d, stream=side)
        _churn(nbytes)
        side.synchronize()
        torch.cuda.synchronize()
        used, got_bits = (int(v) for v in totals.cpu().tolist())
        assert (used, got_bits) == (want.size, bits)
        assert np.array_equal(stream_out.cpu().numpy()[:used], want)
