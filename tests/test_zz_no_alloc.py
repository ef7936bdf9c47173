"""The entry point that allocates nothing: fh_classify_channels_static keeps the partial sums of
the channel classification in the library's static device buffer.  Called through the C ABI
and compared with fh_classify_channels (caller-provided workspace), whose results the other
tests compare with the oracle: statistics bit-exact, counts and mask exact, on two calls in a
row, the second on a smaller input (the buffer keeps the first call's contents)."""
from __future__ import annotations

import numpy as np
import pytest

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


def _both(api, x, outer, C, inner, k, min_out, dtype):
    xd = _device(x, dtype)
    want = api.fh_classify_channels(xd, outer, C, inner, k, min_out)
    stats = torch.full((4,), -1.0, dtype=torch.float64, device="cuda")
    counts = torch.full((C,), 77, dtype=torch.int32, device="cuda")
    mask = torch.full((C,), 9, dtype=torch.uint8, device="cuda")
    torch.cuda.synchronize()
    # requests served by torch's allocator so far (a count that only grows: blocks that earlier tests handed to
    # side streams may be given back at any time, so the bytes in use can fall during the call)
    before = torch.cuda.memory_stats()["allocation.all.allocated"]
    api.fh_classify_channels_static(xd, outer, C, inner, k, min_out, stats, counts, mask)
    torch.cuda.synchronize()
    assert torch.cuda.memory_stats()["allocation.all.allocated"] == before
    for got, ref, what in zip((stats, counts, mask), want, ("stats", "counts", "mask")):
        g, r = got.cpu().numpy(), ref.cpu().numpy()
        assert np.array_equal(g.view(np.uint8), r.view(np.uint8)), f"{what} differ: {g[:8]} vs {r[:8]}"
    return stats.cpu().numpy()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_two_calls_in_a_row_the_second_smaller(api, dtype):
    # 5.6 M elements: two levels of the partial-sum tree; then 70 k elements, one level, into
    # the same buffer, which still holds the first call's partial sums
    for outer, C, inner in ((28, 64, 56 * 56), (3, 24, 31 * 31)):
        print(f"[no-alloc] {dtype} [{outer}][{C}][{inner}]", flush=True)
        x, _ = W.outlier_channel_tensor(outer, C, inner, seed=outer, dist="relu", dtype=dtype)
        s = _both(api, x, outer, C, inner, 3.0, max(1, outer * inner // 100), dtype)
        assert s[3] == outer * C * inner and s[1] > 0.0


def test_empty_tensor_and_size_limit(api):
    print("[no-alloc] empty tensor, size limit", flush=True)
    stats = torch.full((4,), -1.0, dtype=torch.float64, device="cuda")
    counts = torch.full((8,), 5, dtype=torch.int32, device="cuda")
    mask = torch.full((8,), 5, dtype=torch.uint8, device="cuda")
    x = torch.empty(0, dtype=torch.float32, device="cuda")
    api.fh_classify_channels_static(x, 0, 8, 16, 3.0, 1, stats, counts, mask)
    torch.cuda.synchronize()
    assert stats.cpu().tolist() == [0.0, 0.0, 0.0, 0.0] and not counts.any() and not mask.any()
    # one element more than the static buffer serves: refused on the host, nothing launched
    limit = api.classify_static_scratch_bytes()
    assert limit == 4 << 20
    lib = api.raw_library()
    n_ok = 261_887 * 1024                        # 261887 + 256 + 1 pairs = 4 MiB exactly
    assert api.classify_workspace_bytes(n_ok) == limit and api.classify_workspace_bytes(n_ok + 1) > limit
    fake = 0x10000
    assert lib.fh_classify_channels_static(fake, 0, 1, 1, n_ok + 1, 3.0, 1, fake, fake, fake, None) == 13
    assert "static buffer" in api.status_string(13)
