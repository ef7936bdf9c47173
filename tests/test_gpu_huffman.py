"""Parity of the HIP Huffman stage with the CPU oracle (Section 4.4.1: the quantisation codes
of the predictive form are encoded with Huffman coding; restoring begins with Huffman
decoding).  Bar: the stream -- length bytes, chunk offsets, payload words -- and the totals
bit-exact; decoding restores the input bytes."""
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


def _check(api, data, name=""):
    print(f"[huffman] {name} n={data.size}", flush=True)
    want, bits = oracle.huffman_encode(data)
    d = torch.from_numpy(data).cuda() if data.size else torch.empty(0, dtype=torch.uint8, device="cuda")
    stream, totals = api.fh_huffman_encode(d)
    torch.cuda.synchronize()
    used, got_bits = (int(v) for v in totals.cpu().tolist())
    assert (used, got_bits) == (want.size, bits), f"{name}: totals {(used, got_bits)} vs {(want.size, bits)}"
    got = stream.cpu().numpy()[:used]
    assert np.array_equal(got[:256], want[:256]), f"{name}: code lengths differ"
    chunks = (data.size + 255) // 256
    end = 256 + 4 * (chunks + 1)
    assert np.array_equal(got[256:end], want[256:end]), f"{name}: chunk offsets differ"
    bad = np.flatnonzero(got[end:] != want[end:])
    assert bad.size == 0, f"{name}: payload differs first at byte {bad[:4]}"
    back = api.fh_huffman_decode(stream[:used], data.size)
    torch.cuda.synchronize()
    assert np.array_equal(back.cpu().numpy(), data), f"{name}: decoded bytes differ"
    return used


@pytest.mark.parametrize("n", [0, 1, 15, 16, 17, 255, 256, 257, 4095, 65535, 65536, 65537, 1 << 20, (1 << 22) + 13])
def test_sizes_around_vectors_chunks_and_groups(api, n):
    rng = np.random.default_rng(n)
    data = np.clip(np.rint(rng.normal(128, 2.5, n)), 0, 255).astype(np.uint8)
    _check(api, data, "normal around 128")


@pytest.mark.parametrize("spread", [2.5, 14.0, 20.0, -1.0, 0.0])
def test_streams_long_enough_that_a_workgroup_decodes_several_groups(api, spread):
    # The decoder takes 768 chunks per workgroup and one workgroup per compute unit: 300 such groups and a ragged
    # tail are more than the device holds at once, so a workgroup takes two and the last one the ragged one.
    # spread 14: codes longer than the decoder's fast table occur; 20: more words per chunk than the decoder's LDS
    # stage holds for 768 chunks, so its passes seat fewer; -1: a clustered first half and noise behind it, passes of
    # every kind in one launch; 0: uniform bytes, whose 64 words per chunk do not fit the LDS stage of either side
    # (the direct payload stores and the per-thread rings)
    n = 256 * 768 * 300 + 77
    rng = np.random.default_rng(int(abs(spread) * 10))
    if spread > 0:
        data = np.clip(np.rint(rng.normal(128, spread, n)), 0, 255)
    elif spread < 0:
        data = np.concatenate([np.clip(np.rint(rng.normal(128, 3.0, n // 2)), 0, 255), rng.integers(0, 256, n - n // 2)])
    else:
        data = rng.integers(0, 256, n)
    _check(api, data.astype(np.uint8), f"spread {spread}")


@pytest.mark.parametrize("kind", ["uniform", "one", "two", "geometric", "all-once", "ties"])
def test_distributions(api, kind):
    rng = np.random.default_rng(1)
    n = 300001
    data = {"uniform": lambda: rng.integers(0, 256, n),
            "one": lambda: np.full(n, 77),
            "two": lambda: rng.integers(0, 2, n) * 200 + 3,
            "geometric": lambda: rng.geometric(0.05, n) % 256,
            "all-once": lambda: np.arange(256),
            "ties": lambda: np.tile(np.arange(37), 1000)}[kind]().astype(np.uint8)
    _check(api, data, kind)


def test_codes_that_would_exceed_24_bits(api):
    fib = [1, 1]
    while len(fib) < 28:
        fib.append(fib[-1] + fib[-2])
    data = np.repeat(np.arange(10, 38, dtype=np.uint8), fib)          # a 27-deep comb: counts are halved
    rng = np.random.default_rng(2)
    rng.shuffle(data)
    used = _check(api, data, "comb")
    assert used < data.size


def test_index_stream_of_the_predictive_form_end_to_end(api):
    """sparse storage with an error bound -> Huffman on its code bytes -> back -> restored maps
    equal the oracle's, and the code bytes shrink."""
    maps, h, w, n, eps = 64, 56, 56, 4, 0.02
    x = W.salient_feature_maps(maps, h, w, seed=4, zero_level=0.0)
    b = api.fh_sparse_encode(torch.from_numpy(x).cuda(), maps, h, w, n, 0.3, eps=eps)
    torch.cuda.synchronize()
    nv, ni = (int(v) for v in b.totals.cpu().tolist()[:2])
    idx = b.indices[:ni].contiguous()
    stream, totals = api.fh_huffman_encode(idx)
    torch.cuda.synchronize()
    used = int(totals[0])
    want, _ = oracle.huffman_encode(idx.cpu().numpy())
    assert np.array_equal(stream.cpu().numpy()[:used], want)
    print(f"[huffman] index stream {ni} -> {used} bytes", flush=True)
    assert used < 0.9 * ni
    idx_back = api.fh_huffman_decode(stream[:used], ni)
    out = api.fh_sparse_decode(b.info, b.values[:nv], idx_back, maps, h, w, n, eps=eps)
    torch.cuda.synchronize()
    info, v, i, _ = oracle.sparse_encode(x, maps, h, w, n, 0.3, eps=eps)
    assert np.array_equal(out.cpu().numpy().view(np.uint32), oracle.sparse_decode(info, v, i, maps, h, w, n, eps=eps).view(np.uint32))


def test_decoder_stays_inside_truncated_or_foreign_streams(api):
    rng = np.random.default_rng(3)
    data = np.clip(np.rint(rng.normal(128, 6, 200000)), 0, 255).astype(np.uint8)
    stream, totals = api.fh_huffman_encode(torch.from_numpy(data).cuda())
    torch.cuda.synchronize()
    used = int(totals[0])
    chunks = (data.size + 255) // 256
    header = 256 + 4 * (chunks + 1)
    # payload cut in half: the chunks that are still there come back exactly
    cut = header + ((used - header) // 8) * 4
    out = api.fh_huffman_decode(stream[:cut], data.size).cpu().numpy()
    torch.cuda.synchronize()
    assert np.array_equal(out[: data.size // 4], data[: data.size // 4]) and not np.array_equal(out, data)
    # random bytes as a stream (lengths, offsets and payload): must simply finish
    junk = torch.randint(0, 256, (used,), dtype=torch.uint8, device="cuda")
    out = api.fh_huffman_decode(junk, data.size)
    torch.cuda.synchronize()
    assert out.numel() == data.size
    # a stream too short to hold the lengths and the offsets is refused on the host
    with pytest.raises(api.FedHybridError):
        api.fh_huffman_decode(stream[: header - 4], data.size)


def test_buffers_can_be_reused_and_errors_reach_the_caller(api):
    a = (np.arange(100000) % 7).astype(np.uint8)
    b = (np.arange(50000) % 200).astype(np.uint8)
    out = torch.empty(api.huffman_stream_bytes(a.size), dtype=torch.uint8, device="cuda")
    tot = torch.zeros(2, dtype=torch.int64, device="cuda")
    ws = torch.empty(api.huffman_workspace_bytes(a.size), dtype=torch.uint8, device="cuda")
    for data in (a, b, a):
        api.fh_huffman_encode(torch.from_numpy(data).cuda(), stream_out=out, totals=tot, workspace=ws)
        torch.cuda.synchronize()
        want, bits = oracle.huffman_encode(data)
        assert tot.cpu().tolist() == [want.size, bits]
        assert np.array_equal(out.cpu().numpy()[: want.size], want)
    with pytest.raises(api.FedHybridError):
        api.fh_huffman_encode(torch.from_numpy(a).cuda(), stream_out=out[:1000], totals=tot, workspace=ws)
    with pytest.raises(api.FedHybridError):
        api.fh_huffman_encode(torch.from_numpy(a).cuda()[1:], stream_out=out, totals=tot, workspace=ws)   # misaligned


def test_batched_calls_match_the_oracle_for_every_stream(api):
    """More streams than one launch holds, an empty one among them, sizes from one symbol to a few groups."""
    rng = np.random.default_rng(9)
    sizes = [1, 0, 300, 65536, 200001, 77] + [1000 + 4099 * i for i in range(14)]
    datas = []
    for i, n in enumerate(sizes):
        spread = 1.0 + (i % 5) * 3.0
        datas.append(np.clip(np.rint(rng.normal(128, spread, n)), 0, 255).astype(np.uint8))
    assert len(datas) > api.huffman_batch_capacity()
    dev = [torch.from_numpy(d).cuda() if d.size else torch.empty(0, dtype=torch.uint8, device="cuda") for d in datas]
    batch = api.HuffmanBatch(dev)
    api.fh_huffman_encode_batch(batch)
    torch.cuda.synchronize()
    used = batch.refresh()
    api.fh_huffman_decode_batch(batch)
    torch.cuda.synchronize()
    totals = batch.totals.cpu().tolist()
    for i, d in enumerate(datas):
        want, bits = oracle.huffman_encode(d)
        assert totals[i] == [want.size, bits], f"stream {i}: totals"
        assert np.array_equal(batch.streams[i].cpu().numpy()[: used[i]], want), f"stream {i}: bytes"
        assert np.array_equal(batch.out[i].cpu().numpy(), d), f"stream {i}: decoded"


def test_symbol_count_taken_from_device_memory(api):
    """The buffer's length is the output of an earlier call on the stream: buffers and launches are
    sized for an upper bound, the count comes from device memory, and nothing is read back between
    encode and decode."""
    rng = np.random.default_rng(5)
    cap = 300_000
    full = np.clip(np.rint(rng.normal(128.0, 5.0, cap)), 0, 255).astype(np.uint8)
    counts = [0, 1, 255, 256, 257, 65_536, 65_537, 200_001, cap, cap + 999]        # the last: clipped to the bound
    data = [torch.from_numpy(full.copy()).cuda() for _ in counts]
    n_dev = [torch.tensor([c], dtype=torch.int64, device="cuda") for c in counts]
    batch = api.HuffmanBatch(data, n_device=n_dev)
    for o in batch.out:
        o.fill_(0xEE)
    torch.cuda.synchronize()
    api.fh_huffman_encode_batch(batch)
    api.fh_huffman_decode_batch(batch)                       # no refresh: stream capacities bound the reads
    torch.cuda.synchronize()
    totals = batch.totals.cpu().numpy()
    for k, c in enumerate(counts):
        n = min(c, cap)
        print(f"[huffman] device count {c} of capacity {cap}", flush=True)
        want, bits = oracle.huffman_encode(full[:n])
        assert (int(totals[k, 0]), int(totals[k, 1])) == (want.size, bits)
        assert np.array_equal(batch.streams[k].cpu().numpy()[:want.size], want)
        back = batch.out[k].cpu().numpy()
        assert np.array_equal(back[:n], full[:n])
        assert np.all(back[-(-n // 16) * 16:] == 0xEE)          # nothing written past the count's last 16-byte vector
