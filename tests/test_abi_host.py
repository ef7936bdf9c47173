"""Host-side checks of the C ABI that need no GPU: the library loads, exports every
symbol the header declares, sizes its buffers like the definition says, and rejects
bad arguments before anything could be launched."""
from __future__ import annotations

import ctypes
import os
import re

import pytest

import oracle
from paper_2510_11400_amd import api

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "fedhybrid.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(fh_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _declared_symbols()
    assert set(names) == set(api.EXPORTS)
    lib = api.raw_library()
    for n in names:
        assert getattr(lib, n) is not None


def test_size_helpers_match_the_definition():
    for bits in (2, 4, 8):
        for n in (1, 7, 8, 63, 64, 65, 255, 256, 257, 4095, 4096, 4097, 10 ** 9 + 7):
            raw = -(-n * bits // 8)
            assert api.packed_bytes(n, bits) == -(-raw // 16) * 16 == oracle.packed_bytes(n, bits)
    for g in (64, 128, 256):
        for n in (1, g - 1, g, g + 1, 10 ** 9 + 7):
            assert api.meta_bytes(n, g) == 8 * -(-n // g) == oracle.meta_bytes(n, g)
    assert api.packed_bytes(0, 4) == 0 and api.packed_bytes(-3, 4) == 0 and api.packed_bytes(10, 3) == 0
    assert api.meta_bytes(0, 64) == 0 and api.meta_bytes(5, 0) == 0
    assert 1 <= api.batch_capacity() <= 64


def test_struct_layout_matches_the_header():
    assert ctypes.sizeof(api.fh_params) == 32
    assert ctypes.sizeof(api.fh_item) == 8 + 8 + 8 + 16 + 16 + 16 + 32
    assert api.fh_item.params.offset == 72


FAKE = 0x10000  # an aligned non-NULL address; never dereferenced because validation fails first


def _compress(x=FAKE, dtype=0, n=1024, g=256, b=4, r=0, packed=FAKE, pcap=1 << 20, meta=FAKE, mcap=1 << 20):
    p = api.fh_params(g, b, r, 0, 0, 0)
    return api.raw_library().fh_compress(x, dtype, n, ctypes.byref(p), packed, pcap, meta, mcap, None)


def _decompress(packed=FAKE, meta=FAKE, n=1024, g=256, b=4, odt=0, out=FAKE, ocap=1 << 20):
    p = api.fh_params(g, b, 0, 0, 0, 0)
    return api.raw_library().fh_decompress(packed, meta, n, ctypes.byref(p), odt, out, ocap, None)


def test_compress_rejects_bad_arguments_before_any_launch():
    assert _compress(g=100) == 3 and _compress(g=512) == 3
    assert _compress(b=3) == 4 and _compress(b=16) == 4
    assert _compress(r=2) == 5
    assert _compress(dtype=7) == 2
    assert _compress(n=-1) == 6
    assert _compress(x=None) == 1 and _compress(packed=None) == 1 and _compress(meta=None) == 1
    assert _compress(x=FAKE + 4) == 8 and _compress(packed=FAKE + 8) == 8 and _compress(meta=FAKE + 4) == 8
    assert _compress(pcap=511) == 7 and _compress(mcap=31) == 7
    assert api.raw_library().fh_compress(FAKE, 0, 1024, None, FAKE, 1 << 20, FAKE, 1 << 20, None) == 1
    # numel == 0 is fine and launches nothing, whatever the pointers
    assert _compress(n=0, x=None, packed=None, meta=None) == 0


def test_decompress_rejects_bad_arguments_before_any_launch():
    assert _decompress(g=32) == 3 and _decompress(b=1) == 4 and _decompress(odt=2) == 2
    assert _decompress(n=-5) == 6
    assert _decompress(packed=None) == 1 and _decompress(meta=None) == 1 and _decompress(out=None) == 1
    assert _decompress(out=FAKE + 2) == 8
    assert _decompress(ocap=4095) == 7 and _decompress(odt=1, ocap=2047) == 7
    assert _decompress(n=0, out=None) == 0


def test_batch_validates_every_item_before_the_first_launch():
    items = (api.fh_item * 2)()
    for it in items:
        it.x = it.packed = it.meta = it.out = FAKE
        it.numel = 256
        it.packed_cap = it.meta_cap = it.out_cap = 1 << 20
        it.params = api.fh_params(256, 8, 0, 0, 0, 0)
    items[1].params.bits = 5                      # second item is bad: nothing may run
    lib = api.raw_library()
    assert lib.fh_compress_batch(items, 2, None) == 4
    assert lib.fh_decompress_batch(items, 2, None) == 4
    assert lib.fh_roundtrip_batch(items, 2, None) == 4
    assert lib.fh_compress_batch(items, -1, None) == 10
    assert lib.fh_compress_batch(None, 1, None) == 1
    assert lib.fh_compress_batch(None, 0, None) == 0


def test_status_strings():
    seen = set()
    for s in range(0, 13):
        msg = api.status_string(s)
        assert msg and msg != "unknown status"
        seen.add(msg)
    assert len(seen) == 13
    assert api.status_string(99) == "unknown status"
    with pytest.raises(api.FedHybridError) as e:
        api._check(4)
    assert "bits" in str(e.value)


def _classify(x=FAKE, dtype=0, outer=4, channels=8, inner=16, k=3.0, min_out=1, ws=FAKE, ws_cap=1 << 20,
              stats=FAKE, counts=FAKE, mask=FAKE):
    return api.raw_library().fh_classify_channels(x, dtype, outer, channels, inner, k, min_out, ws, ws_cap,
                                                   stats, counts, mask, None)


def test_classify_rejects_bad_arguments_before_any_launch():
    assert _classify(dtype=3) == 2
    assert _classify(outer=-1) == 11 and _classify(inner=0) == 11
    assert _classify(channels=0) == 11 and _classify(channels=16385) == 11
    assert _classify(k=0.0) == 12 and _classify(k=-3.0) == 12 and _classify(k=float("nan")) == 12
    assert _classify(min_out=0) == 12
    assert _classify(x=None) == 1 and _classify(ws=None) == 1 and _classify(stats=None) == 1
    assert _classify(counts=None) == 1 and _classify(mask=None) == 1
    assert _classify(x=FAKE + 8) == 8 and _classify(ws=FAKE + 8) == 8 and _classify(stats=FAKE + 4) == 8
    assert _classify(ws_cap=15) == 7
    assert _classify(outer=1 << 30, channels=16384, inner=1 << 20) == 6


def test_classify_workspace_size_covers_every_level_of_the_tree():
    for n in (1, 1023, 1024, 1025, 1 << 20, (1 << 20) + 1, 536870496):
        pairs, m = 0, -(-n // 1024)
        while True:
            pairs += m
            if m == 1:
                break
            m = -(-m // 1024)
        assert api.classify_workspace_bytes(n) == 16 * pairs
    assert api.classify_workspace_bytes(0) == 16


def _params(G=64, B=4, rounding=0):
    return api.fh_params(G, B, rounding, 0, 0, 0)


def _cmixed(x=FAKE, dtype=0, outer=4, channels=8, inner=16, params="default", slots=FAKE, raw_channels=2,
            packed=FAKE, packed_cap=1 << 20, meta=FAKE, meta_cap=1 << 20, raw=FAKE, raw_cap=1 << 20):
    p = _params() if params == "default" else params
    return api.raw_library().fh_compress_mixed(x, dtype, outer, channels, inner,
                                               ctypes.byref(p) if p is not None else None, slots, raw_channels,
                                               packed, packed_cap, meta, meta_cap, raw, raw_cap, None)


def _dmixed(packed=FAKE, meta=FAKE, raw=FAKE, raw_dtype=0, outer=4, channels=8, inner=16, params="default",
            slots=FAKE, raw_channels=2, out_dtype=0, out=FAKE, out_cap=1 << 20):
    p = _params() if params == "default" else params
    return api.raw_library().fh_decompress_mixed(packed, meta, raw, raw_dtype, outer, channels, inner,
                                                 ctypes.byref(p) if p is not None else None, slots, raw_channels,
                                                 out_dtype, out, out_cap, None)


def test_mixed_calls_reject_bad_arguments_before_any_launch():
    assert _cmixed(params=None) == 1 and _dmixed(params=None) == 1
    assert _cmixed(params=_params(G=32)) == 3 and _cmixed(params=_params(B=3)) == 4
    assert _cmixed(params=_params(rounding=2)) == 5
    assert _cmixed(dtype=2) == 2 and _dmixed(raw_dtype=2) == 2 and _dmixed(out_dtype=-1) == 2
    for call in (_cmixed, _dmixed):
        assert call(outer=-1) == 11 and call(inner=0) == 11 and call(channels=0) == 11
        assert call(channels=16385) == 11 and call(raw_channels=9) == 11 and call(raw_channels=-1) == 11
        assert call(outer=1 << 20, channels=4096, inner=1 << 10) == 6         # more than 2^31 elements
        assert call(slots=None) == 1 and call(raw=None) == 1
        assert call(slots=FAKE + 2) == 8 and call(raw=FAKE + 4) == 8
    assert _cmixed(x=None) == 1 and _cmixed(packed=None) == 1 and _cmixed(meta=None) == 1
    assert _cmixed(x=FAKE + 4) == 8 and _cmixed(meta=FAKE + 4) == 8
    n = 4 * 8 * 16
    assert _cmixed(packed_cap=api.packed_bytes(n, 4) - 1) == 7
    assert _cmixed(meta_cap=api.meta_bytes(n, 64) - 1) == 7
    assert _cmixed(raw_cap=4 * 2 * 16 * 4 - 1) == 7
    assert _dmixed(out=None) == 1 and _dmixed(out_cap=n * 4 - 1) == 7 and _dmixed(out_dtype=1, out_cap=n * 2 - 1) == 7
    # nothing to do: no pointer is looked at
    assert _cmixed(outer=0, x=None, packed=None, meta=None, raw=None, slots=None) == 0
    assert _dmixed(outer=0, packed=None, meta=None, raw=None, slots=None, out=None) == 0
    # no raw rows: raw may be NULL -- but this would launch, so only the check before it is probed
    assert _cmixed(raw_channels=0, raw=None, x=None) == 1


def test_channel_slots_rejects_bad_arguments_before_any_launch():
    f = api.raw_library().fh_channel_slots
    assert f(FAKE, 0, 0, FAKE, None) == 11 and f(FAKE, 16385, 0, FAKE, None) == 11
    assert f(FAKE, 8, 9, FAKE, None) == 11 and f(FAKE, 8, -1, FAKE, None) == 11
    assert f(None, 8, 2, FAKE, None) == 1 and f(FAKE, 8, 2, None, None) == 1
    assert f(FAKE, 8, 2, FAKE + 2, None) == 8


def test_raw_store_size():
    import torch
    assert api.raw_bytes(4, 3, 50, torch.float32) == 4 * 3 * 50 * 4
    assert api.raw_bytes(4, 3, 50, torch.bfloat16) == 4 * 3 * 50 * 2
    assert api.raw_bytes(0, 3, 50, torch.float32) == 0 and api.raw_bytes(4, 0, 50, torch.float32) == 0


def _sencode(x=FAKE, dtype=0, maps=4, h=10, w=10, n=4, tau=0.5, info=FAKE, info_cap=1 << 20, values=FAKE,
             values_cap=1 << 20, indices=FAKE, indices_cap=1 << 20, totals=FAKE, ws=FAKE, ws_cap=1 << 20):
    return api.raw_library().fh_sparse_encode(x, dtype, maps, h, w, n, tau, 0.0, info, info_cap, values, values_cap,
                                              indices, indices_cap, totals, ws, ws_cap, None)


def _sdecode(info=FAKE, values=FAKE, values_bytes=1 << 20, indices=FAKE, indices_bytes=1 << 20, dtype=0, maps=4,
             h=10, w=10, n=4, out=FAKE, out_cap=1 << 20, ws=FAKE, ws_cap=1 << 20):
    return api.raw_library().fh_sparse_decode(info, values, values_bytes, indices, indices_bytes, dtype, maps, h, w, n,
                                              0.0, out, out_cap, ws, ws_cap, None)


def test_sparse_calls_reject_bad_arguments_before_any_launch():
    for call in (_sencode, _sdecode):
        assert call(dtype=2) == 2
        assert call(n=3) == 12 and call(n=16) == 12 and call(n=0) == 12
        assert call(maps=-1) == 11 and call(h=0) == 11 and call(w=0) == 11
        assert call(maps=1 << 20, h=1 << 10, w=1 << 10) == 6              # more than 2^31 elements
        assert call(ws=None) == 1 and call(info=None) == 1
        assert call(ws=FAKE + 4) == 8
        assert call(ws_cap=23) == 7
    assert _sencode(x=None) == 1 and _sencode(values=None) == 1 and _sencode(indices=None) == 1
    assert _sencode(totals=None) == 1 and _sencode(totals=FAKE + 4) == 8 and _sencode(x=FAKE + 2) == 8
    assert _sencode(info_cap=4 * 9 - 1) == 7 and _sencode(values_cap=4 * 100 * 4 - 1) == 7
    assert _sencode(indices_cap=api.sparse_index_bytes(4, 10, 10, 4) - 1) == 7
    assert _sdecode(out=None) == 1 and _sdecode(out_cap=4 * 100 * 4 - 1) == 7 and _sdecode(out=FAKE + 2) == 8
    assert _sdecode(values=None) == 1 and _sdecode(indices=None) == 1
    assert _sdecode(maps=0, info=None, values=None, indices=None, out=None, ws=None) == 0


def test_sparse_size_helpers():
    # 4 maps of 10 x 10 with 4 x 4 windows: 3 x 3 blocks per map
    assert api.sparse_info_bytes(4, 10, 10, 4) == 36 == oracle.sparse_blocks(4, 10, 10, 4)
    assert api.sparse_index_bytes(4, 10, 10, 4) == 36 * 5 + 400
    assert api.sparse_workspace_bytes(4, 10, 10, 4) == 24
    assert api.sparse_workspace_bytes(1000, 16, 16, 2) == 24 * -(-64000 // 256)
    assert api.sparse_info_bytes(4, 10, 10, 3) == 0 and api.sparse_info_bytes(0, 10, 10, 4) == 0


def test_classify_item_layout_and_batch_argument_checks():
    # the C struct: pointer, two int32, three int64, double, int64, pointer + size, three pointers
    assert ctypes.sizeof(api.fh_classify_item) == 8 + 8 + 24 + 16 + 16 + 24 == 96
    assert api.fh_classify_item.outer.offset == 16 and api.fh_classify_item.k_sigma.offset == 40
    assert api.fh_classify_item.workspace.offset == 56 and api.fh_classify_item.mask.offset == 88
    assert api.classify_batch_capacity() == 16
    f = api.raw_library().fh_classify_channels_batch
    assert f(None, 0, None) == 0 and f(None, 1, None) == 1 and f(None, -1, None) == 10

    def item(**kw):
        it = api.fh_classify_item(FAKE, 0, 0, 4, 8, 16, 3.0, 1, FAKE, 1 << 20, FAKE, FAKE, FAKE)
        for k, v in kw.items():
            setattr(it, k, v)
        return it

    arr = (api.fh_classify_item * 3)(item(), item(), item(channels=0))
    assert f(arr, 3, None) == 11                             # the bad third item is found before any launch
    arr = (api.fh_classify_item * 2)(item(), item(k_sigma=-1.0))
    assert f(arr, 2, None) == 12
    arr = (api.fh_classify_item * 2)(item(x_dtype=5), item())
    assert f(arr, 2, None) == 2
    arr = (api.fh_classify_item * 1)(item(workspace_cap=8))
    assert f(arr, 1, None) == 7


def test_sparse_item_layouts_and_batch_argument_checks():
    assert ctypes.sizeof(api.fh_sparse_encode_item) == 8 + 8 + 24 + 8 + 6 * 8 + 8 + 16 == 120
    assert api.fh_sparse_encode_item.tau.offset == 40 and api.fh_sparse_encode_item.info.offset == 48
    assert api.fh_sparse_encode_item.totals.offset == 96 and api.fh_sparse_encode_item.workspace_cap.offset == 112
    assert ctypes.sizeof(api.fh_sparse_decode_item) == 5 * 8 + 8 + 24 + 8 + 4 * 8 == 112
    assert api.fh_sparse_decode_item.dtype.offset == 40 and api.fh_sparse_decode_item.eps.offset == 72
    assert api.fh_sparse_decode_item.out.offset == 80
    assert api.sparse_batch_capacity() == 16
    lib = api.raw_library()
    for f in (lib.fh_sparse_encode_batch, lib.fh_sparse_decode_batch):
        assert f(None, 0, None) == 0 and f(None, 2, None) == 1 and f(None, -1, None) == 10
    good = api.fh_sparse_encode_item(FAKE, 0, 4, 4, 10, 10, 0.5, 0.0, FAKE, 1 << 20, FAKE, 1 << 20, FAKE, 1 << 20,
                                     FAKE, FAKE, 1 << 20)
    bad = api.fh_sparse_encode_item(FAKE, 0, 3, 4, 10, 10, 0.5, 0.0, FAKE, 1 << 20, FAKE, 1 << 20, FAKE, 1 << 20,
                                    FAKE, FAKE, 1 << 20)
    arr = (api.fh_sparse_encode_item * 2)(good, bad)
    assert lib.fh_sparse_encode_batch(arr, 2, None) == 12          # found before any launch


def test_mixed_item_layout_and_batch_argument_checks():
    assert ctypes.sizeof(api.fh_mixed_item) == 16 + 24 + 16 + 3 * 16 + 8 + 16 + 32 + 8 == 168
    assert api.fh_mixed_item.rows_in_use.offset == 160
    assert api.fh_mixed_item.slots.offset == 40 and api.fh_mixed_item.raw_dtype.offset == 104
    assert api.fh_mixed_item.out.offset == 112 and api.fh_mixed_item.params.offset == 128
    assert api.mixed_batch_capacity() == 16
    lib = api.raw_library()
    for f in (lib.fh_compress_mixed_batch, lib.fh_decompress_mixed_batch):
        assert f(None, 0, None) == 0 and f(None, 2, None) == 1 and f(None, -1, None) == 10
    arr = (api.fh_mixed_item * 2)()
    for it in arr:
        it.x, it.outer, it.channels, it.inner, it.slots, it.raw_channels = FAKE, 4, 8, 16, FAKE, 2
        it.packed, it.packed_cap, it.meta, it.meta_cap, it.raw, it.raw_cap = FAKE, 1 << 20, FAKE, 1 << 20, FAKE, 1 << 20
        it.out, it.out_cap = FAKE, 1 << 20
        it.params = api.make_params(64, 4)
    arr[1].params.bits = 3
    assert lib.fh_compress_mixed_batch(arr, 2, None) == 4 and lib.fh_decompress_mixed_batch(arr, 2, None) == 4
    arr[1].params.bits = 4
    arr[1].raw_cap = 4 * 2 * 16 * 4 - 1
    assert lib.fh_compress_mixed_batch(arr, 2, None) == 7 and lib.fh_decompress_mixed_batch(arr, 2, None) == 7


def test_huffman_sizes_and_argument_checks():
    lib = api.raw_library()
    assert api.huffman_stream_bytes(0) == 256 + 4
    assert api.huffman_stream_bytes(1) == 256 + 8 + 768
    assert api.huffman_stream_bytes(257) == 256 + 12 + 2 * 768          # 256 symbols of 24 bits = 192 words a chunk
    assert api.huffman_workspace_bytes(0) == 4 * 513 and api.huffman_workspace_bytes(65537) == 4 * 514
    assert api.huffman_stream_bytes(1 << 32) == 0                       # n < 2^32
    fake = ctypes.c_void_p(0x10000)
    enc = lambda data, n, out, cap, tot, ws, wcap: lib.fh_huffman_encode(data, n, out, cap, tot, ws, wcap, None)
    assert enc(fake, 1 << 32, fake, 1 << 40, fake, fake, 1 << 20) == 6          # FH_ERR_BAD_NUMEL
    assert enc(None, 100, fake, 1 << 20, fake, fake, 1 << 20) == 1              # FH_ERR_NULL
    assert enc(fake, 100, fake, 1 << 20, None, fake, 1 << 20) == 1
    assert enc(ctypes.c_void_p(0x10004), 100, fake, 1 << 20, fake, fake, 1 << 20) == 8   # FH_ERR_ALIGNMENT
    assert enc(fake, 100, fake, 100, fake, fake, 1 << 20) == 7                  # FH_ERR_BUFFER_TOO_SMALL
    assert enc(fake, 100, fake, 1 << 20, fake, fake, 16) == 7
    dec = lambda s, sb, n, out, cap: lib.fh_huffman_decode(s, sb, n, out, cap, None)
    assert dec(None, 0, 0, None, 0) == 0                                        # nothing to restore
    assert dec(None, 1000, 10, fake, 10) == 1
    assert dec(fake, 1000, 10, fake, 9) == 7
    assert dec(fake, 200, 10, fake, 10) == 7                                    # not even the lengths and the offsets
    assert dec(fake, 1000, 1 << 32, fake, 1 << 33) == 6


def test_huffman_item_layouts_and_batch_argument_checks():
    assert ctypes.sizeof(api.fh_huffman_encode_item) == 64 and ctypes.sizeof(api.fh_huffman_decode_item) == 48
    assert api.fh_huffman_encode_item.n_device.offset == 56 and api.fh_huffman_decode_item.n_device.offset == 40
    assert api.fh_huffman_encode_item.workspace_cap.offset == 48 and api.fh_huffman_decode_item.out.offset == 24
    lib = api.raw_library()
    assert api.huffman_batch_capacity() == 16
    assert lib.fh_huffman_encode_batch(None, 0, None) == 0 and lib.fh_huffman_decode_batch(None, 0, None) == 0
    assert lib.fh_huffman_encode_batch(None, 2, None) == 1 and lib.fh_huffman_decode_batch(None, -1, None) != 0
    items = (api.fh_huffman_encode_item * 2)()
    for it in items:
        it.bytes = it.stream_out = it.totals = it.workspace = 0x10000
        it.n, it.stream_cap, it.workspace_cap = 100, 1 << 20, 1 << 20
    items[1].stream_cap = 10                                   # the second item is bad: nothing may be launched
    assert lib.fh_huffman_encode_batch(items, 2, None) == 7
    dec = (api.fh_huffman_decode_item * 1)()
    dec[0].stream_in = dec[0].out = 0x10000
    dec[0].n, dec[0].stream_bytes, dec[0].out_cap = 100, 100, 100
    assert lib.fh_huffman_decode_batch(dec, 1, None) == 7


def test_reserved_fields_must_be_zero():
    lib = api.raw_library()
    p = api.fh_params(256, 4, 0, 1, 0, 0)                      # reserved = 1
    assert lib.fh_compress(FAKE, 0, 1024, ctypes.byref(p), FAKE, 1 << 20, FAKE, 1 << 20, None) == 12
    assert lib.fh_decompress(FAKE, FAKE, 1024, ctypes.byref(p), 0, FAKE, 1 << 20, None) == 12
    assert lib.fh_roundtrip(FAKE, 0, 1024, ctypes.byref(p), FAKE, 1 << 20, FAKE, 1 << 20, 0, FAKE, 1 << 20, None) == 12
    it = api.fh_classify_item(FAKE, 0, 7, 4, 8, 16, 3.0, 1, FAKE, 1 << 20, FAKE, FAKE, FAKE)
    assert lib.fh_classify_channels_batch((api.fh_classify_item * 1)(it), 1, None) == 12
    arr = (api.fh_mixed_item * 1)()
    m = arr[0]
    m.x, m.outer, m.channels, m.inner, m.slots, m.raw_channels = FAKE, 4, 8, 16, FAKE, 2
    m.packed, m.packed_cap, m.meta, m.meta_cap, m.raw, m.raw_cap = FAKE, 1 << 20, FAKE, 1 << 20, FAKE, 1 << 20
    m.out, m.out_cap = FAKE, 1 << 20
    m.params = api.make_params(64, 4)
    m.reserved = 3
    assert lib.fh_compress_mixed_batch(arr, 1, None) == 12 and lib.fh_decompress_mixed_batch(arr, 1, None) == 12
    m.reserved = 0
    m.params.reserved = 1
    assert lib.fh_compress_mixed_batch(arr, 1, None) == 12 and lib.fh_decompress_mixed_batch(arr, 1, None) == 12
    dec = (api.fh_sparse_decode_item * 1)()
    d = dec[0]
    d.info = d.values = d.indices = d.out = d.workspace = FAKE
    d.values_bytes = d.indices_bytes = d.out_cap = d.workspace_cap = 1 << 20
    d.dtype, d.n, d.maps, d.h, d.w, d.eps, d.reserved = 0, 4, 4, 10, 10, 0.0, 9
    assert lib.fh_sparse_decode_batch(dec, 1, None) == 12


def test_static_scratch_entry_point_refuses_oversized_tensors_on_the_host():
    lib = api.raw_library()
    limit = api.classify_static_scratch_bytes()
    assert limit == 4 << 20
    n_ok = 261_887 * 1024                        # 261887 + 256 + 1 partial-sum pairs of 16 bytes = 4 MiB
    assert api.classify_workspace_bytes(n_ok) == limit < api.classify_workspace_bytes(n_ok + 1)
    # refused before the device is even asked for the buffer's address (no GPU needed here)
    assert lib.fh_classify_channels_static(FAKE, 0, 1, 1, n_ok + 1, 3.0, 1, FAKE, FAKE, FAKE, None) == 13
    assert lib.fh_classify_channels_static(FAKE, 0, 4, 1024, 1 << 20, 3.0, 1, FAKE, FAKE, FAKE, None) == 13
    assert "static buffer" in api.status_string(13)


def test_mix_item_layout_and_host_side_layout_call():
    assert ctypes.sizeof(api.fh_mix_item) == 192 and api.fh_mix_item.quant.offset == 64
    assert api.fh_mix_item.k_sigma.offset == 96 and api.fh_mix_item.window.offset == 120
    assert api.fh_mix_item.store.offset == 144 and api.fh_mix_item.out_cap.offset == 184
    assert ctypes.sizeof(api.fh_mix_regions) == 8 * len(api.MIX_REGION_FIELDS) == 232
    it = api.fh_mix_item()
    it.x_dtype = 0
    it.outer, it.channels, it.inner = 8, 32, 196
    it.maps, it.h, it.w = 32, 14, 14
    it.quant = api.make_params(128, 4)
    it.k_sigma, it.min_outliers, it.raw_channels = 3.0, 1, 4
    it.window, it.entropy, it.tau, it.eps = 4, 1, 0.5, 0.02
    r = api.mix_layout(it)
    n = 8 * 32 * 196
    assert r.packed_bytes == api.packed_bytes(n, 4) and r.meta_bytes == api.meta_bytes(n, 128)
    assert r.raw_bytes == 8 * 4 * 196 * 4 == r.values_cap and r.slots_bytes == 64
    assert r.info_bytes == api.sparse_info_bytes(32, 14, 14, 4) and r.indices_cap == api.sparse_index_bytes(32, 14, 14, 4)
    assert r.huffman_cap == api.huffman_stream_bytes(r.indices_cap) and r.indices == 0 and r.huffman > r.values
    offs = [r.header, r.slots, r.packed, r.meta, r.info, r.values, r.huffman]
    assert offs == sorted(offs) and all(o % 256 == 0 for o in offs) and r.store_bytes % 256 == 0
    assert r.store_bytes >= r.huffman + r.huffman_cap
    it.entropy = 0
    r0 = api.mix_layout(it)
    assert r0.huffman_cap == 0 and r0.indices > r0.values and r0.store_bytes < r.store_bytes
    it.raw_channels = 0
    r1 = api.mix_layout(it)
    assert r1.raw_bytes == r1.info_bytes == r1.values_cap == r1.indices_cap == 0
    lib = api.raw_library()
    it.raw_channels, it.maps = 4, 31
    assert lib.fh_mix_layout(ctypes.byref(it), ctypes.byref(r)) == 11
    assert lib.fh_mix_compress(None, None) == 1 and lib.fh_mix_compress_batch(None, -1, None) == 10
    assert lib.fh_mix_compress_batch(None, 0, None) == 0 and lib.fh_mix_decompress_batch(None, 2, None) == 1
