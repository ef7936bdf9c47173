"""ctypes access to the CPU oracle (`fho.c`).

TEST INFRASTRUCTURE ONLY: the oracle defines the expected result of the group
quantiser (FedHybrid Section 4.4.1, normal-channel quantisation; Section 3,
compress in forward / decompress in backward).  Only the tests, the smoke check
and the benchmark's CPU-baseline leg import this package.  It neither imports nor
is imported by the HIP package.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "libfho.so")
_SRCS = [os.path.join(_HERE, n) for n in ("fho.c", "fho_classify.c", "fho_mixed.c", "fho_sparse.c", "fho_huffman.c")]

F32, BF16 = 0, 1
NEAREST, STOCHASTIC = 0, 1

_DTYPES = {"f32": F32, "bf16": BF16, F32: F32, BF16: BF16}
_ROUNDS = {"nearest": NEAREST, "stochastic": STOCHASTIC, NEAREST: NEAREST, STOCHASTIC: STOCHASTIC}


def build(force: bool = True) -> str:
    """Compile fho.c into libfho.so with gcc (strict binary32 semantics: no
    contraction, no fast-math)."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < max(os.path.getmtime(p) for p in _SRCS):
        cmd = ["gcc", "-std=c11", "-O2", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared",
               "-Wall", "-Wextra", "-o", _SO, *_SRCS, "-lm"]
        subprocess.run(cmd, check=True, cwd=_HERE)
    return _SO


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        build(force=False)
        L = ctypes.CDLL(_SO)
        u32p = ctypes.POINTER(ctypes.c_uint32)
        L.fho_philox4x32_10.argtypes = [u32p, u32p, u32p]
        L.fho_philox4x32_10.restype = None
        L.fho_random16.argtypes = [ctypes.c_uint64, ctypes.c_uint64, ctypes.c_uint64]
        L.fho_random16.restype = ctypes.c_uint32
        L.fho_packed_bytes.argtypes = [ctypes.c_int64, ctypes.c_int]
        L.fho_packed_bytes.restype = ctypes.c_size_t
        L.fho_meta_bytes.argtypes = [ctypes.c_int64, ctypes.c_int]
        L.fho_meta_bytes.restype = ctypes.c_size_t
        L.fho_compress.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_int, ctypes.c_int,
                                   ctypes.c_int, ctypes.c_uint64, ctypes.c_uint64,
                                   ctypes.c_void_p, ctypes.c_void_p]
        L.fho_compress.restype = ctypes.c_int
        L.fho_decompress.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_int,
                                     ctypes.c_int, ctypes.c_int, ctypes.c_void_p]
        L.fho_decompress.restype = ctypes.c_int
        L.fho_unpack_codes.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_void_p]
        L.fho_unpack_codes.restype = ctypes.c_int
        dp = ctypes.POINTER(ctypes.c_double)
        L.fho_pairwise_moments.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, dp, dp]
        L.fho_pairwise_moments.restype = None
        L.fho_classify_channels.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_int64,
                                            ctypes.c_int64, ctypes.c_double, ctypes.c_int64,
                                            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
        L.fho_classify_channels.restype = ctypes.c_int
        L.fho_channel_slots.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_void_p]
        L.fho_channel_slots.restype = ctypes.c_int64
        L.fho_compress_mixed.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_int64,
                                         ctypes.c_int64, ctypes.c_void_p, ctypes.c_int64,
                                         ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_uint64,
                                         ctypes.c_uint64, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
        L.fho_compress_mixed.restype = ctypes.c_int
        L.fho_decompress_mixed.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int,
                                           ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
                                           ctypes.c_void_p, ctypes.c_int64,
                                           ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_void_p]
        L.fho_decompress_mixed.restype = ctypes.c_int
        L.fho_sparse_blocks.argtypes = [ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_int]
        L.fho_sparse_blocks.restype = ctypes.c_int64
        L.fho_sparse_encode.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
                                        ctypes.c_int, ctypes.c_float, ctypes.c_float, ctypes.c_void_p, ctypes.c_void_p,
                                        ctypes.c_void_p, ctypes.c_void_p]
        L.fho_sparse_encode.restype = ctypes.c_int
        L.fho_sparse_decode.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int,
                                        ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_int, ctypes.c_float,
                                        ctypes.c_void_p]
        L.fho_sparse_decode.restype = ctypes.c_int
        L.fho_huffman_lengths.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
        L.fho_huffman_lengths.restype = None
        L.fho_huffman_codes.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
        L.fho_huffman_codes.restype = None
        L.fho_huffman_stream_bytes.argtypes = [ctypes.c_uint64]
        L.fho_huffman_stream_bytes.restype = ctypes.c_size_t
        L.fho_huffman_encode.argtypes = [ctypes.c_void_p, ctypes.c_uint64, ctypes.c_void_p, ctypes.c_void_p]
        L.fho_huffman_encode.restype = ctypes.c_int
        L.fho_huffman_decode.argtypes = [ctypes.c_void_p, ctypes.c_uint64, ctypes.c_uint64, ctypes.c_void_p]
        L.fho_huffman_decode.restype = ctypes.c_int
        _lib = L
    return _lib


def philox4x32_10(ctr, key) -> Tuple[int, int, int, int]:
    c = (ctypes.c_uint32 * 4)(*[int(v) & 0xFFFFFFFF for v in ctr])
    k = (ctypes.c_uint32 * 2)(*[int(v) & 0xFFFFFFFF for v in key])
    o = (ctypes.c_uint32 * 4)()
    lib().fho_philox4x32_10(c, k, o)
    return tuple(int(v) for v in o)


def random16(seed: int, tensor_id: int, index: int) -> int:
    return int(lib().fho_random16(seed, tensor_id, index))


def packed_bytes(numel: int, bits: int) -> int:
    return int(lib().fho_packed_bytes(numel, bits))


def meta_bytes(numel: int, group_size: int) -> int:
    return int(lib().fho_meta_bytes(numel, group_size))


def _check_input(x: np.ndarray, dtype) -> int:
    d = _DTYPES[dtype]
    want = np.float32 if d == F32 else np.uint16
    if x.dtype != want or not x.flags.c_contiguous:
        raise TypeError(f"expected C-contiguous {want.__name__} array for dtype {dtype!r}")
    return d


def compress(x: np.ndarray, group_size: int, bits: int, rounding="nearest", seed: int = 0,
             tensor_id: int = 0, dtype="f32") -> Tuple[np.ndarray, np.ndarray]:
    """-> (packed uint8[packed_bytes], meta float32[n_groups, 2] = {scale, zero})."""
    d = _check_input(x, dtype)
    n = int(x.size)
    packed = np.empty(packed_bytes(n, bits), dtype=np.uint8)
    meta = np.empty((meta_bytes(n, group_size) // 8, 2), dtype=np.float32)
    rc = lib().fho_compress(x.ctypes.data, d, n, group_size, bits, _ROUNDS[rounding], seed, tensor_id,
                            packed.ctypes.data, meta.ctypes.data)
    if rc != 0:
        raise ValueError("fho_compress rejected its arguments")
    return packed, meta


def decompress(packed: np.ndarray, meta: np.ndarray, numel: int, group_size: int, bits: int,
               out_dtype="f32") -> np.ndarray:
    """-> float32[numel], or uint16[numel] bf16 bit patterns."""
    d = _DTYPES[out_dtype]
    out = np.empty(numel, dtype=np.float32 if d == F32 else np.uint16)
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    meta = np.ascontiguousarray(meta, dtype=np.float32)
    rc = lib().fho_decompress(packed.ctypes.data, meta.ctypes.data, int(numel), group_size, bits, d,
                              out.ctypes.data)
    if rc != 0:
        raise ValueError("fho_decompress rejected its arguments")
    return out


def unpack_codes(packed: np.ndarray, numel: int, bits: int) -> np.ndarray:
    codes = np.empty(numel, dtype=np.uint8)
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    rc = lib().fho_unpack_codes(packed.ctypes.data, int(numel), bits, codes.ctypes.data)
    if rc != 0:
        raise ValueError("fho_unpack_codes rejected its arguments")
    return codes


def pairwise_moments(x: np.ndarray, dtype="f32") -> Tuple[float, float]:
    """Pairwise binary64 sums (sum x, sum x*x) in element order."""
    d = _check_input(x, dtype)
    s1, s2 = ctypes.c_double(), ctypes.c_double()
    lib().fho_pairwise_moments(x.ctypes.data, d, int(x.size), ctypes.byref(s1), ctypes.byref(s2))
    return s1.value, s2.value


def classify_channels(x: np.ndarray, outer: int, channels: int, inner: int, k_sigma: float = 3.0,
                      min_outliers: int = 1, dtype="f32"):
    """-> (stats float64[4] = {mean, variance, threshold, numel}, counts uint32[C], mask uint8[C])."""
    d = _check_input(x, dtype)
    if x.size != outer * channels * inner:
        raise ValueError("x.size != outer * channels * inner")
    stats = np.zeros(4, dtype=np.float64)
    counts = np.zeros(channels, dtype=np.uint32)
    mask = np.zeros(channels, dtype=np.uint8)
    rc = lib().fho_classify_channels(x.ctypes.data, d, outer, channels, inner, float(k_sigma), int(min_outliers),
                                     stats.ctypes.data, counts.ctypes.data, mask.ctypes.data)
    if rc != 0:
        raise ValueError("fho_classify_channels rejected its arguments")
    return stats, counts, mask


def channel_slots(mask: np.ndarray, raw_channels: int) -> Tuple[np.ndarray, int]:
    """-> (slots int16[C]: raw-store row of each kept salient channel, -1 otherwise; slots used)."""
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    slots = np.empty(mask.size, dtype=np.int16)
    used = lib().fho_channel_slots(mask.ctypes.data, int(mask.size), int(raw_channels), slots.ctypes.data)
    if used < 0:
        raise ValueError("fho_channel_slots rejected its arguments")
    return slots, int(used)


def compress_mixed(x: np.ndarray, outer: int, channels: int, inner: int, slots: np.ndarray, raw_channels: int,
                   group_size: int, bits: int, rounding="nearest", seed: int = 0, tensor_id: int = 0,
                   dtype="f32", raw_fill=0):
    """-> (packed, meta[n_groups, 2], raw[outer * raw_channels * inner] in x's dtype; rows of
    unused slots keep `raw_fill`)."""
    d = _check_input(x, dtype)
    n = outer * channels * inner
    if x.size != n:
        raise ValueError("x.size != outer * channels * inner")
    slots = np.ascontiguousarray(slots, dtype=np.int16)
    packed = np.empty(packed_bytes(n, bits), dtype=np.uint8)
    meta = np.empty((meta_bytes(n, group_size) // 8, 2), dtype=np.float32)
    raw = np.full(outer * raw_channels * inner, raw_fill, dtype=x.dtype)
    rc = lib().fho_compress_mixed(x.ctypes.data, d, outer, channels, inner, slots.ctypes.data, int(raw_channels),
                                  group_size, bits, _ROUNDS[rounding], seed, tensor_id,
                                  packed.ctypes.data, meta.ctypes.data, raw.ctypes.data)
    if rc != 0:
        raise ValueError("fho_compress_mixed rejected its arguments")
    return packed, meta, raw


def decompress_mixed(packed: np.ndarray, meta: np.ndarray, raw: np.ndarray, outer: int, channels: int, inner: int,
                     slots: np.ndarray, raw_channels: int, group_size: int, bits: int,
                     raw_dtype="f32", out_dtype="f32") -> np.ndarray:
    rd = _check_input(raw, raw_dtype) if raw.size else _DTYPES[raw_dtype]
    od = _DTYPES[out_dtype]
    n = outer * channels * inner
    out = np.empty(n, dtype=np.float32 if od == F32 else np.uint16)
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    meta = np.ascontiguousarray(meta, dtype=np.float32)
    slots = np.ascontiguousarray(slots, dtype=np.int16)
    rc = lib().fho_decompress_mixed(packed.ctypes.data, meta.ctypes.data, raw.ctypes.data, rd,
                                    outer, channels, inner, slots.ctypes.data, int(raw_channels),
                                    group_size, bits, od, out.ctypes.data)
    if rc != 0:
        raise ValueError("fho_decompress_mixed rejected its arguments")
    return out


def sparse_blocks(maps: int, h: int, w: int, n: int) -> int:
    return int(lib().fho_sparse_blocks(maps, h, w, n))


def sparse_encode(x: np.ndarray, maps: int, h: int, w: int, n: int, tau: float, dtype="f32", eps: float = 0.0):
    """-> (info uint8[blocks], values (trimmed to what was written), indices uint8 (trimmed),
    totals uint64[4] = {values, index bytes, sparse blocks, dense blocks}).  eps > 0 stores
    dense blocks by Lorenzo prediction within that error bound."""
    d = _check_input(x, dtype)
    if x.size != maps * h * w:
        raise ValueError("x.size != maps * h * w")
    nb = sparse_blocks(maps, h, w, n)
    if nb < 0:
        raise ValueError("bad shape")
    info = np.zeros(nb, dtype=np.uint8)
    values = np.zeros(max(1, x.size), dtype=x.dtype)
    indices = np.zeros(max(1, nb * (n + 1) + x.size), dtype=np.uint8)
    totals = np.zeros(4, dtype=np.uint64)
    rc = lib().fho_sparse_encode(x.ctypes.data, d, maps, h, w, n, float(tau), float(eps), info.ctypes.data,
                                 values.ctypes.data, indices.ctypes.data, totals.ctypes.data)
    if rc != 0:
        raise ValueError("fho_sparse_encode rejected its arguments")
    return info, values[:int(totals[0])].copy(), indices[:int(totals[1])].copy(), totals


def sparse_decode(info: np.ndarray, values: np.ndarray, indices: np.ndarray, maps: int, h: int, w: int, n: int,
                  dtype="f32", eps: float = 0.0) -> np.ndarray:
    d = _DTYPES[dtype]
    out = np.empty(maps * h * w, dtype=np.float32 if d == F32 else np.uint16)
    info = np.ascontiguousarray(info, dtype=np.uint8)
    values = np.ascontiguousarray(np.concatenate([values, np.zeros(1, values.dtype)]))
    indices = np.ascontiguousarray(np.concatenate([indices.astype(np.uint8), np.zeros(1, np.uint8)]))
    rc = lib().fho_sparse_decode(info.ctypes.data, values.ctypes.data, indices.ctypes.data, d, maps, h, w, n,
                                 float(eps), out.ctypes.data)
    if rc != 0:
        raise ValueError(f"fho_sparse_decode failed ({rc})")
    return out


def huffman_lengths(hist) -> np.ndarray:
    """Code length of every byte value for the histogram `hist` (256 counts) -> uint8[256]."""
    h = np.ascontiguousarray(hist, dtype=np.uint64)
    if h.size != 256:
        raise ValueError("a histogram has 256 counts")
    out = np.zeros(256, dtype=np.uint8)
    lib().fho_huffman_lengths(h.ctypes.data, out.ctypes.data)
    return out


def huffman_codes(lengths) -> np.ndarray:
    """Canonical codes for the lengths -> uint32[256] (0 where the length is 0)."""
    l = np.ascontiguousarray(lengths, dtype=np.uint8)
    out = np.zeros(256, dtype=np.uint32)
    lib().fho_huffman_codes(l.ctypes.data, out.ctypes.data)
    return out


def huffman_encode(data: np.ndarray):
    """-> (stream uint8[used], payload bits)."""
    d = np.ascontiguousarray(data, dtype=np.uint8).reshape(-1)
    stream = np.zeros(lib().fho_huffman_stream_bytes(d.size), dtype=np.uint8)
    totals = np.zeros(2, dtype=np.uint64)
    if lib().fho_huffman_encode(d.ctypes.data, d.size, stream.ctypes.data, totals.ctypes.data) != 0:
        raise ValueError("fho_huffman_encode rejected its arguments")
    return stream[: int(totals[0])].copy(), int(totals[1])


def huffman_decode(stream: np.ndarray, n: int) -> np.ndarray:
    s = np.ascontiguousarray(stream, dtype=np.uint8).reshape(-1)
    out = np.zeros(n, dtype=np.uint8)
    rc = lib().fho_huffman_decode(s.ctypes.data, s.size, n, out.ctypes.data)
    if rc != 0:
        raise ValueError(f"fho_huffman_decode failed ({rc})")
    return out
