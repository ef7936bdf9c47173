"""Thin ctypes binding over libfedhybrid.so: argument marshalling only.

Every step of the method runs in the HIP kernels behind the C ABI declared in
include/fedhybrid.h (FedHybrid Section 3: compress in the forward pass, decompress in
the backward pass; Section 4.4.1: linear-scale quantisation of normal channels).
PyTorch supplies device memory and the current HIP stream, nothing else.  There is
no CPU fallback: if the library is missing, importing this module raises.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import List, Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libfedhybrid.so")

if not os.path.exists(_LIB_PATH):
    raise ImportError(
        f"{_LIB_PATH} is missing: build it with `python -m paper_2510_11400_amd.build` "
        "(hipcc, gfx950). There is no fallback implementation.")

_lib = ctypes.CDLL(_LIB_PATH)

FH_F32, FH_BF16 = 0, 1
FH_ROUND_NEAREST, FH_ROUND_STOCHASTIC = 0, 1

EXPORTS = ("fh_packed_bytes", "fh_meta_bytes", "fh_compress", "fh_decompress", "fh_roundtrip",
           "fh_compress_batch", "fh_decompress_batch", "fh_roundtrip_batch", "fh_batch_capacity",
           "fh_classify_workspace_bytes", "fh_classify_channels", "fh_classify_channels_batch",
           "fh_classify_batch_capacity", "fh_classify_static_scratch_bytes", "fh_classify_channels_static",
           "fh_raw_bytes", "fh_channel_slots", "fh_channel_slots_used", "fh_channel_slots_batch", "fh_compress_mixed", "fh_decompress_mixed",
           "fh_compress_mixed_batch", "fh_decompress_mixed_batch", "fh_mixed_batch_capacity",
           "fh_sparse_info_bytes", "fh_sparse_index_bytes", "fh_sparse_workspace_bytes", "fh_sparse_encode",
           "fh_sparse_decode", "fh_sparse_encode_batch", "fh_sparse_decode_batch", "fh_sparse_batch_capacity",
           "fh_huffman_stream_bytes", "fh_huffman_workspace_bytes", "fh_huffman_encode", "fh_huffman_decode",
           "fh_huffman_encode_batch", "fh_huffman_decode_batch", "fh_huffman_batch_capacity",
           "fh_mix_layout", "fh_mix_compress", "fh_mix_decompress", "fh_mix_compress_batch", "fh_mix_decompress_batch",
           "fh_status_string")


class fh_params(ctypes.Structure):
    _fields_ = [("group_size", ctypes.c_int32), ("bits", ctypes.c_int32), ("rounding", ctypes.c_int32),
                ("reserved", ctypes.c_int32), ("seed", ctypes.c_uint64), ("tensor_id", ctypes.c_uint64)]


class fh_item(ctypes.Structure):
    _fields_ = [("x", ctypes.c_void_p), ("x_dtype", ctypes.c_int32), ("out_dtype", ctypes.c_int32),
                ("numel", ctypes.c_int64),
                ("packed", ctypes.c_void_p), ("packed_cap", ctypes.c_size_t),
                ("meta", ctypes.c_void_p), ("meta_cap", ctypes.c_size_t),
                ("out", ctypes.c_void_p), ("out_cap", ctypes.c_size_t),
                ("params", fh_params)]


class fh_classify_item(ctypes.Structure):
    _fields_ = [("x", ctypes.c_void_p), ("x_dtype", ctypes.c_int32), ("reserved", ctypes.c_int32),
                ("outer", ctypes.c_int64), ("channels", ctypes.c_int64), ("inner", ctypes.c_int64),
                ("k_sigma", ctypes.c_double), ("min_outliers", ctypes.c_int64),
                ("workspace", ctypes.c_void_p), ("workspace_cap", ctypes.c_size_t),
                ("stats", ctypes.c_void_p), ("counts", ctypes.c_void_p), ("mask", ctypes.c_void_p)]


class fh_mixed_item(ctypes.Structure):
    _fields_ = [("x", ctypes.c_void_p), ("x_dtype", ctypes.c_int32), ("out_dtype", ctypes.c_int32),
                ("outer", ctypes.c_int64), ("channels", ctypes.c_int64), ("inner", ctypes.c_int64),
                ("slots", ctypes.c_void_p), ("raw_channels", ctypes.c_int64),
                ("packed", ctypes.c_void_p), ("packed_cap", ctypes.c_size_t),
                ("meta", ctypes.c_void_p), ("meta_cap", ctypes.c_size_t),
                ("raw", ctypes.c_void_p), ("raw_cap", ctypes.c_size_t),
                ("raw_dtype", ctypes.c_int32), ("reserved", ctypes.c_int32),
                ("out", ctypes.c_void_p), ("out_cap", ctypes.c_size_t),
                ("params", fh_params), ("rows_in_use", ctypes.c_void_p)]


class fh_slots_item(ctypes.Structure):
    _fields_ = [("mask", ctypes.c_void_p), ("channels", ctypes.c_int64), ("raw_channels", ctypes.c_int64),
                ("slots", ctypes.c_void_p), ("used", ctypes.c_void_p)]


class fh_sparse_encode_item(ctypes.Structure):
    _fields_ = [("x", ctypes.c_void_p), ("dtype", ctypes.c_int32), ("n", ctypes.c_int32),
                ("maps", ctypes.c_int64), ("h", ctypes.c_int64), ("w", ctypes.c_int64),
                ("tau", ctypes.c_float), ("eps", ctypes.c_float),
                ("info", ctypes.c_void_p), ("info_cap", ctypes.c_size_t),
                ("values", ctypes.c_void_p), ("values_cap", ctypes.c_size_t),
                ("indices", ctypes.c_void_p), ("indices_cap", ctypes.c_size_t),
                ("totals", ctypes.c_void_p), ("workspace", ctypes.c_void_p), ("workspace_cap", ctypes.c_size_t)]


class fh_sparse_decode_item(ctypes.Structure):
    _fields_ = [("info", ctypes.c_void_p), ("values", ctypes.c_void_p), ("values_bytes", ctypes.c_size_t),
                ("indices", ctypes.c_void_p), ("indices_bytes", ctypes.c_size_t),
                ("dtype", ctypes.c_int32), ("n", ctypes.c_int32),
                ("maps", ctypes.c_int64), ("h", ctypes.c_int64), ("w", ctypes.c_int64),
                ("eps", ctypes.c_float), ("reserved", ctypes.c_int32),
                ("out", ctypes.c_void_p), ("out_cap", ctypes.c_size_t),
                ("workspace", ctypes.c_void_p), ("workspace_cap", ctypes.c_size_t)]


_P = ctypes.POINTER
_lib.fh_packed_bytes.argtypes = [ctypes.c_int64, ctypes.c_int32]
_lib.fh_packed_bytes.restype = ctypes.c_size_t
_lib.fh_meta_bytes.argtypes = [ctypes.c_int64, ctypes.c_int32]
_lib.fh_meta_bytes.restype = ctypes.c_size_t
_lib.fh_compress.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, _P(fh_params),
                             ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
_lib.fh_compress.restype = ctypes.c_int
_lib.fh_decompress.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, _P(fh_params),
                               ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
_lib.fh_decompress.restype = ctypes.c_int
_lib.fh_roundtrip.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, _P(fh_params),
                              ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_size_t,
                              ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
_lib.fh_roundtrip.restype = ctypes.c_int
for _name in ("fh_compress_batch", "fh_decompress_batch", "fh_roundtrip_batch"):
    getattr(_lib, _name).argtypes = [_P(fh_item), ctypes.c_int32, ctypes.c_void_p]
    getattr(_lib, _name).restype = ctypes.c_int
_lib.fh_classify_workspace_bytes.argtypes = [ctypes.c_int64]
_lib.fh_classify_workspace_bytes.restype = ctypes.c_size_t
_lib.fh_classify_channels.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
                                      ctypes.c_double, ctypes.c_int64, ctypes.c_void_p, ctypes.c_size_t,
                                      ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
_lib.fh_classify_channels.restype = ctypes.c_int
_lib.fh_classify_static_scratch_bytes.argtypes = []
_lib.fh_classify_static_scratch_bytes.restype = ctypes.c_size_t
_lib.fh_classify_channels_static.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_int64,
                                             ctypes.c_int64, ctypes.c_double, ctypes.c_int64,
                                             ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
_lib.fh_classify_channels_static.restype = ctypes.c_int
_lib.fh_classify_channels_batch.argtypes = [_P(fh_classify_item), ctypes.c_int32, ctypes.c_void_p]
_lib.fh_classify_channels_batch.restype = ctypes.c_int
_lib.fh_classify_batch_capacity.argtypes = []
_lib.fh_classify_batch_capacity.restype = ctypes.c_int32
_lib.fh_raw_bytes.argtypes = [ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_int]
_lib.fh_raw_bytes.restype = ctypes.c_size_t
_lib.fh_channel_slots.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p]
_lib.fh_channel_slots.restype = ctypes.c_int
_lib.fh_channel_slots_used.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p,
                                       ctypes.c_void_p]
_lib.fh_channel_slots_used.restype = ctypes.c_int
_lib.fh_channel_slots_batch.argtypes = [_P(fh_slots_item), ctypes.c_int32, ctypes.c_void_p]
_lib.fh_channel_slots_batch.restype = ctypes.c_int
_lib.fh_compress_mixed.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
                                   _P(fh_params), ctypes.c_void_p, ctypes.c_int64,
                                   ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_size_t,
                                   ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
_lib.fh_compress_mixed.restype = ctypes.c_int
_lib.fh_decompress_mixed.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int,
                                     ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
                                     _P(fh_params), ctypes.c_void_p, ctypes.c_int64,
                                     ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
_lib.fh_decompress_mixed.restype = ctypes.c_int
for _name in ("fh_sparse_info_bytes", "fh_sparse_index_bytes", "fh_sparse_workspace_bytes"):
    getattr(_lib, _name).argtypes = [ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_int32]
    getattr(_lib, _name).restype = ctypes.c_size_t
_lib.fh_sparse_encode.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
                                  ctypes.c_int32, ctypes.c_float, ctypes.c_float, ctypes.c_void_p, ctypes.c_size_t,
                                  ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_size_t,
                                  ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
_lib.fh_sparse_encode.restype = ctypes.c_int
_lib.fh_sparse_decode.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_size_t,
                                  ctypes.c_int, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_int32,
                                  ctypes.c_float,
                                  ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
_lib.fh_sparse_decode.restype = ctypes.c_int
for _name in ("fh_compress_mixed_batch", "fh_decompress_mixed_batch"):
    getattr(_lib, _name).argtypes = [_P(fh_mixed_item), ctypes.c_int32, ctypes.c_void_p]
    getattr(_lib, _name).restype = ctypes.c_int
_lib.fh_mixed_batch_capacity.argtypes = []
_lib.fh_mixed_batch_capacity.restype = ctypes.c_int32
_lib.fh_sparse_encode_batch.argtypes = [_P(fh_sparse_encode_item), ctypes.c_int32, ctypes.c_void_p]
_lib.fh_sparse_encode_batch.restype = ctypes.c_int
_lib.fh_sparse_decode_batch.argtypes = [_P(fh_sparse_decode_item), ctypes.c_int32, ctypes.c_void_p]
_lib.fh_sparse_decode_batch.restype = ctypes.c_int
_lib.fh_sparse_batch_capacity.argtypes = []
_lib.fh_sparse_batch_capacity.restype = ctypes.c_int32
_lib.fh_batch_capacity.argtypes = []
_lib.fh_batch_capacity.restype = ctypes.c_int32
for _name in ("fh_huffman_stream_bytes", "fh_huffman_workspace_bytes"):
    getattr(_lib, _name).argtypes = [ctypes.c_uint64]
    getattr(_lib, _name).restype = ctypes.c_size_t
_lib.fh_huffman_encode.argtypes = [ctypes.c_void_p, ctypes.c_uint64, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p,
                                   ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
_lib.fh_huffman_encode.restype = ctypes.c_int
_lib.fh_huffman_decode.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_uint64, ctypes.c_void_p, ctypes.c_size_t,
                                   ctypes.c_void_p]
_lib.fh_huffman_decode.restype = ctypes.c_int
_lib.fh_status_string.argtypes = [ctypes.c_int]
_lib.fh_status_string.restype = ctypes.c_char_p


class fh_huffman_encode_item(ctypes.Structure):
    _fields_ = [("bytes", ctypes.c_void_p), ("n", ctypes.c_uint64),
                ("stream_out", ctypes.c_void_p), ("stream_cap", ctypes.c_size_t),
                ("totals", ctypes.c_void_p),
                ("workspace", ctypes.c_void_p), ("workspace_cap", ctypes.c_size_t),
                ("n_device", ctypes.c_void_p)]


class fh_huffman_decode_item(ctypes.Structure):
    _fields_ = [("stream_in", ctypes.c_void_p), ("stream_bytes", ctypes.c_size_t), ("n", ctypes.c_uint64),
                ("out", ctypes.c_void_p), ("out_cap", ctypes.c_size_t), ("n_device", ctypes.c_void_p)]


_lib.fh_huffman_encode_batch.argtypes = [_P(fh_huffman_encode_item), ctypes.c_int32, ctypes.c_void_p]
_lib.fh_huffman_encode_batch.restype = ctypes.c_int
_lib.fh_huffman_decode_batch.argtypes = [_P(fh_huffman_decode_item), ctypes.c_int32, ctypes.c_void_p]
_lib.fh_huffman_decode_batch.restype = ctypes.c_int
_lib.fh_huffman_batch_capacity.argtypes = []
_lib.fh_huffman_batch_capacity.restype = ctypes.c_int32


class fh_mix_item(ctypes.Structure):
    _fields_ = [("x", ctypes.c_void_p), ("x_dtype", ctypes.c_int32), ("out_dtype", ctypes.c_int32),
                ("outer", ctypes.c_int64), ("channels", ctypes.c_int64), ("inner", ctypes.c_int64),
                ("maps", ctypes.c_int64), ("h", ctypes.c_int64), ("w", ctypes.c_int64),
                ("quant", fh_params),
                ("k_sigma", ctypes.c_double), ("min_outliers", ctypes.c_int64),
                ("raw_channels", ctypes.c_int64),
                ("window", ctypes.c_int32), ("entropy", ctypes.c_int32),
                ("tau", ctypes.c_float), ("eps", ctypes.c_float),
                ("reserved", ctypes.c_int64),
                ("store", ctypes.c_void_p), ("store_cap", ctypes.c_size_t),
                ("workspace", ctypes.c_void_p), ("workspace_cap", ctypes.c_size_t),
                ("out", ctypes.c_void_p), ("out_cap", ctypes.c_size_t)]


MIX_REGION_FIELDS = ("store_bytes", "workspace_bytes",
                     "header", "slots", "packed", "meta", "info", "values", "indices", "huffman",
                     "stats", "counts", "mask", "classify_ws", "raw", "sparse_ws", "indices_ws", "huffman_ws",
                     "slots_bytes", "packed_bytes", "meta_bytes", "info_bytes", "values_cap", "indices_cap",
                     "huffman_cap", "raw_bytes", "classify_ws_bytes", "sparse_ws_bytes", "huffman_ws_bytes")


class fh_mix_regions(ctypes.Structure):
    _fields_ = [(name, ctypes.c_size_t) for name in MIX_REGION_FIELDS]


_lib.fh_mix_layout.argtypes = [_P(fh_mix_item), _P(fh_mix_regions)]
_lib.fh_mix_layout.restype = ctypes.c_int
for _name in ("fh_mix_compress", "fh_mix_decompress"):
    getattr(_lib, _name).argtypes = [_P(fh_mix_item), ctypes.c_void_p]
    getattr(_lib, _name).restype = ctypes.c_int
for _name in ("fh_mix_compress_batch", "fh_mix_decompress_batch"):
    getattr(_lib, _name).argtypes = [_P(fh_mix_item), ctypes.c_int32, ctypes.c_void_p]
    getattr(_lib, _name).restype = ctypes.c_int


class FedHybridError(RuntimeError):
    def __init__(self, status: int):
        self.status = int(status)
        super().__init__(f"fedhybrid status {self.status}: {status_string(self.status)}")


def _check(status: int) -> None:
    if status != 0:
        raise FedHybridError(status)


def raw_library() -> ctypes.CDLL:
    """The loaded C library, for callers that marshal their own arguments."""
    return _lib


def status_string(status: int) -> str:
    return _lib.fh_status_string(int(status)).decode()


def packed_bytes(numel: int, bits: int) -> int:
    return int(_lib.fh_packed_bytes(numel, bits))


def meta_bytes(numel: int, group_size: int) -> int:
    return int(_lib.fh_meta_bytes(numel, group_size))


def batch_capacity() -> int:
    return int(_lib.fh_batch_capacity())


_DT = {torch.float32: FH_F32, torch.bfloat16: FH_BF16}
_ROUND = {"nearest": FH_ROUND_NEAREST, "stochastic": FH_ROUND_STOCHASTIC,
          FH_ROUND_NEAREST: FH_ROUND_NEAREST, FH_ROUND_STOCHASTIC: FH_ROUND_STOCHASTIC}


def _dtype_code(t: torch.Tensor) -> int:
    try:
        return _DT[t.dtype]
    except KeyError:
        raise TypeError(f"unsupported dtype {t.dtype}; expected float32 or bfloat16") from None


def _device_tensor(t: torch.Tensor, what: str) -> torch.Tensor:
    if not t.is_cuda:
        raise ValueError(f"{what} must live in device memory (got a {t.device} tensor)")
    if not t.is_contiguous():
        raise ValueError(f"{what} must be contiguous")
    return t


def _stream_ptr(stream: Optional[torch.cuda.Stream]) -> int:
    s = stream if stream is not None else torch.cuda.current_stream()
    return int(s.cuda_stream)


def _scratch(nbytes: int, device, stream: Optional[torch.cuda.Stream]) -> torch.Tensor:
    """A temporary device buffer for work enqueued on `stream`.  The caching allocator hands a
    freed block to the next allocation on the stream it was allocated on (the current one), so a
    buffer a kernel on ANOTHER stream still uses is marked as in use there before it is dropped."""
    t = torch.empty(max(16, int(nbytes)), dtype=torch.uint8, device=device)
    if stream is not None:
        t.record_stream(stream)
    return t


def make_params(group_size: int, bits: int, rounding="nearest", seed: int = 0, tensor_id: int = 0) -> fh_params:
    return fh_params(int(group_size), int(bits), _ROUND[rounding], 0,
                     int(seed) & 0xFFFFFFFFFFFFFFFF, int(tensor_id) & 0xFFFFFFFFFFFFFFFF)


def alloc_compressed(numel: int, group_size: int, bits: int, device) -> "tuple[torch.Tensor, torch.Tensor]":
    """Device buffers of exactly the sizes fh_compress writes: (packed uint8, meta float32[n_g, 2])."""
    packed = torch.empty(packed_bytes(numel, bits), dtype=torch.uint8, device=device)
    meta = torch.empty((meta_bytes(numel, group_size) // 8, 2), dtype=torch.float32, device=device)
    return packed, meta


def fh_compress(x: torch.Tensor, group_size: int, bits: int, rounding="nearest", seed: int = 0,
                tensor_id: int = 0, packed: Optional[torch.Tensor] = None,
                meta: Optional[torch.Tensor] = None, stream=None):
    """Enqueue compression of `x`; returns (packed, meta) device tensors."""
    _device_tensor(x, "x")
    n = x.numel()
    if packed is None or meta is None:
        packed, meta = alloc_compressed(n, group_size, bits, x.device)
    p = make_params(group_size, bits, rounding, seed, tensor_id)
    with torch.cuda.device(x.device):
        _check(_lib.fh_compress(x.data_ptr(), _dtype_code(x), n, ctypes.byref(p),
                                packed.data_ptr(), packed.numel() * packed.element_size(),
                                meta.data_ptr(), meta.numel() * meta.element_size(), _stream_ptr(stream)))
    return packed, meta


def fh_decompress(packed: torch.Tensor, meta: torch.Tensor, numel: int, group_size: int, bits: int,
                  out_dtype=torch.float32, out: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """Enqueue decompression; returns the flat restored tensor."""
    _device_tensor(packed, "packed")
    _device_tensor(meta, "meta")
    if out is None:
        out = torch.empty(numel, dtype=out_dtype, device=packed.device)
    _device_tensor(out, "out")
    if packed.numel() * packed.element_size() < packed_bytes(numel, bits) or \
            meta.numel() * meta.element_size() < meta_bytes(numel, group_size):
        raise FedHybridError(7)
    p = make_params(group_size, bits)
    with torch.cuda.device(packed.device):
        _check(_lib.fh_decompress(packed.data_ptr(), meta.data_ptr(), numel, ctypes.byref(p),
                                  _dtype_code(out), out.data_ptr(), out.numel() * out.element_size(),
                                  _stream_ptr(stream)))
    return out


def fh_roundtrip(x: torch.Tensor, group_size: int, bits: int, rounding="nearest", seed: int = 0,
                 tensor_id: int = 0, out_dtype=torch.float32, packed=None, meta=None, out=None, stream=None):
    """Compress then decompress on one stream; returns (packed, meta, out)."""
    _device_tensor(x, "x")
    n = x.numel()
    if packed is None or meta is None:
        packed, meta = alloc_compressed(n, group_size, bits, x.device)
    if out is None:
        out = torch.empty(n, dtype=out_dtype, device=x.device)
    p = make_params(group_size, bits, rounding, seed, tensor_id)
    with torch.cuda.device(x.device):
        _check(_lib.fh_roundtrip(x.data_ptr(), _dtype_code(x), n, ctypes.byref(p),
                                 packed.data_ptr(), packed.numel() * packed.element_size(),
                                 meta.data_ptr(), meta.numel() * meta.element_size(),
                                 _dtype_code(out), out.data_ptr(), out.numel() * out.element_size(),
                                 _stream_ptr(stream)))
    return packed, meta, out


@dataclass
class BatchEntry:
    """One tensor of a batched call; buffers a call does not use may stay None."""
    group_size: int
    bits: int
    rounding: object = "nearest"
    seed: int = 0
    tensor_id: int = 0
    x: Optional[torch.Tensor] = None
    packed: Optional[torch.Tensor] = None
    meta: Optional[torch.Tensor] = None
    out: Optional[torch.Tensor] = None
    numel: Optional[int] = None


class Batch:
    """A marshalled fh_item array, reusable across calls (the buffers are fixed)."""

    def __init__(self, entries: Sequence[BatchEntry]):
        self.entries: List[BatchEntry] = list(entries)
        self.items = (fh_item * max(1, len(self.entries)))()
        self.count = len(self.entries)
        self.device = None
        for it, e in zip(self.items, self.entries):
            ref = e.x if e.x is not None else e.packed
            if ref is None:
                raise ValueError("a batch entry needs at least x or packed")
            self.device = self.device or ref.device
            n = e.numel if e.numel is not None else (e.x.numel() if e.x is not None else e.out.numel())
            it.numel = n
            it.params = make_params(e.group_size, e.bits, e.rounding, e.seed, e.tensor_id)
            if e.x is not None:
                _device_tensor(e.x, "x")
                it.x, it.x_dtype = e.x.data_ptr(), _dtype_code(e.x)
            if e.packed is not None:
                _device_tensor(e.packed, "packed")
                it.packed, it.packed_cap = e.packed.data_ptr(), e.packed.numel() * e.packed.element_size()
            if e.meta is not None:
                _device_tensor(e.meta, "meta")
                it.meta, it.meta_cap = e.meta.data_ptr(), e.meta.numel() * e.meta.element_size()
            if e.out is not None:
                _device_tensor(e.out, "out")
                it.out, it.out_dtype, it.out_cap = (e.out.data_ptr(), _dtype_code(e.out),
                                                    e.out.numel() * e.out.element_size())

    def _call(self, fn, stream) -> None:
        if self.count == 0:
            return
        with torch.cuda.device(self.device):
            _check(fn(self.items, self.count, _stream_ptr(stream)))


def fh_compress_batch(batch: Batch, stream=None) -> None:
    batch._call(_lib.fh_compress_batch, stream)


def fh_decompress_batch(batch: Batch, stream=None) -> None:
    batch._call(_lib.fh_decompress_batch, stream)


def fh_roundtrip_batch(batch: Batch, stream=None) -> None:
    batch._call(_lib.fh_roundtrip_batch, stream)


def classify_workspace_bytes(numel: int) -> int:
    return int(_lib.fh_classify_workspace_bytes(numel))


def fh_classify_channels(x: torch.Tensor, outer: int, channels: int, inner: int, k_sigma: float = 3.0,
                         min_outliers: int = 1, workspace: Optional[torch.Tensor] = None,
                         stats: Optional[torch.Tensor] = None, counts: Optional[torch.Tensor] = None,
                         mask: Optional[torch.Tensor] = None, stream=None):
    """Enqueue the channel classification of `x` viewed as [outer][channels][inner];
    returns device tensors (stats float64[4] = {mean, variance, threshold, numel},
    counts int32[channels] (bit pattern of uint32), mask uint8[channels])."""
    _device_tensor(x, "x")
    if x.numel() != outer * channels * inner:
        raise ValueError("x.numel() != outer * channels * inner")
    dev = x.device
    if workspace is None:
        workspace = _scratch(classify_workspace_bytes(x.numel()), dev, stream)
    if stats is None:
        stats = torch.empty(4, dtype=torch.float64, device=dev)
    if counts is None:
        counts = torch.empty(channels, dtype=torch.int32, device=dev)
    if mask is None:
        mask = torch.empty(channels, dtype=torch.uint8, device=dev)
    for t, what in ((workspace, "workspace"), (stats, "stats"), (counts, "counts"), (mask, "mask")):
        _device_tensor(t, what)
    if stats.numel() * stats.element_size() < 32 or counts.numel() * counts.element_size() < 4 * channels \
            or mask.numel() * mask.element_size() < channels:
        raise FedHybridError(7)
    with torch.cuda.device(dev):
        _check(_lib.fh_classify_channels(x.data_ptr(), _dtype_code(x), outer, channels, inner, float(k_sigma),
                                         int(min_outliers), workspace.data_ptr(),
                                         workspace.numel() * workspace.element_size(),
                                         stats.data_ptr(), counts.data_ptr(), mask.data_ptr(), _stream_ptr(stream)))
    return stats, counts, mask


def classify_static_scratch_bytes() -> int:
    return int(_lib.fh_classify_static_scratch_bytes())


def fh_classify_channels_static(x: torch.Tensor, outer: int, channels: int, inner: int, k_sigma: float,
                                min_outliers: int, stats: torch.Tensor, counts: torch.Tensor, mask: torch.Tensor,
                                stream=None) -> None:
    """fh_classify_channels with the partial sums in the library's own static device buffer: the
    call allocates nothing, so every output is the caller's (stats float64[4], counts int32
    [channels], mask uint8[channels])."""
    for t, what in ((x, "x"), (stats, "stats"), (counts, "counts"), (mask, "mask")):
        _device_tensor(t, what)
    if x.numel() != outer * channels * inner:
        raise ValueError("x.numel() != outer * channels * inner")
    if _nbytes(stats) < 32 or _nbytes(counts) < 4 * channels or _nbytes(mask) < channels:
        raise FedHybridError(7)
    with torch.cuda.device(x.device):
        _check(_lib.fh_classify_channels_static(x.data_ptr(), _dtype_code(x), outer, channels, inner,
                                                float(k_sigma), int(min_outliers), stats.data_ptr(),
                                                counts.data_ptr(), mask.data_ptr(), _stream_ptr(stream)))


def raw_bytes(outer: int, raw_channels: int, inner: int, dtype) -> int:
    return int(_lib.fh_raw_bytes(outer, raw_channels, inner, _DT[dtype]))


def _nbytes(t: Optional[torch.Tensor]) -> int:
    return 0 if t is None else t.numel() * t.element_size()


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None or t.numel() == 0 else t.data_ptr()


def fh_channel_slots(mask: torch.Tensor, raw_channels: int, slots: Optional[torch.Tensor] = None,
                     stream=None, used: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Enqueue the numbering of the salient channels in `mask` (uint8[channels]); returns the
    device tensor slots int16[channels].  `used` (device int64[1], optional) receives the number
    of raw-store rows in use, which the mixed calls take as `rows_in_use`."""
    _device_tensor(mask, "mask")
    channels = mask.numel()
    if slots is None:
        slots = torch.empty(channels, dtype=torch.int16, device=mask.device)
    _device_tensor(slots, "slots")
    if mask.element_size() != 1 or _nbytes(slots) < 2 * channels or (used is not None and _nbytes(used) < 8):
        raise FedHybridError(7)
    with torch.cuda.device(mask.device):
        _check(_lib.fh_channel_slots_used(mask.data_ptr(), channels, int(raw_channels), slots.data_ptr(),
                                          None if used is None else used.data_ptr(), _stream_ptr(stream)))
    return slots


def fh_channel_slots_batch(masks: Sequence[torch.Tensor], raw_channels: Sequence[int], stream=None):
    """Slot numbering for several tensors with one launch per 16 of them; returns (slots, used): lists
    of device tensors int16[channels] and int64[1] (raw-store rows in use)."""
    if not masks:
        return [], []
    dev = masks[0].device
    items = (fh_slots_item * len(masks))()
    slots, used = [], torch.empty(len(masks), dtype=torch.int64, device=dev)
    for k, (m, rc) in enumerate(zip(masks, raw_channels)):
        _device_tensor(m, "mask")
        s_k = torch.empty(m.numel(), dtype=torch.int16, device=dev)
        slots.append(s_k)
        items[k] = fh_slots_item(m.data_ptr(), m.numel(), int(rc), s_k.data_ptr(), used[k:].data_ptr())
    with torch.cuda.device(dev):
        _check(_lib.fh_channel_slots_batch(items, len(masks), _stream_ptr(stream)))
    return slots, [used[k:k + 1] for k in range(len(masks))]


def fh_compress_mixed(x: torch.Tensor, outer: int, channels: int, inner: int, slots: torch.Tensor,
                      raw_channels: int, group_size: int, bits: int, rounding="nearest", seed: int = 0,
                      tensor_id: int = 0, packed: Optional[torch.Tensor] = None,
                      meta: Optional[torch.Tensor] = None, raw: Optional[torch.Tensor] = None, stream=None,
                      rows_in_use: Optional[torch.Tensor] = None):
    """Enqueue compression of `x` viewed as [outer][channels][inner] with the channels that
    `slots` marks kept verbatim; returns (packed, meta, raw) device tensors.  `rows_in_use`
    (device int64[1] written by fh_channel_slots(..., used=)): a tensor for which it reads 0
    takes the plain quantiser's code path."""
    _device_tensor(x, "x")
    _device_tensor(slots, "slots")
    n = x.numel()
    if n != outer * channels * inner:
        raise ValueError("x.numel() != outer * channels * inner")
    if _nbytes(slots) < 2 * channels:
        raise FedHybridError(7)
    if packed is None or meta is None:
        packed, meta = alloc_compressed(n, group_size, bits, x.device)
    if raw is None:
        raw = torch.empty(max(0, outer * raw_channels * inner), dtype=x.dtype, device=x.device)
    p = make_params(group_size, bits, rounding, seed, tensor_id)
    with torch.cuda.device(x.device):
        if rows_in_use is not None:                           # the count travels in the item struct: a batch of one
            _device_tensor(rows_in_use, "rows_in_use")
            it = fh_mixed_item(x.data_ptr(), _dtype_code(x), FH_F32, outer, channels, inner, slots.data_ptr(),
                               int(raw_channels), _ptr(packed), _nbytes(packed), _ptr(meta), _nbytes(meta),
                               _ptr(raw), _nbytes(raw), _dtype_code(x), 0, None, 0, p, rows_in_use.data_ptr())
            _check(_lib.fh_compress_mixed_batch(ctypes.byref(it), 1, _stream_ptr(stream)))
            return packed, meta, raw
        _check(_lib.fh_compress_mixed(x.data_ptr(), _dtype_code(x), outer, channels, inner, ctypes.byref(p),
                                      slots.data_ptr(), int(raw_channels),
                                      _ptr(packed), _nbytes(packed), _ptr(meta), _nbytes(meta),
                                      _ptr(raw), _nbytes(raw), _stream_ptr(stream)))
    return packed, meta, raw


def fh_decompress_mixed(packed: torch.Tensor, meta: torch.Tensor, raw: torch.Tensor, outer: int, channels: int,
                        inner: int, slots: torch.Tensor, raw_channels: int, group_size: int, bits: int,
                        out_dtype=torch.float32, out: Optional[torch.Tensor] = None, stream=None,
                        rows_in_use: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Enqueue the inverse of fh_compress_mixed; returns the flat restored tensor."""
    for t, what in ((packed, "packed"), (meta, "meta"), (raw, "raw"), (slots, "slots")):
        _device_tensor(t, what)
    n = outer * channels * inner
    if out is None:
        out = torch.empty(n, dtype=out_dtype, device=packed.device)
    _device_tensor(out, "out")
    if _nbytes(packed) < packed_bytes(n, bits) or _nbytes(meta) < meta_bytes(n, group_size) \
            or _nbytes(slots) < 2 * channels or _nbytes(raw) < raw_bytes(outer, raw_channels, inner, raw.dtype):
        raise FedHybridError(7)
    p = make_params(group_size, bits)
    with torch.cuda.device(packed.device):
        if rows_in_use is not None:
            _device_tensor(rows_in_use, "rows_in_use")
            it = fh_mixed_item(None, FH_F32, _dtype_code(out), outer, channels, inner, slots.data_ptr(),
                               int(raw_channels), _ptr(packed), _nbytes(packed), _ptr(meta), _nbytes(meta),
                               _ptr(raw), _nbytes(raw), _dtype_code(raw), 0, _ptr(out), _nbytes(out), p,
                               rows_in_use.data_ptr())
            _check(_lib.fh_decompress_mixed_batch(ctypes.byref(it), 1, _stream_ptr(stream)))
            return out
        _check(_lib.fh_decompress_mixed(_ptr(packed), _ptr(meta), _ptr(raw), _dtype_code(raw),
                                        outer, channels, inner, ctypes.byref(p), slots.data_ptr(),
                                        int(raw_channels), _dtype_code(out), _ptr(out), _nbytes(out),
                                        _stream_ptr(stream)))
    return out


def sparse_info_bytes(maps: int, h: int, w: int, n: int) -> int:
    return int(_lib.fh_sparse_info_bytes(maps, h, w, n))


def sparse_index_bytes(maps: int, h: int, w: int, n: int) -> int:
    return int(_lib.fh_sparse_index_bytes(maps, h, w, n))


def sparse_workspace_bytes(maps: int, h: int, w: int, n: int) -> int:
    return int(_lib.fh_sparse_workspace_bytes(maps, h, w, n))


@dataclass
class SparseBuffers:
    """Worst-case sized device buffers of one fh_sparse_encode call; `totals` (uint64[4] as
    int64: values written, index bytes written, sparse blocks, dense blocks) says how much of
    `values` and `indices` is in use."""
    info: torch.Tensor
    values: torch.Tensor
    indices: torch.Tensor
    totals: torch.Tensor
    workspace: torch.Tensor


def alloc_sparse(maps: int, h: int, w: int, n: int, dtype, device) -> SparseBuffers:
    return SparseBuffers(
        info=torch.empty(max(1, sparse_info_bytes(maps, h, w, n)), dtype=torch.uint8, device=device),
        values=torch.empty(max(1, maps * h * w), dtype=dtype, device=device),
        indices=torch.empty(max(1, sparse_index_bytes(maps, h, w, n)), dtype=torch.uint8, device=device),
        totals=torch.zeros(4, dtype=torch.int64, device=device),
        workspace=torch.empty(max(8, sparse_workspace_bytes(maps, h, w, n)), dtype=torch.uint8, device=device))


def fh_sparse_encode(x: torch.Tensor, maps: int, h: int, w: int, n: int, tau: float,
                     buffers: Optional[SparseBuffers] = None, stream=None, eps: float = 0.0) -> SparseBuffers:
    """Enqueue the block-wise sparse storage of `x` viewed as [maps][h][w]; eps > 0 stores dense
    blocks by Lorenzo prediction within that error bound instead of verbatim."""
    _device_tensor(x, "x")
    if x.numel() != maps * h * w:
        raise ValueError("x.numel() != maps * h * w")
    b = buffers if buffers is not None else alloc_sparse(maps, h, w, n, x.dtype, x.device)
    for t, what in ((b.info, "info"), (b.values, "values"), (b.indices, "indices"), (b.totals, "totals"),
                    (b.workspace, "workspace")):
        _device_tensor(t, what)
    if b.values.dtype != x.dtype or _nbytes(b.totals) < 32:
        raise FedHybridError(7)
    with torch.cuda.device(x.device):
        _check(_lib.fh_sparse_encode(_ptr(x), _dtype_code(x), maps, h, w, int(n), float(tau), float(eps),
                                     b.info.data_ptr(), _nbytes(b.info), b.values.data_ptr(), _nbytes(b.values),
                                     b.indices.data_ptr(), _nbytes(b.indices), b.totals.data_ptr(),
                                     b.workspace.data_ptr(), _nbytes(b.workspace), _stream_ptr(stream)))
    return b


def fh_sparse_decode(info: torch.Tensor, values: torch.Tensor, indices: torch.Tensor, maps: int, h: int, w: int,
                     n: int, out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                     stream=None, eps: float = 0.0) -> torch.Tensor:
    """Enqueue the inverse; `values` and `indices` are the valid prefixes of the two streams
    (their sizes bound what the kernel reads).  Returns the flat [maps][h][w] tensor."""
    for t, what in ((info, "info"), (values, "values"), (indices, "indices")):
        _device_tensor(t, what)
    if out is None:
        out = torch.empty(maps * h * w, dtype=values.dtype, device=info.device)
    if workspace is None:
        workspace = _scratch(sparse_workspace_bytes(maps, h, w, n), info.device, stream)
    _device_tensor(out, "out")
    _device_tensor(workspace, "workspace")
    if _nbytes(info) < sparse_info_bytes(maps, h, w, n) or out.dtype != values.dtype:
        raise FedHybridError(7)
    with torch.cuda.device(info.device):
        _check(_lib.fh_sparse_decode(_ptr(info), _ptr(values), _nbytes(values), _ptr(indices), _nbytes(indices),
                                     _dtype_code(out), maps, h, w, int(n), float(eps), _ptr(out), _nbytes(out),
                                     workspace.data_ptr(), _nbytes(workspace), _stream_ptr(stream)))
    return out


def huffman_stream_bytes(n: int) -> int:
    return int(_lib.fh_huffman_stream_bytes(n))


def huffman_workspace_bytes(n: int) -> int:
    return int(_lib.fh_huffman_workspace_bytes(n))


def fh_huffman_encode(data: torch.Tensor, stream_out: Optional[torch.Tensor] = None,
                      totals: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None, stream=None):
    """Enqueue Huffman coding of the bytes of `data` (a device uint8 tensor); returns
    (stream_out, totals): a worst-case sized uint8 tensor and int64[2] = {stream bytes in use,
    payload bits}, valid once the stream has reached them."""
    _device_tensor(data, "data")
    if data.dtype != torch.uint8:
        raise ValueError("data must be uint8")
    n = data.numel()
    if stream_out is None:
        stream_out = torch.empty(huffman_stream_bytes(n), dtype=torch.uint8, device=data.device)
    if totals is None:
        totals = torch.zeros(2, dtype=torch.int64, device=data.device)
    if workspace is None:
        workspace = _scratch(huffman_workspace_bytes(n), data.device, stream)
    for t, what in ((stream_out, "stream_out"), (totals, "totals"), (workspace, "workspace")):
        _device_tensor(t, what)
    if _nbytes(totals) < 16:
        raise FedHybridError(7)
    with torch.cuda.device(data.device):
        _check(_lib.fh_huffman_encode(_ptr(data), n, stream_out.data_ptr(), _nbytes(stream_out), totals.data_ptr(),
                                      workspace.data_ptr(), _nbytes(workspace), _stream_ptr(stream)))
    return stream_out, totals


def fh_huffman_decode(stream_in: torch.Tensor, n: int, out: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """Enqueue the inverse; `stream_in` is the valid prefix of an encoded stream (its size bounds
    what the kernel reads).  Returns the n restored bytes."""
    _device_tensor(stream_in, "stream_in")
    if out is None:
        out = torch.empty(n, dtype=torch.uint8, device=stream_in.device)
    _device_tensor(out, "out")
    with torch.cuda.device(stream_in.device):
        _check(_lib.fh_huffman_decode(_ptr(stream_in), _nbytes(stream_in), n, _ptr(out), _nbytes(out),
                                      _stream_ptr(stream)))
    return out


def huffman_batch_capacity() -> int:
    return int(_lib.fh_huffman_batch_capacity())


class HuffmanBatch:
    """Several byte buffers coded with one call each way.  `data`: device uint8 tensors; the
    worst-case sized streams, the totals (int64[2] each: stream bytes in use, payload bits) and
    the scratch are allocated here once.  After an encode has finished, `refresh()` reads the
    totals back (a synchronising copy) so that decode is given the valid prefixes.
    `n_device`: per buffer None or a device int64 tensor whose first element holds the number of
    bytes of `data` that count (the buffer's size is then only the upper bound); with it, decode
    needs no refresh: the stream's capacity bounds what it reads."""

    def __init__(self, data, n_device=None):
        self.data = list(data)
        self.n_device = list(n_device) if n_device is not None else [None] * len(self.data)
        for d in self.data:
            _device_tensor(d, "data")
            if d.dtype != torch.uint8:
                raise ValueError("data must be uint8")
        self.device = self.data[0].device if self.data else None
        self.count = len(self.data)
        self.streams = [torch.empty(huffman_stream_bytes(d.numel()), dtype=torch.uint8, device=d.device) for d in self.data]
        self.totals = torch.zeros((max(self.count, 1), 2), dtype=torch.int64, device=self.device)
        self.workspaces = [torch.empty(huffman_workspace_bytes(d.numel()), dtype=torch.uint8, device=d.device)
                           for d in self.data]
        self.out = [torch.empty(d.numel(), dtype=torch.uint8, device=d.device) for d in self.data]
        self.enc = (fh_huffman_encode_item * max(self.count, 1))()
        self.dec = (fh_huffman_decode_item * max(self.count, 1))()
        for i, d in enumerate(self.data):
            e = self.enc[i]
            e.bytes, e.n = _ptr(d), d.numel()
            e.stream_out, e.stream_cap = self.streams[i].data_ptr(), _nbytes(self.streams[i])
            e.totals = self.totals[i].data_ptr()
            e.workspace, e.workspace_cap = self.workspaces[i].data_ptr(), _nbytes(self.workspaces[i])
            q = self.dec[i]
            q.stream_in, q.stream_bytes, q.n = self.streams[i].data_ptr(), _nbytes(self.streams[i]), d.numel()
            q.out, q.out_cap = _ptr(self.out[i]), _nbytes(self.out[i])
            if self.n_device[i] is not None:
                _device_tensor(self.n_device[i], "n_device")
                e.n_device = q.n_device = self.n_device[i].data_ptr()

    def refresh(self):
        used = self.totals.cpu()[:, 0].tolist()
        for i in range(self.count):
            self.dec[i].stream_bytes = int(used[i])
        return used[: self.count]


def fh_huffman_encode_batch(batch: HuffmanBatch, stream=None) -> None:
    if batch.count:
        with torch.cuda.device(batch.device):
            _check(_lib.fh_huffman_encode_batch(batch.enc, batch.count, _stream_ptr(stream)))


def fh_huffman_decode_batch(batch: HuffmanBatch, stream=None) -> None:
    if batch.count:
        with torch.cuda.device(batch.device):
            _check(_lib.fh_huffman_decode_batch(batch.dec, batch.count, _stream_ptr(stream)))


@dataclass
class ClassifyEntry:
    """One tensor of a batched classification; buffers left None are allocated."""
    x: torch.Tensor
    outer: int
    channels: int
    inner: int
    k_sigma: float = 3.0
    min_outliers: int = 1
    workspace: Optional[torch.Tensor] = None
    stats: Optional[torch.Tensor] = None
    counts: Optional[torch.Tensor] = None
    mask: Optional[torch.Tensor] = None


class ClassifyBatch:
    """A marshalled fh_classify_item array, reusable across calls (the buffers are fixed)."""

    def __init__(self, entries: Sequence[ClassifyEntry]):
        self.entries: List[ClassifyEntry] = list(entries)
        self.count = len(self.entries)
        self.items = (fh_classify_item * max(1, self.count))()
        self.device = None
        for it, e in zip(self.items, self.entries):
            _device_tensor(e.x, "x")
            if e.x.numel() != e.outer * e.channels * e.inner:
                raise ValueError("x.numel() != outer * channels * inner")
            dev = e.x.device
            self.device = self.device or dev
            if e.workspace is None:
                e.workspace = torch.empty(classify_workspace_bytes(e.x.numel()), dtype=torch.uint8, device=dev)
            if e.stats is None:
                e.stats = torch.empty(4, dtype=torch.float64, device=dev)
            if e.counts is None:
                e.counts = torch.empty(e.channels, dtype=torch.int32, device=dev)
            if e.mask is None:
                e.mask = torch.empty(e.channels, dtype=torch.uint8, device=dev)
            for t, what in ((e.workspace, "workspace"), (e.stats, "stats"), (e.counts, "counts"), (e.mask, "mask")):
                _device_tensor(t, what)
            if _nbytes(e.stats) < 32 or _nbytes(e.counts) < 4 * e.channels or _nbytes(e.mask) < e.channels:
                raise FedHybridError(7)
            it.x, it.x_dtype, it.reserved = _ptr(e.x), _dtype_code(e.x), 0
            it.outer, it.channels, it.inner = e.outer, e.channels, e.inner
            it.k_sigma, it.min_outliers = float(e.k_sigma), int(e.min_outliers)
            it.workspace, it.workspace_cap = e.workspace.data_ptr(), _nbytes(e.workspace)
            it.stats, it.counts, it.mask = e.stats.data_ptr(), e.counts.data_ptr(), e.mask.data_ptr()


def classify_batch_capacity() -> int:
    return int(_lib.fh_classify_batch_capacity())


def fh_classify_channels_batch(batch: ClassifyBatch, stream=None) -> None:
    """Enqueue the classification of every tensor of the batch; results are in the entries'
    stats / counts / mask tensors."""
    if batch.count == 0:
        return
    with torch.cuda.device(batch.device):
        _check(_lib.fh_classify_channels_batch(batch.items, batch.count, _stream_ptr(stream)))


@dataclass
class SparseEntry:
    """One set of maps of a batched sparse encode / decode.  `buffers` are allocated when left
    None; for decoding, `values` / `indices` are the valid prefixes of the two streams (default:
    the whole buffers, which is safe -- the decoder reads no further than the info bytes say)."""
    maps: int
    h: int
    w: int
    n: int
    tau: float = 0.5
    eps: float = 0.0
    x: Optional[torch.Tensor] = None
    buffers: Optional[SparseBuffers] = None
    values: Optional[torch.Tensor] = None
    indices: Optional[torch.Tensor] = None
    out: Optional[torch.Tensor] = None


def sparse_batch_capacity() -> int:
    return int(_lib.fh_sparse_batch_capacity())


class SparseBatch:
    """Marshalled fh_sparse_encode_item / fh_sparse_decode_item arrays, reusable across calls."""

    def __init__(self, entries: Sequence[SparseEntry]):
        self.entries: List[SparseEntry] = list(entries)
        self.count = len(self.entries)
        self.device = None
        self.enc = (fh_sparse_encode_item * max(1, self.count))()
        self.dec = (fh_sparse_decode_item * max(1, self.count))()
        for e in self.entries:
            ref = e.x if e.x is not None else (e.out if e.out is not None else e.buffers.values)
            self.device = self.device or ref.device
            if e.buffers is None:
                e.buffers = alloc_sparse(e.maps, e.h, e.w, e.n, ref.dtype, ref.device)
        self.refresh()

    def refresh(self) -> None:
        """Re-marshal after entries' tensors (x, out, stream prefixes) were replaced."""
        for enc, dec, e in zip(self.enc, self.dec, self.entries):
            b = e.buffers
            if e.x is not None:
                _device_tensor(e.x, "x")
                if e.x.numel() != e.maps * e.h * e.w or e.x.dtype != b.values.dtype:
                    raise ValueError("x does not match maps * h * w or the buffers' dtype")
                enc.x, enc.dtype = _ptr(e.x), _dtype_code(e.x)
            else:
                enc.x, enc.dtype = None, _dtype_code(b.values)
            enc.n, enc.maps, enc.h, enc.w, enc.tau, enc.eps = int(e.n), e.maps, e.h, e.w, float(e.tau), float(e.eps)
            enc.info, enc.info_cap = b.info.data_ptr(), _nbytes(b.info)
            enc.values, enc.values_cap = b.values.data_ptr(), _nbytes(b.values)
            enc.indices, enc.indices_cap = b.indices.data_ptr(), _nbytes(b.indices)
            enc.totals, enc.workspace, enc.workspace_cap = b.totals.data_ptr(), b.workspace.data_ptr(), _nbytes(b.workspace)
            vals = e.values if e.values is not None else b.values
            idx = e.indices if e.indices is not None else b.indices
            dec.info = b.info.data_ptr()
            dec.values, dec.values_bytes = _ptr(vals), _nbytes(vals)
            dec.indices, dec.indices_bytes = _ptr(idx), _nbytes(idx)
            dec.dtype, dec.n, dec.maps, dec.h, dec.w = _dtype_code(b.values), int(e.n), e.maps, e.h, e.w
            dec.eps, dec.reserved = float(e.eps), 0
            if e.out is not None:
                _device_tensor(e.out, "out")
                dec.out, dec.out_cap = _ptr(e.out), _nbytes(e.out)
            else:
                dec.out, dec.out_cap = None, 0
            dec.workspace, dec.workspace_cap = b.workspace.data_ptr(), _nbytes(b.workspace)


def fh_sparse_encode_batch(batch: SparseBatch, stream=None) -> None:
    if batch.count:
        with torch.cuda.device(batch.device):
            _check(_lib.fh_sparse_encode_batch(batch.enc, batch.count, _stream_ptr(stream)))


def fh_sparse_decode_batch(batch: SparseBatch, stream=None) -> None:
    if batch.count:
        with torch.cuda.device(batch.device):
            _check(_lib.fh_sparse_decode_batch(batch.dec, batch.count, _stream_ptr(stream)))


@dataclass
class MixedEntry:
    """One tensor of a batched mixed compress / decompress; buffers left None are allocated."""
    outer: int
    channels: int
    inner: int
    slots: torch.Tensor
    raw_channels: int
    group_size: int
    bits: int
    rounding: object = "nearest"
    seed: int = 0
    tensor_id: int = 0
    x: Optional[torch.Tensor] = None
    packed: Optional[torch.Tensor] = None
    meta: Optional[torch.Tensor] = None
    raw: Optional[torch.Tensor] = None
    out: Optional[torch.Tensor] = None
    rows_in_use: Optional[torch.Tensor] = None     # device int64[1], as fh_channel_slots(..., used=) writes it


def mixed_batch_capacity() -> int:
    return int(_lib.fh_mixed_batch_capacity())


class MixedBatch:
    """A marshalled fh_mixed_item array, reusable across calls (the buffers are fixed)."""

    def __init__(self, entries: Sequence[MixedEntry]):
        self.entries: List[MixedEntry] = list(entries)
        self.count = len(self.entries)
        self.items = (fh_mixed_item * max(1, self.count))()
        self.device = None
        for it, e in zip(self.items, self.entries):
            n = e.outer * e.channels * e.inner
            ref = e.x if e.x is not None else e.raw
            if ref is None:
                raise ValueError("a mixed entry needs x (to compress) or raw (to restore)")
            dev = ref.device
            self.device = self.device or dev
            if e.packed is None or e.meta is None:
                e.packed, e.meta = alloc_compressed(n, e.group_size, e.bits, dev)
            if e.raw is None:
                e.raw = torch.empty(max(0, e.outer * e.raw_channels * e.inner), dtype=ref.dtype, device=dev)
            for t, what in ((e.slots, "slots"), (e.packed, "packed"), (e.meta, "meta"), (e.raw, "raw")):
                _device_tensor(t, what)
            if _nbytes(e.slots) < 2 * e.channels:
                raise FedHybridError(7)
            it.outer, it.channels, it.inner = e.outer, e.channels, e.inner
            it.slots, it.raw_channels = e.slots.data_ptr(), int(e.raw_channels)
            it.packed, it.packed_cap = _ptr(e.packed), _nbytes(e.packed)
            it.meta, it.meta_cap = _ptr(e.meta), _nbytes(e.meta)
            it.raw, it.raw_cap, it.raw_dtype = _ptr(e.raw), _nbytes(e.raw), _dtype_code(e.raw)
            it.params = make_params(e.group_size, e.bits, e.rounding, e.seed, e.tensor_id)
            if e.rows_in_use is not None:
                _device_tensor(e.rows_in_use, "rows_in_use")
                it.rows_in_use = e.rows_in_use.data_ptr()
            if e.x is not None:
                _device_tensor(e.x, "x")
                if e.x.numel() != n:
                    raise ValueError("x.numel() != outer * channels * inner")
                it.x, it.x_dtype = _ptr(e.x), _dtype_code(e.x)
            if e.out is not None:
                _device_tensor(e.out, "out")
                it.out, it.out_dtype, it.out_cap = _ptr(e.out), _dtype_code(e.out), _nbytes(e.out)


def fh_compress_mixed_batch(batch: MixedBatch, stream=None) -> None:
    if batch.count:
        with torch.cuda.device(batch.device):
            _check(_lib.fh_compress_mixed_batch(batch.items, batch.count, _stream_ptr(stream)))


def fh_decompress_mixed_batch(batch: MixedBatch, stream=None) -> None:
    if batch.count:
        with torch.cuda.device(batch.device):
            _check(_lib.fh_decompress_mixed_batch(batch.items, batch.count, _stream_ptr(stream)))


@dataclass
class MixEntry:
    """One tensor of the whole channel-wise mix compressor (fh_mix_compress / fh_mix_decompress):
    `x` viewed as [outer][channels][inner]; its raw store viewed as `maps` maps of h x w."""
    outer: int
    channels: int
    inner: int
    raw_channels: int
    group_size: int
    bits: int
    rounding: object = "nearest"
    seed: int = 0
    tensor_id: int = 0
    k_sigma: float = 3.0
    min_outliers: int = 1
    maps: int = 0
    h: int = 0
    w: int = 0
    window: int = 4
    tau: float = 0.5
    eps: float = 0.0
    entropy: int = 1
    x: Optional[torch.Tensor] = None
    out: Optional[torch.Tensor] = None
    store: Optional[torch.Tensor] = None
    workspace: Optional[torch.Tensor] = None
    dtype: Optional[torch.dtype] = None            # of x, when only decompressing
    out_dtype: Optional[torch.dtype] = None


class MixBatch:
    """A marshalled fh_mix_item array.  `store` and `workspace` (uint8 device tensors) are
    allocated here when an entry brings none; `regions[i]` says where the parts lie, and
    `part(i, name)` returns a uint8 view of one of them."""

    def __init__(self, entries: Sequence[MixEntry], device=None, shared_workspace: bool = False):
        self.entries = list(entries)
        self.count = len(self.entries)
        self.items = (fh_mix_item * max(1, self.count))()
        self.regions: List[fh_mix_regions] = []
        self.device = device
        for it, e in zip(self.items, self.entries):
            ref = e.x if e.x is not None else (e.store if e.store is not None else e.out)
            if ref is not None:
                self.device = self.device or ref.device
            x_dtype = e.x.dtype if e.x is not None else (e.dtype or torch.float32)
            it.x_dtype = _DT[x_dtype]
            it.out_dtype = _DT[e.out.dtype if e.out is not None else (e.out_dtype or torch.float32)]
            it.outer, it.channels, it.inner = int(e.outer), int(e.channels), int(e.inner)
            it.maps, it.h, it.w = int(e.maps), int(e.h), int(e.w)
            it.quant = make_params(e.group_size, e.bits, e.rounding, e.seed, e.tensor_id)
            it.k_sigma, it.min_outliers, it.raw_channels = float(e.k_sigma), int(e.min_outliers), int(e.raw_channels)
            it.window, it.entropy, it.tau, it.eps, it.reserved = int(e.window), int(e.entropy), float(e.tau), float(e.eps), 0
            r = fh_mix_regions()
            _check(_lib.fh_mix_layout(ctypes.byref(it), ctypes.byref(r)))
            self.regions.append(r)
        if self.device is None:
            raise ValueError("no device: give the batch a device or an entry a tensor")
        shared = None
        if shared_workspace and self.count:            # calls on one stream may share their scratch ... one item at a time
            shared = torch.empty(max(r.workspace_bytes for r in self.regions), dtype=torch.uint8, device=self.device)
        for it, e, r in zip(self.items, self.entries, self.regions):
            if e.store is None:
                e.store = torch.empty(max(256, r.store_bytes), dtype=torch.uint8, device=self.device)
            if e.workspace is None:
                e.workspace = shared if shared is not None else \
                    torch.empty(max(256, r.workspace_bytes), dtype=torch.uint8, device=self.device)
            for t, what in ((e.store, "store"), (e.workspace, "workspace")):
                _device_tensor(t, what)
            it.store, it.store_cap = e.store.data_ptr(), _nbytes(e.store)
            it.workspace, it.workspace_cap = e.workspace.data_ptr(), _nbytes(e.workspace)
            if e.x is not None:
                _device_tensor(e.x, "x")
                if e.x.numel() != e.outer * e.channels * e.inner:
                    raise ValueError("x.numel() != outer * channels * inner")
                it.x = _ptr(e.x)
            if e.out is not None:
                _device_tensor(e.out, "out")
                it.out, it.out_cap = _ptr(e.out), _nbytes(e.out)

    def part(self, i: int, name: str) -> torch.Tensor:
        r = self.regions[i]
        store_parts = {"header": 64, "slots": r.slots_bytes, "packed": r.packed_bytes, "meta": r.meta_bytes,
                       "info": r.info_bytes, "values": r.values_cap, "indices": r.indices_cap, "huffman": r.huffman_cap}
        work_parts = {"stats": 32, "counts": 4 * self.entries[i].channels, "mask": self.entries[i].channels,
                      "raw": r.raw_bytes, "indices_ws": r.indices_cap}
        if name in store_parts:
            off = getattr(r, name)
            return self.entries[i].store[off: off + store_parts[name]]
        off = getattr(r, name)
        return self.entries[i].workspace[off: off + work_parts[name]]

    def header(self, i: int) -> torch.Tensor:
        """int64[8] view of the stored form's header."""
        return self.part(i, "header").view(torch.int64)

    def _call(self, fn, stream) -> None:
        if self.count:
            with torch.cuda.device(self.device):
                _check(fn(self.items, self.count, _stream_ptr(stream)))


def mix_layout(item: fh_mix_item) -> fh_mix_regions:
    r = fh_mix_regions()
    _check(_lib.fh_mix_layout(ctypes.byref(item), ctypes.byref(r)))
    return r


def fh_mix_compress_batch(batch: MixBatch, stream=None) -> None:
    batch._call(_lib.fh_mix_compress_batch, stream)


def fh_mix_decompress_batch(batch: MixBatch, stream=None) -> None:
    batch._call(_lib.fh_mix_decompress_batch, stream)
