"""A second, vectorised numpy implementation of the group quantiser, written
independently of `oracle/fho.c` (different language, different structure: whole
arrays at a time, padded 2-D group view, Philox on uint64 lanes).  The tests use it
to catch slips in the C oracle that the closed-form pins would not; it is not an
authority of its own -- the pins in test_oracle_pins.py are.

Definition followed: the linear-scale quantiser FedHybrid applies to normal
channels (Section 4.4.1), with group size, bit width, rounding and seed as inputs.
"""
from __future__ import annotations

import numpy as np

_M0 = np.uint64(0xD2511F53)
_M1 = np.uint64(0xCD9E8D57)
_W0 = np.uint64(0x9E3779B9)
_W1 = np.uint64(0xBB67AE85)
_MASK = np.uint64(0xFFFFFFFF)
_S32 = np.uint64(32)


def philox4x32_10_np(c0, c1, c2, c3, k0, k1):
    """Vectorised Philox4x32-10 on uint64 arrays holding 32-bit words."""
    c0, c1, c2, c3 = (np.asarray(v, dtype=np.uint64) & _MASK for v in (c0, c1, c2, c3))
    k0 = np.uint64(k0) & _MASK
    k1 = np.uint64(k1) & _MASK
    for r in range(10):
        if r:
            k0 = (k0 + _W0) & _MASK
            k1 = (k1 + _W1) & _MASK
        p0 = _M0 * c0
        p1 = _M1 * c2
        c0, c1, c2, c3 = ((p1 >> _S32) ^ c1 ^ k0, p1 & _MASK, (p0 >> _S32) ^ c3 ^ k1, p0 & _MASK)
    return c0, c1, c2, c3


def random16_np(seed: int, tensor_id: int, n: int, first: int = 0) -> np.ndarray:
    """16 random bits for elements first .. first+n-1."""
    idx = np.arange(first, first + n, dtype=np.uint64)
    blk = idx >> np.uint64(3)
    ub, inv = np.unique(blk, return_inverse=True)
    w = philox4x32_10_np(ub & _MASK, ub >> _S32,
                         np.full(ub.shape, tensor_id & 0xFFFFFFFF, dtype=np.uint64),
                         np.full(ub.shape, (tensor_id >> 32) & 0xFFFFFFFF, dtype=np.uint64),
                         seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF)
    words = np.stack(w, axis=1)[inv, ((idx & np.uint64(7)) >> np.uint64(1)).astype(np.int64)]
    half = np.where((idx & np.uint64(1)) == 1, words >> np.uint64(16), words & np.uint64(0xFFFF))
    return half.astype(np.uint32)


def compress_np(x32: np.ndarray, G: int, B: int, rounding: str = "nearest", seed: int = 0, tensor_id: int = 0):
    """x32: float32 flat array -> (packed uint8, meta float32[n_g,2], codes uint8[n])."""
    f32 = np.float32
    n = x32.size
    ng = (n + G - 1) // G
    L = f32((1 << B) - 1)
    pad = ng * G - n
    lo = np.concatenate([x32, np.full(pad, np.inf, dtype=f32)]).reshape(ng, G)
    hi = np.concatenate([x32, np.full(pad, -np.inf, dtype=f32)]).reshape(ng, G)
    mn = lo.min(axis=1)
    mx = hi.max(axis=1)
    rng = (mx - mn).astype(f32)
    deg = rng < f32(2.0 ** -100)
    safe = np.where(deg, f32(1), rng).astype(f32)
    scale = np.where(deg, f32(0), (safe / L).astype(f32)).astype(f32)
    inv = np.where(deg, f32(0), (L / safe).astype(f32)).astype(f32)
    zero = (mn + f32(0)).astype(f32)
    xs = np.concatenate([x32, np.zeros(pad, dtype=f32)]).reshape(ng, G)
    with np.errstate(invalid="ignore", over="ignore"):
        q = ((xs - mn[:, None]).astype(f32) * inv[:, None]).astype(f32)
    q = np.minimum(np.maximum(q, f32(0)), L).astype(f32)
    q = np.where(deg[:, None], f32(0), q).ravel()[:n]
    if rounding == "nearest":
        codes = np.rint(q).astype(np.uint32)
    else:
        k = np.floor(q).astype(f32)
        frac = (q - k).astype(f32)
        u = (random16_np(seed, tensor_id, n).astype(f32) * f32(2.0 ** -16)).astype(f32)
        codes = k.astype(np.uint32) + (u < frac).astype(np.uint32)
    per = 8 // B
    raw = (n * B + 7) // 8
    total = (raw + 15) // 16 * 16 if n else 0
    cpad = np.concatenate([codes, np.zeros(raw * per - n, dtype=np.uint32)]).reshape(raw, per)
    shifts = (np.arange(per, dtype=np.uint32) * np.uint32(B))[None, :]
    by = np.bitwise_or.reduce(cpad << shifts, axis=1).astype(np.uint8)
    packed = np.concatenate([by, np.zeros(total - raw, dtype=np.uint8)])
    meta = np.stack([scale, zero], axis=1).astype(f32)
    return packed, meta, codes.astype(np.uint8)


def decompress_np(codes: np.ndarray, meta: np.ndarray, G: int) -> np.ndarray:
    """Single-rounding multiply-add through float64: code*scale is exact in
    float64 (8-bit by 24-bit significands) and so is the following sum whenever the
    exponents are within range of the 53-bit significand, so one rounding to
    float32 equals fmaf except in double-rounding corner cases, which the caller
    tolerates by comparing with at most one ulp of slack."""
    g = np.arange(codes.size) // G
    v = codes.astype(np.float64) * meta[g, 0].astype(np.float64) + meta[g, 1].astype(np.float64)
    return v.astype(np.float32)


def compress_mixed_np(x32: np.ndarray, outer: int, channels: int, inner: int, kept: np.ndarray, G: int, B: int,
                      rounding: str = "nearest", seed: int = 0, tensor_id: int = 0):
    """The same quantiser when the channels flagged in `kept` (bool[channels]) are routed around
    it (Section 4.4.1: only normal channels are quantised): their elements are invisible to
    the group statistics and get code 0.  -> (packed, meta, codes)."""
    f32 = np.float32
    n = x32.size
    assert n == outer * channels * inner
    normal = np.broadcast_to(~np.asarray(kept, dtype=bool)[None, :, None], (outer, channels, inner)).reshape(n)
    ng = (n + G - 1) // G
    L = f32((1 << B) - 1)
    pad = ng * G - n
    lo = np.concatenate([np.where(normal, x32, f32(np.inf)), np.full(pad, np.inf, dtype=f32)]).reshape(ng, G)
    hi = np.concatenate([np.where(normal, x32, f32(-np.inf)), np.full(pad, -np.inf, dtype=f32)]).reshape(ng, G)
    mn = lo.min(axis=1)
    mx = hi.max(axis=1)
    empty = mn > mx
    mn = np.where(empty, f32(0), mn).astype(f32)
    mx = np.where(empty, f32(0), mx).astype(f32)
    rng = (mx - mn).astype(f32)
    deg = rng < f32(2.0 ** -100)
    safe = np.where(deg, f32(1), rng).astype(f32)
    scale = np.where(deg, f32(0), (safe / L).astype(f32)).astype(f32)
    inv = np.where(deg, f32(0), (L / safe).astype(f32)).astype(f32)
    zero = (mn + f32(0)).astype(f32)
    xs = np.concatenate([np.where(normal, x32, f32(0)), np.zeros(pad, dtype=f32)]).reshape(ng, G)
    with np.errstate(invalid="ignore", over="ignore"):
        q = ((xs - mn[:, None]).astype(f32) * inv[:, None]).astype(f32)
    q = np.minimum(np.maximum(q, f32(0)), L).astype(f32)
    q = np.where(deg[:, None], f32(0), q).ravel()[:n]
    if rounding == "nearest":
        codes = np.rint(q).astype(np.uint32)
    else:
        k = np.floor(q).astype(f32)
        frac = (q - k).astype(f32)
        u = (random16_np(seed, tensor_id, n).astype(f32) * f32(2.0 ** -16)).astype(f32)
        codes = k.astype(np.uint32) + (u < frac).astype(np.uint32)
    codes = np.where(normal, codes, np.uint32(0)).astype(np.uint32)
    per = 8 // B
    raw = (n * B + 7) // 8
    total = (raw + 15) // 16 * 16 if n else 0
    cpad = np.concatenate([codes, np.zeros(raw * per - n, dtype=np.uint32)]).reshape(raw, per)
    shifts = (np.arange(per, dtype=np.uint32) * np.uint32(B))[None, :]
    by = np.bitwise_or.reduce(cpad << shifts, axis=1).astype(np.uint8)
    packed = np.concatenate([by, np.zeros(total - raw, dtype=np.uint8)])
    meta = np.stack([scale, zero], axis=1).astype(f32)
    return packed, meta, codes.astype(np.uint8)
