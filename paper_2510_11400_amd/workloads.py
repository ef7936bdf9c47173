"""Seeded synthetic activation workloads (inputs only).

This module builds the tensor sets that stand in for the activations a
training engine saves in the forward pass (FedHybrid, Section 3 "Activation
compression"; the per-sample tensor shapes of the local-engine ablation figure,
panel (a); batch sizes from the experimental setup).  It contains *no* step of
the compression method: no range statistics, no quantisation, no packing, no
random-bit generator of the method.  Both the CPU oracle's tests and the HIP
path's tests draw their inputs from here so that they see identical bytes.

Every tensor is described by a `TensorSpec` (shape, dtype, distribution,
quantiser parameters, tensor id) and materialised on the host by
`materialise()`.  bf16 data is carried as uint16 bit patterns.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Iterator, List, Optional, Sequence, Tuple

import numpy as np

F32 = "f32"
BF16 = "bf16"
NEAREST = "nearest"
STOCHASTIC = "stochastic"


@dataclass(frozen=True)
class TensorSpec:
    """One saved activation and the compression parameters its plan assigns."""

    tensor_id: int
    shape: Tuple[int, ...]
    dtype: str          # F32 | BF16
    dist: str           # 'relu' | 'relu6' | 'gauss' | 'gelu' | 'gauss_outlier'
    group_size: int
    bits: int
    rounding: str       # NEAREST | STOCHASTIC
    seed: int           # seed of the method's random bits (stochastic rounding)

    @property
    def numel(self) -> int:
        n = 1
        for s in self.shape:
            n *= int(s)
        return n

    @property
    def itemsize(self) -> int:
        return 4 if self.dtype == F32 else 2

    @property
    def nbytes(self) -> int:
        return self.numel * self.itemsize


@dataclass
class Workload:
    name: str
    data_seed: int
    tensors: List[TensorSpec] = field(default_factory=list)

    @property
    def numel(self) -> int:
        return sum(t.numel for t in self.tensors)

    @property
    def nbytes(self) -> int:
        return sum(t.nbytes for t in self.tensors)


def _to_bf16_bits(x32: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit patterns (round-to-nearest-even) through torch's CPU cast."""
    import torch

    t = torch.from_numpy(np.ascontiguousarray(x32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16).copy()


def _draw(dist: str, n: int, rng: np.random.Generator) -> np.ndarray:
    """n fp32 values of the named activation distribution."""
    z = rng.standard_normal(n, dtype=np.float32)
    if dist == "relu":            # 0 w.p. 1/2, else half-normal
        np.maximum(z, np.float32(0.0), out=z)
        return z
    if dist == "relu6":           # ReLU6 of N(0,1): ~half exact zeros, capped at 6
        np.clip(z, np.float32(0.0), np.float32(6.0), out=z)
        return z
    if dist == "gauss":
        return z
    if dist == "gelu":            # exact (erf) GELU of N(0,1) pre-activations
        import torch

        return torch.nn.functional.gelu(torch.from_numpy(z)).numpy()
    if dist == "gauss_outlier":   # N(0,1) with an independent 1 % of elements scaled x10
        hit = rng.random(n, dtype=np.float32) < np.float32(0.01)
        z[hit] *= np.float32(10.0)
        return z
    raise ValueError(f"unknown distribution {dist!r}")


def materialise(w: Workload, spec: TensorSpec) -> np.ndarray:
    """Host array for one tensor: float32, or uint16 bf16 bit patterns; flat, C-contiguous.

    The stream depends only on (workload data seed, tensor id), so tensors can be
    generated one at a time and in any order.
    """
    rng = np.random.default_rng(np.random.SeedSequence([w.data_seed, spec.tensor_id]))
    x = _draw(spec.dist, spec.numel, rng)
    if spec.dtype == BF16:
        return _to_bf16_bits(x)
    return x


def iter_materialised(w: Workload) -> Iterator[Tuple[TensorSpec, np.ndarray]]:
    for spec in w.tensors:
        yield spec, materialise(w, spec)


# --------------------------------------------------------------------------
# The five workload configurations
# --------------------------------------------------------------------------

def _scaled_batch(b: int, scale: float) -> int:
    return max(1, int(round(b * scale)))


def config1(seed: int = 0) -> Workload:
    """One 4x64x32x32 fp32 post-ReLU tensor; G=256, 8-bit, nearest."""
    w = Workload("c1_single_relu_g256_b8_nearest", seed)
    w.tensors.append(TensorSpec(0, (4, 64, 32, 32), F32, "relu", 256, 8, NEAREST, seed))
    return w


def config2(seed: int = 0, batch: int = 32) -> Workload:
    """CIFAR-style ResNet-18 saved activations, post-ReLU; G=256, 4-bit, stochastic."""
    w = Workload(f"c2_resnet18_cifar_b{batch}_g256_b4_stochastic", seed)
    tid = 0
    for c, hw in ((64, 32), (128, 16), (256, 8), (512, 4)):
        for _ in range(4):
            w.tensors.append(TensorSpec(tid, (batch, c, hw, hw), F32, "relu", 256, 4, STOCHASTIC, seed))
            tid += 1
    return w


def config3(seed: int = 0, batch: int = 64) -> Workload:
    """MobileNetV2-style ReLU6 activations at 224x224 input; G=128, 4-bit, nearest."""
    w = Workload(f"c3_mobilenetv2_b{batch}_g128_b4_nearest", seed)
    shapes = ((32, 112), (96, 112), (144, 56), (192, 28), (384, 14))
    for tid, (c, hw) in enumerate(shapes):
        w.tensors.append(TensorSpec(tid, (batch, c, hw, hw), F32, "relu6", 128, 4, NEAREST, seed))
    return w


def config4(seed: int = 0, layers: int = 12, batch: int = 16, seq: int = 512) -> Workload:
    """Transformer-encoder activations in bf16; G=64 along the hidden dim, 2-bit, stochastic.

    Tensor id 2*l is layer l's LayerNorm output (N(0,1)), 2*l+1 its GELU output.
    """
    w = Workload(f"c4_transformer_l{layers}_b{batch}_s{seq}_bf16_g64_b2_stochastic", seed)
    for layer in range(layers):
        w.tensors.append(TensorSpec(2 * layer, (batch, seq, 768), BF16, "gauss", 64, 2, STOCHASTIC, seed))
        w.tensors.append(TensorSpec(2 * layer + 1, (batch, seq, 3072), BF16, "gelu", 64, 2, STOCHASTIC, seed))
    return w


def config5(seed: int = 0, total_bytes: int = 2 << 30, count: int = 48) -> Workload:
    """Mixed-plan stress set: `count` fp32 NCHW tensors totalling ~`total_bytes`.

    Shapes B x C x H x H with B in {32,64}, C in [64,512], H in [7,112].  A plain
    uniform draw would overshoot the byte budget by a wide margin, so tensor j is
    drawn uniformly among the shapes whose size is at most twice the mean of what
    is left (remaining budget / remaining count); the last tensor takes the shape
    closest to the remaining budget.  Per tensor: bits from {2,4,8}, rounding from
    {nearest, stochastic}; a seeded permutation marks half the tensors post-ReLU
    and half Gaussian with 1 % outliers x10.  G=256 throughout, so tensors whose
    element count is not a multiple of 256 end in a short group.
    """
    rng = np.random.default_rng(np.random.SeedSequence([seed, 0x5EED5]))
    bs = np.array([32, 64], dtype=np.int64)
    cs = np.arange(64, 513, dtype=np.int64)
    hs = np.arange(7, 113, dtype=np.int64)
    bb, cc, hh = np.meshgrid(bs, cs, hs, indexing="ij")
    bb, cc, hh = bb.ravel(), cc.ravel(), hh.ravel()
    sizes = bb * cc * hh * hh * 4
    order = rng.permutation(count)
    relu_ids = set(int(i) for i in order[: count // 2])
    w = Workload(f"c5_mixed_{total_bytes >> 20}MiB_n{count}_g256", seed)
    remaining = int(total_bytes)
    for j in range(count):
        left = count - j
        if left == 1:
            pick = int(np.argmin(np.abs(sizes - remaining)))
        else:
            cap = 2 * remaining // left
            ok = np.flatnonzero(sizes <= cap)
            if ok.size == 0:                       # budget nearly spent: smallest shape
                ok = np.array([int(np.argmin(sizes))])
            pick = int(ok[rng.integers(0, ok.size)])
        bits = int((2, 4, 8)[int(rng.integers(0, 3))])
        rounding = (NEAREST, STOCHASTIC)[int(rng.integers(0, 2))]
        dist = "relu" if j in relu_ids else "gauss_outlier"
        shape = (int(bb[pick]), int(cc[pick]), int(hh[pick]), int(hh[pick]))
        w.tensors.append(TensorSpec(j, shape, F32, dist, 256, bits, rounding, seed))
        remaining = max(0, remaining - int(sizes[pick]))
    return w


def small_variant(index: int, seed: int = 0) -> Workload:
    """A reduced copy of configuration `index` (1..5) with the same structure:
    same dtypes, distributions, group sizes, bit widths and rounding modes, fewer
    or smaller tensors.  Sized for element-by-element checks in a second or two."""
    if index == 1:
        return config1(seed)
    if index == 2:
        return config2(seed, batch=4)
    if index == 3:
        return config3(seed, batch=1)
    if index == 4:
        return config4(seed, layers=2, batch=2, seq=128)
    if index == 5:
        w = config5(seed, total_bytes=96 << 20, count=48)
        w.name += "_small"
        return w
    raise ValueError(index)


def full_config(index: int, seed: int = 0) -> Workload:
    return {1: config1, 2: config2, 3: config3, 4: config4, 5: config5}[index](seed)


# The per-sample shapes of the paper's local-engine ablation (panel (a)); H*W = 49
# and 196 do not divide any supported group size, so groups straddle channels and
# small batches end in a short group.
ABLATION_SHAPES: Sequence[Tuple[int, int, int]] = (
    (64, 112, 112), (64, 56, 56), (128, 28, 28), (256, 14, 14), (512, 7, 7))


def ablation_set(batch: int = 1, group_size: int = 256, bits: int = 4,
                 rounding: str = NEAREST, seed: int = 0) -> Workload:
    w = Workload(f"ablation_b{batch}_g{group_size}_b{bits}_{rounding}", seed)
    for tid, (c, h, ww) in enumerate(ABLATION_SHAPES):
        w.tensors.append(TensorSpec(tid, (batch, c, h, ww), F32, "relu", group_size, bits, rounding, seed))
    return w


# --------------------------------------------------------------------------
# Activations with channel-clustered outliers (inputs for channel classification)
# --------------------------------------------------------------------------

def outlier_channel_tensor(outer: int, channels: int, inner: int, seed: int = 0, dist: str = "gauss",
                           salient_fraction: float = 0.04, hit_fraction: float = 0.05,
                           magnitude: float = 81.0, dtype: str = F32):
    """A [outer][channels][inner] activation whose outliers are sparse and clustered in a few
    channels, as the paper describes them (Section 4.4.1; magnitudes 81x for CNNs and 347x
    for Transformers are the figures it quotes).  A seeded subset of about
    `salient_fraction` of the channels gets `hit_fraction` of its elements multiplied by
    `magnitude`; every other element follows `dist`.  Returns (flat array, planted channel ids).
    """
    rng = np.random.default_rng(np.random.SeedSequence([seed, 0xC1A55, outer, channels, inner]))
    x = _draw(dist, outer * channels * inner, rng).reshape(outer, channels, inner)
    k = max(1, int(round(channels * salient_fraction)))
    planted = np.sort(rng.choice(channels, size=k, replace=False))
    for c in planted:
        hit = rng.random((outer, inner)) < hit_fraction
        block = x[:, c, :]
        block[hit] = (np.abs(block[hit]) + np.float32(0.5)) * np.float32(magnitude)
    flat = np.ascontiguousarray(x.reshape(-1))
    if dtype == BF16:
        flat = _to_bf16_bits(flat)
    return flat, planted


def salient_feature_maps(maps: int, h: int, w: int, seed: int = 0, zero_level: float = 0.3,
                         outlier_fraction: float = 0.02, magnitude: float = 81.0, dtype: str = F32) -> np.ndarray:
    """[maps][h][w] feature maps of outlier-rich channels as the paper describes them (Section
    4.4.1): many zeros, locally clustered (post-ReLU responses are spatially smooth), and a
    sprinkle of large outliers.  A coarse random field (one value per 8 x 8 patch, so zeros come
    in patches) plus fine noise goes through ReLU; `zero_level` shifts the field down (more
    zeros); `outlier_fraction` of the surviving values is multiplied by `magnitude`.  Returns the
    flat array (float32, or bf16 bit patterns)."""
    rng = np.random.default_rng(np.random.SeedSequence([seed, 0x5AC5E, maps, h, w]))
    ch, cw = (h + 7) // 8, (w + 7) // 8
    coarse = rng.standard_normal((maps, ch, cw), dtype=np.float32)
    field = np.repeat(np.repeat(coarse, 8, axis=1), 8, axis=2)[:, :h, :w]
    x = field + np.float32(0.35) * rng.standard_normal((maps, h, w), dtype=np.float32) - np.float32(zero_level)
    np.maximum(x, np.float32(0.0), out=x)
    hit = (rng.random((maps, h, w), dtype=np.float32) < np.float32(outlier_fraction)) & (x > 0)
    x[hit] *= np.float32(magnitude)
    flat = np.ascontiguousarray(x.reshape(-1))
    if dtype == BF16:
        flat = _to_bf16_bits(flat)
    return flat
