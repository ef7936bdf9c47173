"""Hooking the compressor into a training step, and handing a planner its costs.

`SavedActivations` is the literal "compress in the forward pass, decompress during
backpropagation" of FedHybrid's local training engine (Section 3, Activation compression):
a `torch.autograd.graph.saved_tensors_hooks` pair whose pack side calls `fh_compress` and
whose unpack side calls `fh_decompress` -- or, with a channel dimension given, the channel-wise
mix of Section 4.4.1 (classification, slot numbering, mixed compress / restore).  Only argument
marshalling happens here; every byte is produced by the library's kernels.

`mps` is the paper's reward metric (Section 4.3): RW(d) = SM(d) * FLT(d) and
MPS(d) = RW(d) / (PC(d) + RC(d)), where SM is the memory a technique saves on tensor d, FLT
the time the tensor would otherwise sit unused, PC the cost of purging it and RC the cost of
regaining it.  `SavedActivations(record=True)` measures PC (compress time) and RC (decompress
time) per tensor with events on the stream and reports SM, so that a host-side planner
(Algorithm 1 compares MPS_compute with MPS_compress per tensor) gets MPS_compress from
measurement rather than from a model.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional

import torch

from . import api


def mps(saved_bytes: float, freed_lifetime: float, purge_cost: float, regain_cost: float) -> float:
    """Memory reduced per second (Section 4.3): SM * FLT / (PC + RC)."""
    cost = purge_cost + regain_cost
    if cost <= 0.0:
        raise ValueError("purge cost + regain cost must be positive")
    return saved_bytes * freed_lifetime / cost


def prefer_recompute(mps_compute: float, mps_compress: float) -> bool:
    """The branch Algorithm 1 takes for the tensor with the largest MPS: evict (and recompute
    later) when recomputation rewards more than compression, else compress."""
    return mps_compute > mps_compress


@dataclass
class TensorRecord:
    """What one compressed activation cost and saved."""
    tensor_id: int
    numel: int
    dtype: torch.dtype
    input_bytes: int
    stored_bytes: int                      # codes (padded) + meta
    _pack: Optional[tuple] = field(default=None, repr=False)
    _unpack: Optional[tuple] = field(default=None, repr=False)

    @property
    def saved_bytes(self) -> int:          # SM
        return self.input_bytes - self.stored_bytes

    @property
    def purge_cost(self) -> Optional[float]:   # PC, seconds; call after the stream has drained
        if self._pack is None:
            return None
        share = self._pack[2] if len(self._pack) > 2 else 1.0     # this tensor's part of a batched call, by bytes
        return self._pack[0].elapsed_time(self._pack[1]) * 1e-3 * share

    @property
    def regain_cost(self) -> Optional[float]:  # RC, seconds
        return None if self._unpack is None else self._unpack[0].elapsed_time(self._unpack[1]) * 1e-3

    def mps_compress(self, freed_lifetime: float) -> float:
        if self.purge_cost is None or self.regain_cost is None:
            raise RuntimeError("costs are known only after the tensor has been compressed and restored "
                               "with record=True")
        return mps(self.saved_bytes, freed_lifetime, self.purge_cost, self.regain_cost)


class _Packed:
    __slots__ = ("packed", "meta", "shape", "dtype", "numel", "record", "mixed")

    def __init__(self, packed, meta, shape, dtype, numel, record, mixed=None):
        self.packed, self.meta, self.shape, self.dtype, self.numel, self.record = packed, meta, shape, dtype, numel, record
        self.mixed = mixed                 # (outer, channels, inner, slots, raw_channels, raw) on the channel-wise path


class _Deferred:
    """A tensor handed to the pack hook that waits for its batch: `handle` is the packed form once
    the batch has been compressed, and the tensor itself is let go then."""
    __slots__ = ("x", "tid", "shape", "dtype", "split", "handle")

    def __init__(self, x, tid, shape, dtype, split):
        self.x, self.tid, self.shape, self.dtype, self.split, self.handle = x, tid, shape, dtype, split, None


class SavedActivations(torch.autograd.graph.saved_tensors_hooks):
    """Context manager: tensors that autograd saves inside it are stored compressed.

    Eligible: device tensors of float32 / bfloat16 with at least `min_numel` elements that are
    neither parameters nor listed in `exclude` (weights are saved for backward too, and must
    stay exact: pass `exclude=model.parameters()`; tensors are recognised by their storage
    address).  Everything else is saved as it is.  Non-contiguous tensors are made contiguous first (a copy by torch).
    Under `torch.autocast` a layer saves the low-precision COPY of its weight, which is neither a Parameter
    nor at a parameter's address: such copies are quantised like activations unless the caller keeps them
    out (run the forward pass in the parameters' own dtype, or raise `min_numel` above the weights' sizes).
    Stochastic rounding draws its bits from (seed, tensor_id); tensor ids count up from
    `first_tensor_id` in the order tensors are saved, so a step is reproducible.

    With `channel_dim` set, every tensor takes the channel-wise mix of Section 4.4.1: its
    channels (dimension `channel_dim`, at most 16384 of them) are classified by the 3-sigma rule
    -- salient where more than `outlier_share` of a channel's elements lie beyond `k_sigma`
    standard deviations of the tensor -- and up to `raw_share` of the channels, the salient
    ones, are kept verbatim beside the quantised stream, so that their outliers do not stretch
    the range of the groups they sit in.  All of it is enqueued on the stream; nothing waits
    for the classification's result.

    With `batch_bytes` > 0 tensors are compressed in batches: the pack hook only notes a tensor,
    and once `batch_bytes` of them wait (or one of them is needed back, or the context ends) the
    whole batch goes through the batched entry points -- a handful of launches for the batch
    instead of one to seven per tensor, at the price of holding up to `batch_bytes` of
    activations uncompressed a little longer.  Results are the same bytes either way.
    """

    def __init__(self, group_size: int = 256, bits: int = 4, rounding="nearest", seed: int = 0,
                 min_numel: int = 4096, first_tensor_id: int = 0, record: bool = False, exclude=(),
                 channel_dim: Optional[int] = None, k_sigma: float = 3.0, outlier_share: float = 0.01,
                 raw_share: float = 1.0 / 16.0, batch_bytes: int = 0):
        self.group_size, self.bits, self.rounding, self.seed = group_size, bits, rounding, seed
        self.batch_bytes = int(batch_bytes)
        self._pending: List[_Deferred] = []
        self._pending_bytes = 0
        self.min_numel = min_numel
        self.channel_dim, self.k_sigma, self.outlier_share, self.raw_share = channel_dim, k_sigma, outlier_share, raw_share
        self.next_tensor_id = first_tensor_id
        self.record = record
        self.records: List[TensorRecord] = []
        self._exclude = {int(t.data_ptr()) for t in exclude}
        super().__init__(self._pack, self._unpack)

    def _eligible(self, t: torch.Tensor) -> bool:
        return (t.is_cuda and t.dtype in (torch.float32, torch.bfloat16) and t.numel() >= self.min_numel
                and not isinstance(t, torch.nn.Parameter) and int(t.data_ptr()) not in self._exclude)

    def _pack(self, t: torch.Tensor):
        if not self._eligible(t):
            return t
        x = t.detach().contiguous()
        if x.data_ptr() % 16:                     # a contiguous view at an odd storage offset: the kernels want 16-byte alignment
            x = x.clone()
        tid = self.next_tensor_id
        self.next_tensor_id += 1
        if self.batch_bytes > 0:
            d = _Deferred(x, tid, t.shape, t.dtype, self._split(x))
            self._pending.append(d)
            self._pending_bytes += x.numel() * x.element_size()
            if self._pending_bytes >= self.batch_bytes:
                self.flush()
            return d
        stream = torch.cuda.current_stream(x.device)
        rec = None
        if self.record:
            ev = (torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
            ev[0].record(stream)
        mixed, extra = self._split(x), 0
        if mixed is None:
            packed, meta = api.fh_compress(x.view(-1), self.group_size, self.bits, self.rounding, self.seed, tid,
                                           stream=stream)
        else:
            outer, channels, inner, raw_channels = mixed
            min_outliers = max(1, int(outer * inner * self.outlier_share))
            _, _, mask = api.fh_classify_channels(x.view(-1), outer, channels, inner, self.k_sigma, min_outliers,
                                                  stream=stream)
            used = torch.empty(1, dtype=torch.int64, device=x.device)
            slots = api.fh_channel_slots(mask, raw_channels, stream=stream, used=used)
            # a tensor in which the classification finds nothing salient (most layers) takes the plain
            # quantiser's code path inside the same launch: `used` tells the kernels on the device
            packed, meta, raw = api.fh_compress_mixed(x.view(-1), outer, channels, inner, slots, raw_channels,
                                                      self.group_size, self.bits, self.rounding, self.seed, tid,
                                                      stream=stream, rows_in_use=used)
            mixed = (outer, channels, inner, slots, raw_channels, raw, used)
            extra = raw.numel() * raw.element_size() + slots.numel() * slots.element_size()
        if self.record:
            ev[1].record(stream)
            rec = TensorRecord(tid, x.numel(), x.dtype, x.numel() * x.element_size(),
                               packed.numel() + meta.numel() * meta.element_size() + extra, _pack=ev)
            self.records.append(rec)
        return _Packed(packed, meta, t.shape, t.dtype, x.numel(), rec, mixed)

    def flush(self) -> None:
        """Compress every tensor that waits for its batch (batched entry points, current stream)."""
        pending, self._pending, self._pending_bytes = self._pending, [], 0
        if not pending:
            return
        stream = torch.cuda.current_stream(pending[0].x.device)
        ev = None
        if self.record:
            ev = (torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
            ev[0].record(stream)
        plain = [d for d in pending if d.split is None]
        routed = [d for d in pending if d.split is not None]
        stored = {}
        if plain:
            entries = []
            for d in plain:
                packed, meta = api.alloc_compressed(d.x.numel(), self.group_size, self.bits, d.x.device)
                entries.append(api.BatchEntry(self.group_size, self.bits, self.rounding, self.seed, d.tid,
                                              x=d.x.view(-1), packed=packed, meta=meta))
            api.fh_compress_batch(api.Batch(entries), stream)
            for d, e in zip(plain, entries):
                d.handle = _Packed(e.packed, e.meta, d.shape, d.dtype, d.x.numel(), None)
                stored[id(d)] = e.packed.numel() + e.meta.numel() * e.meta.element_size()
        if routed:
            cls = api.ClassifyBatch([api.ClassifyEntry(d.x.view(-1), d.split[0], d.split[1], d.split[2], self.k_sigma,
                                                       max(1, int(d.split[0] * d.split[2] * self.outlier_share)))
                                     for d in routed])
            api.fh_classify_channels_batch(cls, stream)
            slots, used = api.fh_channel_slots_batch([e.mask for e in cls.entries], [d.split[3] for d in routed], stream)
            mixed = api.MixedBatch([api.MixedEntry(d.split[0], d.split[1], d.split[2], slots[k], d.split[3],
                                                   self.group_size, self.bits, self.rounding, self.seed, d.tid,
                                                   x=d.x.view(-1), rows_in_use=used[k])
                                    for k, d in enumerate(routed)])
            api.fh_compress_mixed_batch(mixed, stream)
            for k, (d, e) in enumerate(zip(routed, mixed.entries)):
                outer, channels, inner, raw_channels = d.split
                d.handle = _Packed(e.packed, e.meta, d.shape, d.dtype, d.x.numel(), None,
                                   (outer, channels, inner, slots[k], raw_channels, e.raw, used[k]))
                stored[id(d)] = (e.packed.numel() + e.meta.numel() * e.meta.element_size()
                                 + e.raw.numel() * e.raw.element_size() + slots[k].numel() * 2)
        if ev is not None:
            ev[1].record(stream)
            total = float(sum(d.x.numel() * d.x.element_size() for d in pending))
            for d in pending:
                nbytes = d.x.numel() * d.x.element_size()
                d.handle.record = TensorRecord(d.tid, d.x.numel(), d.x.dtype, nbytes, stored[id(d)],
                                               _pack=(ev[0], ev[1], nbytes / total))
                self.records.append(d.handle.record)
        for d in pending:
            d.x = None                                        # the activation itself may go now

    def __exit__(self, *exc):
        self.flush()
        return super().__exit__(*exc)

    def _split(self, x: torch.Tensor):
        """(outer, channels, inner, raw_channels) of the channel-wise path, or None for the plain one."""
        if self.channel_dim is None or x.dim() == 0 or x.numel() > 2 ** 31:
            return None
        d = self.channel_dim % x.dim()
        channels = x.shape[d]
        if not 1 <= channels <= 16384:
            return None
        outer = 1
        for n in x.shape[:d]:
            outer *= n
        inner = x.numel() // (outer * channels)
        return outer, channels, inner, max(1, min(channels, int(channels * self.raw_share + 0.5)))

    def _unpack(self, h):
        if isinstance(h, _Deferred):
            if h.handle is None:
                self.flush()                                  # needed back before its batch was full
            h = h.handle
        if not isinstance(h, _Packed):
            return h
        stream = torch.cuda.current_stream(h.packed.device)
        if h.record is not None:
            ev = (torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
            ev[0].record(stream)
        if h.mixed is None:
            out = api.fh_decompress(h.packed, h.meta, h.numel, self.group_size, self.bits, out_dtype=h.dtype,
                                    stream=stream)
        else:
            outer, channels, inner, slots, raw_channels, raw, used = h.mixed
            out = api.fh_decompress_mixed(h.packed, h.meta, raw, outer, channels, inner, slots, raw_channels,
                                          self.group_size, self.bits, out_dtype=h.dtype, stream=stream, rows_in_use=used)
        if h.record is not None:
            ev[1].record(stream)
            h.record._unpack = ev
        return out.view(h.shape)
