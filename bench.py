#!/usr/bin/env python3
"""Benchmark of the activation compress + decompress round trip on one MI355X.

A step is one pass of the whole hot path over one tensor set: every tensor is
compressed (range statistics, quantisation, bit-packing) and then decompressed
(unpack, fused dequantise) through the batched C-ABI entry points, with the inputs
already resident in device memory.  The default workload is the mixed-plan 2 GiB
stress set (48 fp32 tensors, per-tensor 2/4/8 bits, nearest or stochastic rounding).

Prints one JSON line: whole-job input GB/s, the roofline of the dominant kernel
(algorithmic bytes / event-timed duration vs the 8 TB/s HBM peak) and the CPU oracle
timed on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0      # MI355X HBM3E, published peak


def algorithmic_bytes(spec, out_itemsize=4):
    """(compress bytes, decompress bytes) one tensor moves: input read + codes and
    meta written; codes and meta read + output written."""
    n = spec.numel
    codes = (n * spec.bits + 7) // 8
    meta = 8 * ((n + spec.group_size - 1) // spec.group_size)
    return n * spec.itemsize + codes + meta, codes + meta + n * out_itemsize


def host_threads() -> int:
    """Threads the CPU baseline may use: the cores this process may run on, capped by the
    box's stated share (OMP_NUM_THREADS) where one is set."""
    n = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)
    cap = os.environ.get("OMP_NUM_THREADS", "")
    if cap.isdigit() and int(cap) > 0:
        n = min(n, int(cap))
    return max(1, n)


def run_on_threads(fn, jobs, threads) -> float:
    """Wall-clock seconds to run fn(job) for every job on `threads` host threads (the oracle is
    called through ctypes, which releases the interpreter lock; each call is the untouched
    single-threaded oracle on a whole tensor)."""
    from concurrent.futures import ThreadPoolExecutor
    with ThreadPoolExecutor(max_workers=threads) as pool:
        t0 = time.perf_counter()
        list(pool.map(fn, jobs))
        return time.perf_counter() - t0


def counted(fn):
    """fn with a call counter (`calls`): how many steps a run executed in all, which is what a
    per-dispatch counter total of the same run has to be divided by."""
    def wrapper(*a, **k):
        wrapper.calls += 1
        return fn(*a, **k)
    wrapper.calls = 0
    return wrapper


def copy_calibration(n, dev):
    """n plain 1 GiB device copies: a rocprofv3 --pmc run scales FETCH_SIZE / WRITE_SIZE by what
    the same counters read for them."""
    import torch
    if n <= 0:
        return
    src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
    dst = torch.empty_like(src)
    for _ in range(n):
        dst.copy_(src)                          # reads 1 GiB, writes 1 GiB
    torch.cuda.synchronize()


COLD_PROTOCOL = ("cold: memory-side cache displaced by an untimed 1 GiB read pass before each of the two calls; "
                 "step time = the two calls' own HIP-event intervals")


def time_two_sided(args, dev, stream, forward, backward) -> dict:
    """The round trip's protocol for any op with two sides (encode / decode, compress / restore): what the
    first side wrote is not cached when the second runs -- a training step restores long after it saved --,
    so an untimed pass over 1 GiB displaces the memory-side cache before either, and a step's time is the sum
    of the two calls' own event intervals.  The back-to-back figure (no displacing pass, wall clock over the
    loop) is measured too unless --headline-only.  -> {c_ms, d_ms, wall_ms | None, calls}"""
    import torch
    scrub = torch.zeros(1 << 28, dtype=torch.int32, device=dev)
    calls = 0

    def step(ev=None, displace=True):
        nonlocal calls
        calls += 1
        if displace:
            torch.amax(scrub)
        if ev:
            ev[0].record(stream)
        forward()
        if ev:
            ev[1].record(stream)
        if displace:
            torch.amax(scrub)
        if ev:
            ev[2].record(stream)
        backward()
        if ev:
            ev[3].record(stream)

    for _ in range(args.warmup):
        step()
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    for k in range(args.steps):
        step(evs[k])
    torch.cuda.synchronize()
    c_ms = sum(e[0].elapsed_time(e[1]) for e in evs) / args.steps
    d_ms = sum(e[2].elapsed_time(e[3]) for e in evs) / args.steps
    wall_ms = None
    if not args.headline_only:
        step(None, False)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step(None, False)
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t0) / args.steps * 1e3
    del scrub
    return {"c_ms": c_ms, "d_ms": d_ms, "wall_ms": wall_ms, "calls": calls}


def bench_classify(args, api, W, dev) -> dict:
    """Channel classification (three-sigma outliers, salient channels) over MobileNetV2-style
    NCHW activations at batch 64 with channel-clustered outliers; one step classifies every
    tensor of the set once (one batched call; --per-tensor: one call per tensor).  Two streaming
    passes read each tensor twice."""
    import numpy as np
    import torch

    shapes = ((64, 32, 112 * 112), (64, 96, 112 * 112), (64, 144, 56 * 56), (64, 192, 28 * 28), (64, 384, 14 * 14))
    t0 = time.time()
    host, jobs = [], []
    for i, (outer, C, inner) in enumerate(shapes):
        x, _ = W.outlier_channel_tensor(outer, C, inner, seed=i, dist="relu")
        host.append(x)
        xd = torch.from_numpy(x).to(dev)
        ws = torch.empty(api.classify_workspace_bytes(x.size), dtype=torch.uint8, device=dev)
        stats = torch.empty(4, dtype=torch.float64, device=dev)
        counts = torch.empty(C, dtype=torch.int32, device=dev)
        mask = torch.empty(C, dtype=torch.uint8, device=dev)
        jobs.append((xd, outer, C, inner, outer * inner // 100, ws, stats, counts, mask))
    torch.cuda.synchronize()
    nbytes = sum(x.nbytes for x in host)
    print(f"[bench] classify: {len(jobs)} tensors, {nbytes / 2**20:.1f} MiB resident "
          f"(generated + uploaded in {time.time() - t0:.1f} s)", file=sys.stderr, flush=True)
    stream = torch.cuda.current_stream()

    batch = api.ClassifyBatch([api.ClassifyEntry(xd, outer, C, inner, 3.0, mo, ws, stats, counts, mask)
                               for xd, outer, C, inner, mo, ws, stats, counts, mask in jobs])

    @counted
    def step():
        if args.per_tensor:
            for xd, outer, C, inner, mo, ws, stats, counts, mask in jobs:
                api.fh_classify_channels(xd, outer, C, inner, 3.0, mo, workspace=ws, stats=stats, counts=counts,
                                         mask=mask, stream=stream)
        else:
            api.fh_classify_channels_batch(batch, stream)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = (time.perf_counter() - t_start) / args.steps
    alg = 2 * nbytes                            # each pass reads the tensor once; outputs are negligible
    result = {
        "metric": "channel classification GB/s of input and % of HBM peak on 1 MI355X",
        "value": round(nbytes / elapsed / 1e9, 2), "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(elapsed * 1e3, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f64", "data": "synthetic",
        "config": {"workload": "classify_mobilenetv2_b64_outlier_channels", "tensors": len(jobs),
                   "input_bytes": nbytes, "k_sigma": 3.0,
                   "entry_point": "fh_classify_channels (per tensor)" if args.per_tensor else "fh_classify_channels_batch"},
        "algorithmic_bytes_per_step": alg, "steps_executed": step.calls,
        "roofline": {"bound": "hbm", "kernel": "moments + count passes (whole call)",
                     "achieved": round(alg / elapsed / 1e9, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(alg / elapsed / 1e9 / HBM_PEAK_GBS, 4), "traffic": None},
    }
    if not args.no_cpu_baseline:
        import oracle
        t_cpu, done = 0.0, 0
        for x, (outer, C, inner) in zip(host, shapes):
            t1 = time.perf_counter()
            oracle.classify_channels(x, outer, C, inner, 3.0, outer * inner // 100)
            t_cpu += time.perf_counter() - t1
            done += x.nbytes
            if t_cpu > 20.0:
                break
        result["cpu_baseline"] = {"value": round(done / t_cpu / 1e9, 4), "unit": "GB/s", "cores": 1, "kind": "oracle",
                                  "sample": f"{done / 2**20:.1f} MiB of the set, whole tensors, {t_cpu:.1f} s"}
    return result


def bench_mixed(args, api, W, dev) -> dict:
    """Compress + decompress with salient channels routed around the quantiser, over the same
    MobileNetV2-style activations with channel-clustered outliers as the classification
    bench, or (--config 4) over the transformer set with outliers planted in 4 % of the hidden
    channels (the planted channels are the kept ones; slot tables are built once, outside the
    timed region).  One step = every tensor compressed, then every tensor restored."""
    import numpy as np
    import torch

    if args.config == 4:                                      # transformer activations, one channel per element
        shapes = tuple(s for _ in range(12) for s in ((16 * 512, 768, 1), (16 * 512, 3072, 1)))
        G, B, rounding, dtype, dist = 64, 2, "stochastic", "bf16", ("gauss", "gelu")
        workload = "mixed_transformer_l12_b16_s512_bf16_outlier_channels_g64_b2_stochastic"
    else:
        shapes = ((64, 32, 112 * 112), (64, 96, 112 * 112), (64, 144, 56 * 56), (64, 192, 28 * 28), (64, 384, 14 * 14))
        G, B, rounding, dtype, dist = 128, 4, "nearest", "f32", ("relu", "relu")
        workload = "mixed_mobilenetv2_b64_outlier_channels_g128_b4_nearest"
    tdtype = torch.bfloat16 if dtype == "bf16" else torch.float32
    esize = 2 if dtype == "bf16" else 4
    t0 = time.time()
    host, jobs = [], []
    alg_c = alg_d = 0
    for i, (outer, C, inner) in enumerate(shapes):
        x, planted = W.outlier_channel_tensor(outer, C, inner, seed=i, dist=dist[i % 2], dtype=dtype)
        mask = np.zeros(C, np.uint8)
        mask[planted] = 1
        cap = len(planted)
        host.append((x, mask, cap))
        xd = torch.from_numpy(x.view(np.int16) if dtype == "bf16" else x).to(dev)
        if dtype == "bf16":
            xd = xd.view(torch.bfloat16)
        slots = api.fh_channel_slots(torch.from_numpy(mask).to(dev), cap)
        packed, meta = api.alloc_compressed(x.size, G, B, dev)
        raw = torch.empty(outer * cap * inner, dtype=tdtype, device=dev)
        out = torch.empty(x.size, dtype=tdtype, device=dev)
        jobs.append((xd, outer, C, inner, slots, cap, packed, meta, raw, out, i))
        n = x.size
        side = (n * B + 7) // 8 + 8 * ((n + G - 1) // G) + outer * cap * inner * esize
        alg_c += n * esize + side
        alg_d += side + n * esize
    torch.cuda.synchronize()
    nbytes = sum(x.nbytes for x, _, _ in host)
    print(f"[bench] mixed: {len(jobs)} tensors, {nbytes / 2**20:.1f} MiB resident "
          f"(generated + uploaded in {time.time() - t0:.1f} s)", file=sys.stderr, flush=True)
    stream = torch.cuda.current_stream()

    batch = api.MixedBatch([api.MixedEntry(outer, C, inner, slots, cap, G, B, rounding, 1, tid, x=xd, packed=packed,
                                           meta=meta, raw=raw, out=out)
                            for xd, outer, C, inner, slots, cap, packed, meta, raw, out, tid in jobs])

    def forward():
        if args.per_tensor:
            for xd, outer, C, inner, slots, cap, packed, meta, raw, out, tid in jobs:
                api.fh_compress_mixed(xd, outer, C, inner, slots, cap, G, B, rounding, 1, tid, packed=packed,
                                      meta=meta, raw=raw, stream=stream)
        else:
            api.fh_compress_mixed_batch(batch, stream)

    def backward():
        if args.per_tensor:
            for xd, outer, C, inner, slots, cap, packed, meta, raw, out, tid in reversed(jobs):
                api.fh_decompress_mixed(packed, meta, raw, outer, C, inner, slots, cap, G, B, out=out, stream=stream)
        else:
            api.fh_decompress_mixed_batch(batch, stream)

    t = time_two_sided(args, dev, stream, forward, backward)
    ms_c, ms_d = t["c_ms"], t["d_ms"]
    elapsed = (ms_c + ms_d) * 1e-3
    dom = ("compress_mixed_kernel", alg_c, ms_c) if ms_c >= ms_d else ("decompress_mixed_kernel", alg_d, ms_d)
    result = {
        "metric": "activation compress+decompress GB/s with salient channels kept raw, on 1 MI355X",
        "value": round(nbytes / elapsed / 1e9, 2), "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(elapsed * 1e3, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": dtype, "data": "synthetic",
        "config": {"workload": workload, "tensors": len(jobs),
                   "input_bytes": nbytes,
                   "entry_point": ("fh_compress_mixed + fh_decompress_mixed (per tensor)" if args.per_tensor
                                   else "fh_compress_mixed_batch + fh_decompress_mixed_batch"),
                   "kept_channels": [int(c) for _, _, c in host], "protocol": COLD_PROTOCOL},
        "round_trip_algorithmic_bytes": alg_c + alg_d,
        "algorithmic_bytes_per_step": alg_c + alg_d, "steps_executed": t["calls"],
        "back_to_back": None if t["wall_ms"] is None else {
            "ms_per_step": round(t["wall_ms"], 4), "value": round(nbytes / t["wall_ms"] / 1e6, 2),
            "hbm_frac_round_trip": round((alg_c + alg_d) / t["wall_ms"] / 1e6 / HBM_PEAK_GBS, 4), "clock": "wall, launches included"},
        "hbm_frac_round_trip": round((alg_c + alg_d) / elapsed / 1e9 / HBM_PEAK_GBS, 4),
        "roofline": {"bound": "hbm", "kernel": dom[0] + " (event-timed)",
                     "achieved": round(dom[1] / dom[2] / 1e6, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(dom[1] / dom[2] / 1e6 / HBM_PEAK_GBS, 4), "traffic": None},
        "kernels": {"compress_mixed_kernel": {"ms": round(ms_c, 4), "bytes": alg_c,
                                              "GBps": round(alg_c / ms_c / 1e6, 1)},
                    "decompress_mixed_kernel": {"ms": round(ms_d, 4), "bytes": alg_d,
                                                "GBps": round(alg_d / ms_d / 1e6, 1)}},
    }
    if not args.no_cpu_baseline:
        import oracle
        t_cpu, done = 0.0, 0
        for (x, mask, cap), (outer, C, inner) in zip(host, shapes):
            t1 = time.perf_counter()
            slots, _ = oracle.channel_slots(mask, cap)
            p, m, r = oracle.compress_mixed(x, outer, C, inner, slots, cap, G, B, rounding, 1, 0, dtype=dtype)
            oracle.decompress_mixed(p, m, r, outer, C, inner, slots, cap, G, B, raw_dtype=dtype, out_dtype=dtype)
            t_cpu += time.perf_counter() - t1
            done += x.nbytes
            if t_cpu > 20.0:
                break
        result["cpu_baseline"] = {"value": round(done / t_cpu / 1e9, 4), "unit": "GB/s", "cores": 1, "kind": "oracle",
                                  "sample": f"{done / 2**20:.1f} MiB of the set, whole tensors, {t_cpu:.1f} s"}
    return result


def bench_sparse(args, api, W, dev) -> dict:
    """Sparse-block storage of salient-channel feature maps (non-zero mask, n x n average
    pooling against tau, CSR for sparse blocks): the kept channels (4 %) of the MobileNetV2-style
    set at batch 64, post-ReLU with clustered zeros.  One step = every map set encoded, then
    every one decoded."""
    import numpy as np
    import torch

    layers = ((64 * 1, 112, 112), (64 * 4, 112, 112), (64 * 6, 56, 56), (64 * 8, 28, 28), (64 * 15, 14, 14))
    layers = tuple((maps * args.maps_scale, h, w) for maps, h, w in layers)
    n, tau, eps = 4, 0.5, args.eps
    t0 = time.time()
    host, jobs = [], []
    for i, (maps, h, w) in enumerate(layers):
        x = W.salient_feature_maps(maps, h, w, seed=i)
        host.append(x)
        xd = torch.from_numpy(x).to(dev)
        bufs = api.alloc_sparse(maps, h, w, n, torch.float32, dev)
        out = torch.empty(x.size, dtype=torch.float32, device=dev)
        jobs.append([xd, maps, h, w, bufs, out, None])
    stream = torch.cuda.current_stream()
    for job in jobs:                                          # stream sizes (fixed: the input is)
        xd, maps, h, w, bufs, out, _ = job
        api.fh_sparse_encode(xd, maps, h, w, n, tau, buffers=bufs, stream=stream, eps=eps)
    torch.cuda.synchronize()
    stored = 0
    for job in jobs:
        nv, ni, ns, nd = (int(v) for v in job[4].totals.cpu().tolist())
        job[6] = (job[4].values[:nv], job[4].indices[:ni])
        stored += nv * 4 + ni + job[4].info.numel()
    nbytes = sum(x.nbytes for x in host)
    print(f"[bench] sparse: {len(jobs)} map sets, {nbytes / 2**20:.1f} MiB resident, stored {stored / 2**20:.1f} MiB "
          f"(generated + uploaded in {time.time() - t0:.1f} s)", file=sys.stderr, flush=True)

    batch = api.SparseBatch([api.SparseEntry(maps, h, w, n, tau, eps, x=xd, buffers=bufs, values=vals, indices=idx,
                                             out=out) for xd, maps, h, w, bufs, out, (vals, idx) in jobs])

    def forward():
        if args.per_tensor:
            for xd, maps, h, w, bufs, out, _ in jobs:
                api.fh_sparse_encode(xd, maps, h, w, n, tau, buffers=bufs, stream=stream, eps=eps)
        else:
            api.fh_sparse_encode_batch(batch, stream)

    def backward():
        if args.per_tensor:
            for xd, maps, h, w, bufs, out, (vals, idx) in jobs:
                api.fh_sparse_decode(bufs.info, vals, idx, maps, h, w, n, out=out, workspace=bufs.workspace,
                                     stream=stream, eps=eps)
        else:
            api.fh_sparse_decode_batch(batch, stream)

    t = time_two_sided(args, dev, stream, forward, backward)
    ms_e, ms_d = t["c_ms"], t["d_ms"]
    elapsed = (ms_e + ms_d) * 1e-3
    info_bytes = sum(job[4].info.numel() for job in jobs)
    alg_e = 2 * nbytes + stored + info_bytes                  # two passes over the input, info re-read, streams written
    alg_d = 2 * info_bytes + stored + nbytes                  # info read twice, streams read, maps written
    dom = ("encode (count + scan + write)", alg_e, ms_e) if ms_e >= ms_d else ("decode (sums + scan + read)", alg_d, ms_d)
    result = {
        "metric": "sparse-block storage of salient-channel maps, encode+decode GB/s of input on 1 MI355X",
        "value": round(nbytes / elapsed / 1e9, 2), "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(elapsed * 1e3, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "u32", "data": "synthetic",
        "config": {"workload": "sparse_mobilenetv2_b64_kept_channels_n4_tau0.5" + (f"_eps{eps:g}" if eps > 0 else "")
                   + (f"_x{args.maps_scale}" if args.maps_scale != 1 else ""),
                   "map_sets": len(jobs), "input_bytes": nbytes, "stored_bytes": stored,
                   "entry_point": ("fh_sparse_encode + fh_sparse_decode (per set)" if args.per_tensor
                                   else "fh_sparse_encode_batch + fh_sparse_decode_batch"),
                   "window": n, "tau": tau, "eps": eps, "protocol": COLD_PROTOCOL},
        "algorithmic_bytes_per_step": alg_e + alg_d, "steps_executed": t["calls"],
        "hbm_frac_round_trip": round((alg_e + alg_d) / elapsed / 1e9 / HBM_PEAK_GBS, 4),
        "back_to_back": None if t["wall_ms"] is None else {
            "ms_per_step": round(t["wall_ms"], 4), "value": round(nbytes / t["wall_ms"] / 1e6, 2), "clock": "wall, launches included"},
        "roofline": {"bound": "hbm", "kernel": dom[0] + ", all launches of a step, event-timed",
                     "achieved": round(dom[1] / dom[2] / 1e6, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(dom[1] / dom[2] / 1e6 / HBM_PEAK_GBS, 4), "traffic": None},
        "kernels": {"encode": {"ms": round(ms_e, 4), "bytes": alg_e, "GBps": round(alg_e / ms_e / 1e6, 1)},
                    "decode": {"ms": round(ms_d, 4), "bytes": alg_d, "GBps": round(alg_d / ms_d / 1e6, 1)}},
    }
    if not args.no_cpu_baseline:
        import oracle
        t_cpu, done = 0.0, 0
        for x, (maps, h, w) in zip(host, layers):
            t1 = time.perf_counter()
            info, v, idx, _ = oracle.sparse_encode(x, maps, h, w, n, tau, eps=eps)
            oracle.sparse_decode(info, v, idx, maps, h, w, n, eps=eps)
            t_cpu += time.perf_counter() - t1
            done += x.nbytes
            if t_cpu > 20.0:
                break
        result["cpu_baseline"] = {"value": round(done / t_cpu / 1e9, 4), "unit": "GB/s", "cores": 1, "kind": "oracle",
                                  "sample": f"{done / 2**20:.1f} MiB of the set, whole map sets, {t_cpu:.1f} s"}
    return result


def bench_huffman(args, api, W, dev) -> dict:
    """The entropy stage of the predictive form (Section 4.4.1: Huffman coding of the quantisation
    codes): the index streams -- code bytes of dense blocks, CSR bytes of sparse ones -- that
    fh_sparse_encode writes for the sparse bench's map sets with an error bound (--eps, default
    0.02 here; --maps-scale K times as many maps).  One step = every stream encoded, then every
    one decoded."""
    import numpy as np
    import torch

    layers = ((64 * 1, 112, 112), (64 * 4, 112, 112), (64 * 6, 56, 56), (64 * 8, 28, 28), (64 * 15, 14, 14))
    layers = tuple((maps * args.maps_scale, h, w) for maps, h, w in layers)
    n, tau, eps = 4, 0.5, (args.eps if args.eps > 0 else 0.02)
    stream = torch.cuda.current_stream()
    jobs, host = [], []
    for i, (maps, h, w) in enumerate(layers):
        x = torch.from_numpy(W.salient_feature_maps(maps, h, w, seed=i)).to(dev)
        bufs = api.fh_sparse_encode(x, maps, h, w, n, tau, stream=stream, eps=eps)
        torch.cuda.synchronize()
        ni = int(bufs.totals[1])
        data = bufs.indices[:ni].clone()
        host.append(data.cpu().numpy())
        out = torch.empty(api.huffman_stream_bytes(ni), dtype=torch.uint8, device=dev)
        totals = torch.zeros(2, dtype=torch.int64, device=dev)
        ws = torch.empty(api.huffman_workspace_bytes(ni), dtype=torch.uint8, device=dev)
        api.fh_huffman_encode(data, stream_out=out, totals=totals, workspace=ws, stream=stream)
        torch.cuda.synchronize()
        used = int(totals[0])
        jobs.append((data, ni, out, totals, ws, used, torch.empty(ni, dtype=torch.uint8, device=dev)))
        del x, bufs
    nbytes = sum(j[1] for j in jobs)
    stored = sum(j[5] for j in jobs)
    print(f"[bench] huffman: {len(jobs)} streams, {nbytes / 2**20:.1f} MiB of index bytes, stored {stored / 2**20:.1f} MiB",
          file=sys.stderr, flush=True)

    batch = api.HuffmanBatch([j[0] for j in jobs])
    api.fh_huffman_encode_batch(batch, stream)
    torch.cuda.synchronize()
    batch.refresh()                                           # stream sizes (fixed: the input is)

    def forward():
        if args.per_tensor:
            for data, ni, out, totals, ws, used, back in jobs:
                api.fh_huffman_encode(data, stream_out=out, totals=totals, workspace=ws, stream=stream)
        else:
            api.fh_huffman_encode_batch(batch, stream)

    def backward():
        if args.per_tensor:
            for data, ni, out, totals, ws, used, back in jobs:
                api.fh_huffman_decode(out[:used], ni, out=back, stream=stream)
        else:
            api.fh_huffman_decode_batch(batch, stream)

    t = time_two_sided(args, dev, stream, forward, backward)
    ms_e, ms_d = t["c_ms"], t["d_ms"]
    elapsed = (ms_e + ms_d) * 1e-3
    for k, (data, ni, out, totals, ws, used, back) in enumerate(jobs):
        if not torch.equal(back if args.per_tensor else batch.out[k], data):
            raise RuntimeError("the Huffman round trip did not restore its input")
    alg_e = 3 * nbytes + stored                               # histogram, count and write passes read the bytes
    alg_d = stored + nbytes
    dom = ("encode (histogram + code + count + scan + write)", alg_e, ms_e) if ms_e >= ms_d else ("decode", alg_d, ms_d)
    result = {
        "metric": "Huffman coding of the predictive form's index streams, encode+decode GB/s of input on 1 MI355X",
        "value": round(nbytes / elapsed / 1e9, 2), "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(elapsed * 1e3, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "u8", "data": "synthetic",
        "config": {"workload": f"huffman_index_streams_mobilenetv2_b64_kept_channels_n4_tau0.5_eps{eps:g}_x{args.maps_scale}",
                   "streams": len(jobs), "input_bytes": nbytes, "stored_bytes": stored,
                   "entry_point": ("fh_huffman_encode + fh_huffman_decode (per stream)" if args.per_tensor
                                   else "fh_huffman_encode_batch + fh_huffman_decode_batch"), "protocol": COLD_PROTOCOL},
        "algorithmic_bytes_per_step": alg_e + alg_d, "steps_executed": t["calls"],
        "hbm_frac_round_trip": round((alg_e + alg_d) / elapsed / 1e9 / HBM_PEAK_GBS, 4),
        "back_to_back": None if t["wall_ms"] is None else {
            "ms_per_step": round(t["wall_ms"], 4), "value": round(nbytes / t["wall_ms"] / 1e6, 2), "clock": "wall, launches included"},
        "roofline": {"bound": "hbm", "kernel": dom[0] + ", all launches of a step, event-timed",
                     "achieved": round(dom[1] / dom[2] / 1e6, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(dom[1] / dom[2] / 1e6 / HBM_PEAK_GBS, 4), "traffic": None},
        "kernels": {"encode": {"ms": round(ms_e, 4), "bytes": alg_e, "GBps": round(alg_e / ms_e / 1e6, 1)},
                    "decode": {"ms": round(ms_d, 4), "bytes": alg_d, "GBps": round(alg_d / ms_d / 1e6, 1)}},
    }
    if not args.no_cpu_baseline:
        import oracle
        t_cpu, done = 0.0, 0
        for data in host:
            sample = data[: 1 << 24]
            t1 = time.perf_counter()
            st, _ = oracle.huffman_encode(sample)
            oracle.huffman_decode(st, sample.size)
            t_cpu += time.perf_counter() - t1
            done += sample.size
            if t_cpu > 20.0:
                break
        result["cpu_baseline"] = {"value": round(done / t_cpu / 1e9, 4), "unit": "GB/s", "cores": 1, "kind": "oracle",
                                  "sample": f"leading {done / 2**20:.1f} MiB of the streams, {t_cpu:.1f} s"}
    return result


def bench_chain(args, api, W, dev) -> dict:
    """The whole channel-wise mix compressor (Section 4.4.1 end to end; Algorithm 1's compress and
    decompress actions) through fh_mix_compress_batch / fh_mix_decompress_batch: classification,
    routed quantiser, sparse / predictive storage of the salient channels' maps, Huffman stage,
    and back.  Workload: the MobileNetV2-style set at batch 64 (G128, 4-bit, nearest) or, with
    --config 4, the transformer set (bf16, G64, 2-bit, stochastic), each with outliers planted in
    4 % of the channels; room for 1/16 of the channels in the raw store; window 4, tau 0.5,
    error bound --eps (default 0.02).  Cold protocol as for the plain round trip."""
    import numpy as np
    import torch
    sys.path.insert(0, os.path.join(ROOT, "tests"))

    if args.config == 4:
        shapes = tuple(s for _ in range(12) for s in ((16 * 512, 768, 1, None), (16 * 512, 3072, 1, None)))
        G, B, rounding, dtype, dist = 64, 2, "stochastic", "bf16", ("gauss", "gelu")
        workload = "chain_transformer_l12_b16_s512_bf16_outlier_channels_g64_b2_stochastic"
    else:
        shapes = ((64, 32, 112 * 112, (112, 112)), (64, 96, 112 * 112, (112, 112)), (64, 144, 56 * 56, (56, 56)),
                  (64, 192, 28 * 28, (28, 28)), (64, 384, 14 * 14, (14, 14)))
        G, B, rounding, dtype, dist = 128, 4, "nearest", "f32", ("relu", "relu")
        workload = "chain_mobilenetv2_b64_outlier_channels_g128_b4_nearest"
    eps = args.eps if args.eps > 0 else 0.02
    window, tau, entropy = 4, 0.5, 1
    tdtype = torch.bfloat16 if dtype == "bf16" else torch.float32
    esize = 2 if dtype == "bf16" else 4
    t0 = time.time()
    host, entries = [], []
    for i, (outer, C, inner, hw) in enumerate(shapes):
        x, planted = W.outlier_channel_tensor(outer, C, inner, seed=i, dist=dist[i % 2], dtype=dtype)
        cap = max(1, C // 16)
        maps, h, w = (outer * cap, hw[0], hw[1]) if hw else (1, outer, cap)
        min_out = max(1, outer * inner // 100)
        host.append((x, outer, C, inner, cap, maps, h, w, min_out, i))
        xd = torch.from_numpy(x.view(np.int16) if dtype == "bf16" else x).to(dev)
        if dtype == "bf16":
            xd = xd.view(torch.bfloat16)
        entries.append(api.MixEntry(outer, C, inner, cap, G, B, rounding, seed=1, tensor_id=i, k_sigma=3.0,
                                    min_outliers=min_out, maps=maps, h=h, w=w, window=window, tau=tau, eps=eps,
                                    entropy=entropy, x=xd, out=torch.empty(x.size, dtype=tdtype, device=dev)))
    batch = api.MixBatch(entries, device=dev)
    torch.cuda.synchronize()
    nbytes = sum(h[0].nbytes for h in host)
    print(f"[bench] chain: {len(entries)} tensors, {nbytes / 2**20:.1f} MiB resident, stores "
          f"{sum(r.store_bytes for r in batch.regions) / 2**20:.1f} MiB + workspaces "
          f"{sum(r.workspace_bytes for r in batch.regions) / 2**20:.1f} MiB allotted "
          f"(generated + uploaded in {time.time() - t0:.1f} s)", file=sys.stderr, flush=True)
    stream = torch.cuda.current_stream()
    scrub = torch.zeros(1 << 28, dtype=torch.int32, device=dev)

    @counted
    def step(ev=None, displace=True):
        if displace:
            torch.amax(scrub)
        if ev:
            ev[0].record(stream)
        api.fh_mix_compress_batch(batch, stream)
        if ev:
            ev[1].record(stream)
        if displace:
            torch.amax(scrub)
        if ev:
            ev[2].record(stream)
        api.fh_mix_decompress_batch(batch, stream)
        if ev:
            ev[3].record(stream)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    headers = [batch.header(i).cpu().tolist() for i in range(batch.count)]
    stored = sum(int(h[6]) for h in headers)
    kept_rows = [int(h[7]) for h in headers]

    def timed(displace):
        evs = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
        torch.cuda.synchronize()
        for k in range(args.steps):
            step(evs[k], displace)
        torch.cuda.synchronize()
        return (sum(e[0].elapsed_time(e[1]) for e in evs) / args.steps,
                sum(e[2].elapsed_time(e[3]) for e in evs) / args.steps)

    c_ms, d_ms = timed(True)
    cw_ms, dw_ms = timed(False)
    # what the method has to move: the tensor read three times on the way in (moments, outlier
    # counts -- which need the moments --, quantiser -- which needs the mask), the stored form
    # written; the stored form read and the tensor written on the way back
    alg_c, alg_d = 3 * nbytes + stored, stored + nbytes
    step_ms = c_ms + d_ms
    dom = ("fh_mix_compress_batch", alg_c, c_ms) if c_ms >= d_ms else ("fh_mix_decompress_batch", alg_d, d_ms)
    result = {
        "metric": "whole channel-wise mix compressor, compress+decompress GB/s of input on 1 MI355X",
        "value": round(nbytes / step_ms / 1e6, 2), "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(step_ms, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": dtype, "data": "synthetic",
        "config": {"workload": workload, "tensors": len(entries), "input_bytes": nbytes,
                   "entry_point": "fh_mix_compress_batch + fh_mix_decompress_batch",
                   "window": window, "tau": tau, "eps": eps, "entropy": "huffman", "raw_store_rows": "channels / 16",
                   "protocol": "cold: memory-side cache displaced by an untimed 1 GiB read pass before each call"},
        "stored_bytes": stored, "compression_ratio": round(nbytes / stored, 3), "raw_store_rows_in_use": kept_rows,
        "round_trip_algorithmic_bytes": alg_c + alg_d,
        "algorithmic_bytes_per_step": alg_c + alg_d, "steps_executed": step.calls,
        "hbm_frac_round_trip": round((alg_c + alg_d) / step_ms / 1e6 / HBM_PEAK_GBS, 4),
        "roofline": {"bound": "hbm", "kernel": dom[0] + " (all launches of the call, event-timed)",
                     "achieved": round(dom[1] / dom[2] / 1e6, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(dom[1] / dom[2] / 1e6 / HBM_PEAK_GBS, 4), "traffic": None},
        "kernels": {"fh_mix_compress_batch": {"ms": round(c_ms, 4), "bytes": alg_c, "GBps": round(alg_c / c_ms / 1e6, 1)},
                    "fh_mix_decompress_batch": {"ms": round(d_ms, 4), "bytes": alg_d, "GBps": round(alg_d / d_ms / 1e6, 1)}},
        "warm": {"compress_ms": round(cw_ms, 4), "decompress_ms": round(dw_ms, 4)},
    }
    if not args.no_cpu_baseline:
        import oracle_chain as OC

        def one(job):
            x, outer, C, inner, cap, maps, h, w, min_out, tid = job
            st = OC.mix_compress(x, outer, C, inner, cap, G, B, rounding, 1, tid, 3.0, min_out, maps, h, w, window, tau,
                                 eps, entropy, dtype=dtype)
            OC.mix_decompress(st, outer, C, inner, cap, G, B, maps, h, w, window, eps, entropy, dtype=dtype, out_dtype=dtype)

        sample, t_one = [], 0.0
        for job in sorted(host, key=lambda j: j[0].nbytes):  # smallest first, until about 15 s are spent
            t1 = time.perf_counter()
            one(job)
            t_one += time.perf_counter() - t1
            sample.append(job)
            if t_one > 15.0:
                break
        done = sum(j[0].nbytes for j in sample)
        cores = host_threads()
        t_all = run_on_threads(one, sorted(sample, key=lambda j: -j[0].nbytes), cores)
        result["cpu_baseline"] = {"value": round(done / t_all / 1e9, 4), "unit": "GB/s", "cores": cores, "kind": "oracle",
                                  "sample": f"{len(sample)} whole tensors ({done / 2**20:.1f} MiB), the oracle's stages "
                                            f"composed, tensors handed to {cores} threads, {t_all:.1f} s",
                                  "single_thread": {"value": round(done / t_one / 1e9, 4), "unit": "GB/s", "cores": 1,
                                                    "seconds": round(t_one, 2)},
                                  "host_cpu_count": os.cpu_count()}
    return result


def bench_hooks(args, api, W, dev) -> dict:
    """A training step with the compressor hooked into autograd (saved_tensors_hooks): the
    feed-forward half of a 12-layer transformer encoder at configuration 4's shapes (batch 16,
    sequence 512, hidden 768 / 3072, bf16; LayerNorm outputs and GELU inputs are what autograd
    saves), G64 / 2-bit / stochastic.  Reported: step time and peak memory with and without
    the hooks, and per-tensor SM / PC / RC / FLT with the resulting MPS (Section 4.3).  The
    layers themselves are torch's; only the pack / unpack calls are this library's."""
    import torch
    from paper_2510_11400_amd import hooks

    torch.manual_seed(0)
    layers, hidden, inner, tokens = 12, 768, 3072, 16 * 512
    G, B, rounding = 64, 2, "stochastic"

    class Block(torch.nn.Module):
        def __init__(self):
            super().__init__()
            self.norm = torch.nn.LayerNorm(hidden)
            self.up = torch.nn.Linear(hidden, inner)
            self.down = torch.nn.Linear(inner, hidden)

        def forward(self, x):
            return x + self.down(torch.nn.functional.gelu(self.up(self.norm(x))))

    model = torch.nn.Sequential(*[Block() for _ in range(layers)]).to(dev, torch.bfloat16)
    x = torch.randn(tokens, hidden, device=dev, dtype=torch.bfloat16)
    params = list(model.parameters())

    def step(ctx):
        for p in params:
            p.grad = None
        with ctx:
            y = model(x)
            loss = y.float().square().mean()
        loss.backward()

    import contextlib

    def measure(make_ctx):
        for _ in range(args.warmup):
            step(make_ctx())
        torch.cuda.synchronize()
        torch.cuda.reset_peak_memory_stats()
        base = torch.cuda.memory_allocated()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step(make_ctx())
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / args.steps, torch.cuda.max_memory_allocated() - base

    plain_s, plain_peak = measure(contextlib.nullcontext)
    extra = {"channel_dim": -1} if args.channel_wise else {}
    if args.batch_mib > 0:
        extra["batch_bytes"] = args.batch_mib << 20
    make = lambda record=False: hooks.SavedActivations(G, B, rounding, seed=1, record=record, exclude=params, **extra)
    hooked_s, hooked_peak = measure(make)
    step(make(record=True))                                   # events are created lazily: once untimed
    ctx = make(record=True)                                   # one more step, with events around every call
    step(ctx)
    torch.cuda.synchronize()
    recs = [r for r in ctx.records if r.purge_cost is not None and r.regain_cost is not None]
    sm = sum(r.saved_bytes for r in recs)
    pc = sum(r.purge_cost for r in recs)
    rc = sum(r.regain_cost for r in recs)
    flt = [r._pack[1].elapsed_time(r._unpack[0]) * 1e-3 for r in recs]      # freed lifetime: stored -> needed again
    mps_each = [hooks.mps(r.saved_bytes, f, r.purge_cost, r.regain_cost) for r, f in zip(recs, flt)]
    in_bytes = sum(r.input_bytes for r in recs)
    result = {
        "metric": "training step with activations stored compressed (saved_tensors_hooks), on 1 MI355X",
        "value": round(in_bytes / (pc + rc) / 1e9, 2), "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(hooked_s * 1e3, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "hooks_transformer_ffn_l12_b16_s512_bf16_g64_b2_stochastic" + ("_channel_wise" if args.channel_wise else "")
                   + (f"_batches_{args.batch_mib}MiB" if args.batch_mib > 0 else ""),
                   "layers": layers,
                   "tensors_compressed": len(recs), "input_bytes": in_bytes,
                   "entry_point": ("fh_classify_channels + fh_channel_slots + fh_compress_mixed / fh_decompress_mixed"
                                   if args.channel_wise else "fh_compress / fh_decompress") + " from autograd's pack / unpack hooks"},
        "algorithmic_bytes_per_step": int(in_bytes * 2 + 2 * (in_bytes - sm)),
        "steps_executed": args.warmup + args.steps + 2,      # steps that ran the library's kernels
        "step_ms_without_hooks": round(plain_s * 1e3, 4),
        "peak_activation_bytes_without_hooks": int(plain_peak), "peak_activation_bytes_with_hooks": int(hooked_peak),
        "saved_bytes": int(sm), "purge_cost_ms": round(pc * 1e3, 4), "regain_cost_ms": round(rc * 1e3, 4),
        "freed_lifetime_ms_mean": round(1e3 * sum(flt) / max(len(flt), 1), 4),
        "mps_compress_byte_seconds_per_second": {"min": min(mps_each), "median": sorted(mps_each)[len(mps_each) // 2],
                                                 "max": max(mps_each)} if mps_each else None,
        "roofline": {"bound": "hbm", "kernel": "per-tensor compress + decompress calls (event-timed, launch-inclusive)",
                     "achieved": round((in_bytes * 2 + 2 * (in_bytes - sm)) / (pc + rc) / 1e9, 1), "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": round((in_bytes * 2 + 2 * (in_bytes - sm)) / (pc + rc) / 1e9 / HBM_PEAK_GBS, 4),
                     "traffic": None},
    }
    return result


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=5, help="workload configuration 1..5 (default 5)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="N",
                    help="also run N plain 1 GiB device copies before the timed region, so that a "
                         "rocprofv3 --pmc run can scale FETCH_SIZE / WRITE_SIZE against a known size")
    ap.add_argument("--op", choices=("roundtrip", "classify", "mixed", "sparse", "hooks", "huffman", "chain"), default="roundtrip",
                    help="roundtrip (default): compress + decompress of the tensor set; classify: the "
                         "channel classification step (moments + outlier counts), measured on its own; "
                         "mixed: the round trip with salient channels kept raw beside the quantised stream; "
                         "sparse: block-wise sparse storage of the kept channels' maps; hooks: a training "
                         "step with the compressor in autograd's saved-tensor hooks; huffman: the entropy "
                         "stage over the predictive form's index streams; chain: the whole channel-wise mix compressor "
                         "(fh_mix_compress / fh_mix_decompress) on a set with outlier channels")
    ap.add_argument("--eps", type=float, default=0.0,
                    help="--op sparse: error bound of the predictive form of dense blocks (0 = verbatim)")
    ap.add_argument("--maps-scale", type=int, default=1, metavar="K",
                    help="--op sparse: K times as many maps per set (the kernels at a bandwidth-bound size)")
    ap.add_argument("--same-dtype-out", action="store_true",
                    help="restore bf16 tensors to bf16 instead of fp32 (configuration 4's second figure)")
    ap.add_argument("--channel-wise", action="store_true",
                    help="--op hooks: classify every saved tensor's hidden channels and keep the salient ones raw")
    ap.add_argument("--batch-mib", type=int, default=0, metavar="N",
                    help="--op hooks: compress saved tensors in batches of N MiB through the batched entry points")
    ap.add_argument("--warm", action="store_true",
                    help="--op roundtrip: time compress and decompress back to back (codes still in the "
                         "memory-side cache) instead of the cold protocol")
    ap.add_argument("--displace", choices=("read", "write"), default="read",
                    help="--op roundtrip, cold protocol: what the untimed pass that displaces the memory-side "
                         "cache does with its 1 GiB buffer")
    ap.add_argument("--headline-only", action="store_true",
                    help="--op roundtrip: only the headline protocol's steps (no warm_codes, no other displacing "
                         "pass), so that a kernel trace of the run averages over one protocol")
    ap.add_argument("--no-next-rows", action="store_true",
                    help="default run only: leave out the short runs of the other ops (next_rows)")
    ap.add_argument("--per-tensor", action="store_true",
                    help="time single-tensor fh_roundtrip calls instead of the batched entry point")
    args = ap.parse_args()

    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this path runs on ONE GPU (tensors are independent: no collective, no "
              "sharding code exists); run with --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    lib = os.path.join(ROOT, "paper_2510_11400_amd", "libfedhybrid.so")
    if not os.path.exists(lib):
        from paper_2510_11400_amd.build import build_library
        build_library()
    from paper_2510_11400_amd import api, workloads as W

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")

    copy_calibration(args.copy_calibration, dev)
    ops = {"classify": bench_classify, "mixed": bench_mixed, "sparse": bench_sparse, "hooks": bench_hooks,
           "huffman": bench_huffman, "chain": bench_chain, "roundtrip": bench_roundtrip}
    result = ops[args.op](args, api, W, dev)
    if args.op == "roundtrip" and args.config == 5 and not (args.no_next_rows or args.per_tensor):
        result["next_rows"] = next_rows(args, api, W, dev, ops)
    attach_traffic(result)
    print(json.dumps(result), flush=True)
    return 0


def attach_traffic(result) -> None:
    """roofline.traffic of an op other than the plain round trip: measured HBM bytes per step from the
    committed counter summary of this workload (None when there is none, or the kernels changed since)."""
    from paper_2510_11400_amd.profile_summary import read_step_traffic
    roof = result.get("roofline")
    if roof is not None and roof.get("traffic") is None:
        name = result["config"]["workload"]
        roof["traffic"] = read_step_traffic(os.path.join(ROOT, "profiles", f"counters_{name}.txt"))


def next_rows(args, api, W, dev, ops) -> dict:
    """Short runs of the rows built around the hot path (classification, routed quantiser, sparse /
    predictive storage, Huffman stage, the whole chain), so that one default run records them all:
    GB/s of input, ms per step and the fraction of the HBM peak on each op's algorithmic bytes."""
    import copy
    import torch
    rows = {}
    for name, extra in (("classify", {}), ("mixed", {}), ("mixed_transformer", {"config": 4}), ("sparse", {"maps_scale": 16}),
                        ("sparse_eps", {"maps_scale": 16, "eps": 0.02}), ("huffman", {"maps_scale": 16}),
                        ("chain", {}), ("chain_transformer", {"config": 4})):
        a = copy.copy(args)
        a.steps, a.warmup, a.no_cpu_baseline, a.per_tensor, a.eps, a.maps_scale, a.config = 5, 2, True, False, 0.0, 1, 5
        a.headline_only = True                                # the cold figure only
        for k, v in extra.items():
            setattr(a, k, v)
        r = ops[name.split("_")[0]](a, api, W, dev)
        attach_traffic(r)
        seconds = r["ms_per_step"] * 1e-3
        rows[name] = {"workload": r["config"]["workload"], "value": r["value"], "unit": r["unit"],
                      "ms_per_step": r["ms_per_step"],
                      "hbm_frac": round(r["algorithmic_bytes_per_step"] / seconds / 1e9 / HBM_PEAK_GBS, 4),
                      "traffic": r["roofline"]["traffic"]}
        for key in ("compression_ratio", "stored_bytes"):
            if key in r:
                rows[name][key] = r[key]
        torch.cuda.empty_cache()
    return rows


def bench_roundtrip(args, api, W, dev) -> dict:
    """The hot path: every tensor of the configuration compressed, then every tensor restored,
    through the batched entry points (cold protocol unless --warm / --per-tensor)."""
    import numpy as np
    import torch

    w = W.full_config(args.config)
    t0 = time.time()
    host = []                                   # kept for the CPU baseline sample
    entries = []
    for spec, x in W.iter_materialised(w):
        host.append(x)
        xd = torch.from_numpy(x.view(np.int16) if spec.dtype == "bf16" else x).to(dev)
        if spec.dtype == "bf16":
            xd = xd.view(torch.bfloat16)
        pk, mt = api.alloc_compressed(x.size, spec.group_size, spec.bits, dev)
        out_dtype = torch.bfloat16 if (args.same_dtype_out and spec.dtype == "bf16") else torch.float32
        out = torch.empty(x.size, dtype=out_dtype, device=dev)
        entries.append(api.BatchEntry(spec.group_size, spec.bits, spec.rounding, spec.seed, spec.tensor_id,
                                      x=xd, packed=pk, meta=mt, out=out))
    batch = api.Batch(entries)
    torch.cuda.synchronize()
    print(f"[bench] {w.name}: {len(w.tensors)} tensors, {w.nbytes / 2**20:.1f} MiB resident "
          f"(generated + uploaded in {time.time() - t0:.1f} s)", file=sys.stderr, flush=True)

    cbytes = sum(algorithmic_bytes(s)[0] for s in w.tensors)
    dbytes = sum(algorithmic_bytes(s, 2 if (args.same_dtype_out and s.dtype == "bf16") else 4)[1] for s in w.tensors)
    stream = torch.cuda.current_stream()
    cold = not (args.warm or args.per_tensor)
    # The forward pass saves a tensor long before the backward pass restores it, so nothing a
    # compress call wrote is still in the memory-side cache (256 MB) when its decompress call
    # runs.  The cold protocol reproduces that: an untimed pass over a 1 GiB buffer on the same
    # stream displaces the cache before each of the two calls; the calls are timed by their own
    # events.  The pass READS the buffer (--displace read): a pass that writes leaves 256 MB of
    # modified lines behind, whose write-back to HBM then happens inside the timed call although
    # it is the displacing pass's traffic (--displace write measures exactly that).
    scrub = torch.zeros(1 << 28, dtype=torch.int32, device=dev) if cold else None

    def displace_cache(how):
        if how == "write":
            scrub.fill_(1)
        else:
            torch.amax(scrub)

    @counted
    def step(events=None, displace=None):
        if args.per_tensor:
            for e in entries:
                api.fh_roundtrip(e.x, e.group_size, e.bits, e.rounding, e.seed, e.tensor_id,
                                 packed=e.packed, meta=e.meta, out=e.out, stream=stream)
            return
        if displace:
            displace_cache(displace)
        if events is not None:
            events[0].record(stream)
        api.fh_compress_batch(batch, stream)
        if events is not None:
            events[1].record(stream)
        if displace:
            displace_cache(displace)
        if events is not None:
            events[2].record(stream)
        api.fh_decompress_batch(batch, stream)
        if events is not None:
            events[3].record(stream)

    for _ in range(args.warmup):
        step(displace=args.displace if cold else None)
    torch.cuda.synchronize()

    def timed_loop(displace):
        evs = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
        torch.cuda.synchronize()
        t_start = time.perf_counter()
        for k in range(args.steps):
            step(evs[k], displace)
        torch.cuda.synchronize()
        wall = (time.perf_counter() - t_start) / args.steps
        if args.per_tensor:
            return wall, None, None
        c_ms = sum(e[0].elapsed_time(e[1]) for e in evs) / args.steps
        d_ms = sum(e[2].elapsed_time(e[3]) for e in evs) / args.steps
        return wall, c_ms, d_ms

    wall, c_ms, d_ms = timed_loop(args.displace if cold else None)
    # cold: a step's time is that of its two calls (the displacing writes lie outside both
    # event intervals); otherwise the wall clock over the back-to-back steps
    step_s = (c_ms + d_ms) * 1e-3 if cold else wall
    result = {
        "metric": "activation compress+decompress GB/s and % of HBM peak on 1 MI355X",
        "value": round(w.nbytes / step_s / 1e9, 2), "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(step_s * 1e3, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16" if w.tensors[0].dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": w.name, "tensors": len(w.tensors), "input_bytes": w.nbytes,
                   "entry_point": "fh_roundtrip (per tensor)" if args.per_tensor
                   else "fh_compress_batch + fh_decompress_batch",
                   "restored_dtype": "bf16" if (args.same_dtype_out and w.tensors[0].dtype == "bf16") else "f32",
                   "group_size": w.tensors[0].group_size,
                   "bits": sorted({t.bits for t in w.tensors}),
                   "rounding": sorted({t.rounding for t in w.tensors}),
                   "protocol": (f"cold: memory-side cache displaced by an untimed 1 GiB {args.displace} pass before "
                                "compress and before decompress; step time = event-timed compress + decompress") if cold
                   else "warm: compress and decompress back to back, wall clock"},
        "round_trip_algorithmic_bytes": cbytes + dbytes,
        "algorithmic_bytes_per_step": cbytes + dbytes,
        "hbm_frac_round_trip": round((cbytes + dbytes) / step_s / 1e9 / HBM_PEAK_GBS, 4),
    }
    if cold:
        result["wall_ms_per_step_with_displacing_passes"] = round(wall * 1e3, 4)

    def kernel_block(c_ms, d_ms):
        return {"compress_kernel": {"ms": round(c_ms, 4), "bytes": cbytes, "GBps": round(cbytes / c_ms / 1e6, 1)},
                "decompress_kernel": {"ms": round(d_ms, 4), "bytes": dbytes, "GBps": round(dbytes / d_ms / 1e6, 1)}}

    if not args.per_tensor:
        kern = kernel_block(c_ms, d_ms)
        dom = "compress_kernel" if c_ms >= d_ms else "decompress_kernel"
        # measured HBM bytes per launch of that kernel, from the committed counter summary of
        # this workload; None when there is none or the kernel sources changed since
        from paper_2510_11400_amd.profile_summary import read_traffic
        traffic = None if args.same_dtype_out else \
            read_traffic(os.path.join(ROOT, "profiles", f"compress_decompress_{w.name}.txt")).get(dom)
        result["roofline"] = {"bound": "hbm", "kernel": dom, "achieved": kern[dom]["GBps"], "peak": HBM_PEAK_GBS,
                              "unit": "GB/s", "frac": round(kern[dom]["GBps"] / HBM_PEAK_GBS, 4),
                              "traffic": traffic}
        result["kernels"] = kern
    if cold and not args.headline_only:
        # the same steps back to back, where the backward side finds the most recently written
        # codes in the memory-side cache
        wall_w, cw_ms, dw_ms = timed_loop(None)
        result["warm_codes"] = {"ms_per_step": round(wall_w * 1e3, 4), "value": round(w.nbytes / wall_w / 1e9, 2),
                                "hbm_frac_round_trip": round((cbytes + dbytes) / wall_w / 1e9 / HBM_PEAK_GBS, 4),
                                "kernels": kernel_block(cw_ms, dw_ms)}
        # and with the other kind of displacing pass (see the comment above)
        other = "write" if args.displace == "read" else "read"
        _, co_ms, do_ms = timed_loop(other)
        result["cold_after_" + other + "_pass"] = {
            "ms_per_step": round(co_ms + do_ms, 4),
            "hbm_frac_round_trip": round((cbytes + dbytes) / (co_ms + do_ms) / 1e6 / HBM_PEAK_GBS, 4),
            "kernels": kernel_block(co_ms, do_ms)}
    del scrub

    if not args.no_cpu_baseline:
        import oracle
        # bounded sample: the leading `frac` of every tensor (whole groups), so the mix of
        # bit widths, rounding modes and distributions is that of the workload
        target_elems = 600_000_000
        frac = min(1.0, target_elems / max(1, w.numel))
        jobs = []
        for spec, x in zip(w.tensors, host):
            n = min(x.size, max(spec.group_size, int(x.size * frac) // spec.group_size * spec.group_size))
            jobs.append((spec, np.ascontiguousarray(x[:n]), n))
        sample_bytes = sum(n * spec.itemsize for spec, _, n in jobs)

        def one(job):
            spec, xs, n = job
            p, m = oracle.compress(xs, spec.group_size, spec.bits, spec.rounding, spec.seed, spec.tensor_id,
                                   dtype=spec.dtype)
            oracle.decompress(p, m, n, spec.group_size, spec.bits)

        t1 = time.perf_counter()
        for job in jobs:
            one(job)
        t_one = time.perf_counter() - t1
        cores = host_threads()
        t_all = run_on_threads(one, sorted(jobs, key=lambda j: -j[2]), cores)
        sample = (f"leading {frac:.4f} of each of the {len(w.tensors)} tensors "
                  f"({sample_bytes / 2**20:.1f} MiB input, compress + decompress)")
        result["cpu_baseline"] = {
            "value": round(sample_bytes / t_all / 1e9, 4), "unit": "GB/s", "cores": cores, "kind": "oracle",
            "sample": sample + f"; whole tensors handed to {cores} threads, largest first, {t_all:.1f} s",
            "single_thread": {"value": round(sample_bytes / t_one / 1e9, 4), "unit": "GB/s", "cores": 1,
                              "seconds": round(t_one, 2)},
            "host_cpu_count": os.cpu_count()}

    return result


if __name__ == "__main__":
    sys.exit(main())
