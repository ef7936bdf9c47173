"""Turn rocprofv3 CSV output of `bench.py` runs into the short text summary kept
under profiles/ (per-kernel durations, HBM traffic per launch from the FETCH_SIZE and
WRITE_SIZE counters, the copy-kernel calibration of those counters), and read such a
summary back for bench.py's `roofline.traffic`.

Usage (after the three rocprofv3 runs described in the summary's header):
    python -m paper_2510_11400_amd.profile_summary --trace DIR --fetch DIR --write DIR \
        --bench-json FILE --out profiles/NAME.txt
"""
from __future__ import annotations

import argparse
import csv
import glob
import hashlib
import json
import os
from collections import defaultdict
from typing import Dict, Optional

HERE = os.path.dirname(os.path.abspath(__file__))
KERNEL_SOURCES = ("fh_device.hpp", "fh_kernels.hpp", "fh_batch.hpp", "fh_channels.hpp", "fh_compress.hip", "fh_decompress.hip")   # device code
KERNELS = {"compress_kernel": "::compress_kernel<", "decompress_kernel": "::decompress_kernel<"}
COPY_MARKERS = ("copyBuffer", "copy_kernel", "CopyKernel")


def kernel_source_digest() -> str:
    """sha256 over the kernel sources: counters are only valid for the code they were taken on."""
    h = hashlib.sha256()
    for name in KERNEL_SOURCES:
        with open(os.path.join(HERE, "csrc", name), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()


def _one(pattern: str) -> str:
    hits = sorted(glob.glob(pattern, recursive=True))
    if not hits:
        raise FileNotFoundError(pattern)
    return hits[0]


def _classify(name: str) -> Optional[str]:
    for key, marker in KERNELS.items():
        if marker in name:
            return key
    if any(m in name for m in COPY_MARKERS):
        return "copy"
    return None


def _durations(trace_dir: str) -> Dict[str, dict]:
    out = defaultdict(lambda: {"calls": 0, "total_ns": 0})
    with open(_one(os.path.join(trace_dir, "**", "*kernel_trace.csv"))) as fh:
        for row in csv.DictReader(fh):
            k = _classify(row["Kernel_Name"])
            if k:
                out[k]["calls"] += 1
                out[k]["total_ns"] += int(row["End_Timestamp"]) - int(row["Start_Timestamp"])
    return out


def _counter(pmc_dir: str, counter: str) -> Dict[str, float]:
    """Mean counter value (KiB) per dispatch for each classified kernel."""
    acc = defaultdict(list)
    with open(_one(os.path.join(pmc_dir, "**", "*counter_collection.csv"))) as fh:
        for row in csv.DictReader(fh):
            if row["Counter_Name"] != counter:
                continue
            k = _classify(row["Kernel_Name"])
            if k:
                acc[k].append(float(row["Counter_Value"]))
    if "copy" in acc:                                         # the calibration copies are the large ones
        acc["copy"] = [v for v in acc["copy"] if v >= 0.5 * max(acc["copy"])]
    return {k: sum(v) / len(v) for k, v in acc.items()}


SQ_COUNTERS = ("SQ_WAVES", "SQ_BUSY_CYCLES", "SQ_WAIT_INST_ANY", "SQ_INSTS_VALU", "SQ_INSTS_SALU", "SQ_INSTS_LDS",
               "SQ_ACTIVE_INST_LDS", "SQ_LDS_BANK_CONFLICT")


def _sq_section(sq_dir: str) -> list:
    """Per-launch means of the shader-sequencer counters of a --pmc run, per kernel."""
    vals = {c: _counter(sq_dir, c) for c in SQ_COUNTERS}
    lines = []
    for k in KERNELS:
        if k not in vals["SQ_WAVES"]:
            continue
        lines.append(f"[{k}.sq]")
        for c in SQ_COUNTERS:
            lines.append(f"{c} = {vals[c].get(k, float('nan')):.0f}")
        lds_active = vals["SQ_ACTIVE_INST_LDS"].get(k, 0.0)
        if lds_active > 0:
            lines.append(f"lds_bank_conflict_over_lds_active_cycles = "
                         f"{vals['SQ_LDS_BANK_CONFLICT'].get(k, 0.0) / lds_active:.4f}")
        waves = vals["SQ_WAVES"][k]
        lines.append(f"valu_instructions_per_wave = {vals['SQ_INSTS_VALU'].get(k, 0.0) / waves:.1f}")
        lines.append(f"salu_instructions_per_wave = {vals['SQ_INSTS_SALU'].get(k, 0.0) / waves:.1f}")
        lines.append(f"lds_instructions_per_wave = {vals['SQ_INSTS_LDS'].get(k, 0.0) / waves:.1f}")
        lines.append("")
    return lines


def summarise(trace_dir, fetch_dir, write_dir, bench_json, copy_bytes, commands, sq_dir=None) -> str:
    dur = _durations(trace_dir)
    fetch = _counter(fetch_dir, "FETCH_SIZE")
    write = _counter(write_dir, "WRITE_SIZE")
    bench = json.loads(open(bench_json).read().strip().splitlines()[-1])
    # a copy of `copy_bytes` reads and writes that many bytes: the factor turns KiB counts into bytes
    f_factor = copy_bytes / (fetch["copy"] * 1024.0)
    w_factor = copy_bytes / (write["copy"] * 1024.0)
    lines = ["# rocprofv3 summary: " + bench["config"]["workload"],
             "# commands (each from the repository root, after `cd /tmp && export TMPDIR=/tmp`):"]
    lines += ["#   " + c for c in commands]
    lines += ["kernel_source_sha256 = " + kernel_source_digest(),
              f"workload = {bench['config']['workload']}",
              f"calibration_copy_bytes = {copy_bytes}",
              f"fetch_size_factor = {f_factor:.4f}    # true bytes / (FETCH_SIZE KiB * 1024), from the plain copy",
              f"write_size_factor = {w_factor:.4f}    # true bytes / (WRITE_SIZE KiB * 1024), from the plain copy",
              ""]
    for k in KERNELS:
        d = dur[k]
        avg_us = d["total_ns"] / max(1, d["calls"]) / 1e3
        fb = fetch[k] * 1024.0 * f_factor
        wb = write[k] * 1024.0 * w_factor
        alg = bench["kernels"][k]["bytes"]
        lines += [f"[{k}]",
                  f"calls = {d['calls']}",
                  f"avg_duration_us = {avg_us:.1f}    # rocprofv3 --kernel-trace",
                  f"bench_event_duration_us = {bench['kernels'][k]['ms'] * 1e3:.1f}    # HIP events inside bench.py, same run",
                  f"fetch_size_kib_per_launch = {fetch[k]:.0f}",
                  f"write_size_kib_per_launch = {write[k]:.0f}",
                  f"traffic_bytes_per_launch = {fb + wb:.0f}",
                  f"algorithmic_bytes_per_launch = {alg}",
                  f"traffic_over_algorithmic = {(fb + wb) / alg:.4f}",
                  f"achieved_GBps_algorithmic = {alg / avg_us / 1e3:.1f}",
                  ""]
    if sq_dir:
        lines += _sq_section(sq_dir)
    lines += ["[bench_line]", json.dumps(bench)]
    return "\n".join(lines) + "\n"


def read_traffic(path: str) -> Dict[str, float]:
    """{kernel: HBM bytes per launch} from a summary, or {} when it was taken on other kernel code."""
    if not os.path.exists(path):
        return {}
    out, section, digest = {}, None, None
    with open(path) as fh:
        for raw in fh:
            line = raw.split("#")[0].strip()
            if line.startswith("[") and line.endswith("]"):
                section = line[1:-1]
            elif line.startswith("kernel_source_sha256"):
                digest = line.split("=")[1].strip()
            elif line.startswith("traffic_bytes_per_launch") and section in KERNELS:
                out[section] = float(line.split("=")[1])
    return out if digest == kernel_source_digest() else {}


def summarise_trace_only(trace_dir, bench_json, commands) -> str:
    """Per-kernel call counts and durations of every library kernel in a kernel trace."""
    per = defaultdict(lambda: [0, 0, 10 ** 18, 0])
    with open(_one(os.path.join(trace_dir, "**", "*kernel_trace.csv"))) as fh:
        for row in csv.DictReader(fh):
            name = row["Kernel_Name"]
            if "fh::" not in name:
                continue
            short = name.split("fh::(anonymous namespace)::", 1)[1].split("(")[0]
            d = int(row["End_Timestamp"]) - int(row["Start_Timestamp"])
            e = per[short]
            e[0] += 1; e[1] += d; e[2] = min(e[2], d); e[3] = max(e[3], d)
    bench = json.loads(open(bench_json).read().strip().splitlines()[-1])
    lines = ["# rocprofv3 summary: " + bench["config"]["workload"],
             "# commands (each from the repository root, after `cd /tmp && export TMPDIR=/tmp`):"]
    lines += ["#   " + c for c in commands]
    lines += ["", f"{'kernel':44s} {'calls':>6s} {'avg_us':>9s} {'min_us':>9s} {'max_us':>9s} {'total_us':>10s}"]
    for k, (calls, total, lo, hi) in sorted(per.items(), key=lambda kv: -kv[1][1]):
        lines.append(f"{k:44s} {calls:6d} {total / calls / 1e3:9.1f} {lo / 1e3:9.1f} {hi / 1e3:9.1f} {total / 1e3:10.1f}")
    lines += ["", "[bench_line]", json.dumps(bench)]
    return "\n".join(lines) + "\n"


def library_source_digest() -> str:
    """sha256 over every device source of the library."""
    h = hashlib.sha256()
    for path in sorted(glob.glob(os.path.join(HERE, "csrc", "*"))):
        with open(path, "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()


def _short(name: str) -> Optional[str]:
    if "fh::" not in name:
        return None
    return name.split("fh::(anonymous namespace)::", 1)[-1].split("(")[0]


def _per_kernel_counter(pmc_dir: str, counter: str):
    """{short kernel name: [values per dispatch]} and the values of the plain copies."""
    per, copies = defaultdict(list), []
    with open(_one(os.path.join(pmc_dir, "**", "*counter_collection.csv"))) as fh:
        for row in csv.DictReader(fh):
            if row["Counter_Name"] != counter:
                continue
            name = row["Kernel_Name"]
            if any(m in name for m in COPY_MARKERS):
                copies.append(float(row["Counter_Value"]))
            k = _short(name)
            if k:
                per[k].append(float(row["Counter_Value"]))
    return per, copies


def summarise_op(trace_dir, fetch_dir, write_dir, bench_jsons, copy_bytes, commands, sq_dir=None) -> str:
    """Counters of one bench op: per library kernel the duration, the calibrated HBM bytes read and
    written per launch, and for the whole step the measured traffic over the op's algorithmic
    bytes.  `bench_jsons`: the JSON lines of the trace, fetch and write runs (each says how many
    steps its run executed, which is what that run's counter totals are divided by)."""
    b_trace, b_fetch, b_write = (json.loads(open(f).read().strip().splitlines()[-1]) for f in bench_jsons)
    fetch, f_copy = _per_kernel_counter(fetch_dir, "FETCH_SIZE")
    write, w_copy = _per_kernel_counter(write_dir, "WRITE_SIZE")
    # the calibration copies are the large ones (small device-to-host copies of results use the same kernel)
    f_copy = [v for v in f_copy if v >= 0.5 * max(f_copy)]
    w_copy = [v for v in w_copy if v >= 0.5 * max(w_copy)]
    f_factor = copy_bytes / (sum(f_copy) / len(f_copy) * 1024.0)
    w_factor = copy_bytes / (sum(w_copy) / len(w_copy) * 1024.0)
    per = defaultdict(lambda: [0, 0])
    with open(_one(os.path.join(trace_dir, "**", "*kernel_trace.csv"))) as fh:
        for row in csv.DictReader(fh):
            k = _short(row["Kernel_Name"])
            if k:
                per[k][0] += 1
                per[k][1] += int(row["End_Timestamp"]) - int(row["Start_Timestamp"])
    read_step = sum(sum(v) for v in fetch.values()) * 1024.0 * f_factor / b_fetch["steps_executed"]
    written_step = sum(sum(v) for v in write.values()) * 1024.0 * w_factor / b_write["steps_executed"]
    alg = b_trace["algorithmic_bytes_per_step"]
    lines = ["# rocprofv3 counter summary: " + b_trace["config"]["workload"],
             "# commands (each from the repository root, after `cd /tmp && export TMPDIR=/tmp`):"]
    lines += ["#   " + c for c in commands]
    lines += ["library_source_sha256 = " + library_source_digest(),
              f"workload = {b_trace['config']['workload']}",
              f"calibration_copy_bytes = {copy_bytes}",
              f"fetch_size_factor = {f_factor:.4f}    # true bytes / (FETCH_SIZE KiB * 1024), from the plain copies of the same run",
              f"write_size_factor = {w_factor:.4f}    # true bytes / (WRITE_SIZE KiB * 1024), idem",
              "",
              "[step]    # all library kernels of one step (one pass of the op over its workload)",
              f"hbm_bytes_read_per_step = {read_step:.0f}",
              f"hbm_bytes_written_per_step = {written_step:.0f}",
              f"traffic_bytes_per_step = {read_step + written_step:.0f}",
              f"algorithmic_bytes_per_step = {alg}",
              f"traffic_over_algorithmic = {(read_step + written_step) / alg:.4f}",
              f"kernel_time_per_step_us = {sum(v[1] for v in per.values()) / 1e3 / b_trace['steps_executed']:.1f}",
              "",
              f"{'kernel':44s} {'launches/step':>13s} {'avg_us':>9s} {'read_KiB':>10s} {'written_KiB':>12s}    # per launch, calibrated"]
    for k, (calls, total) in sorted(per.items(), key=lambda kv: -kv[1][1]):
        fr = sum(fetch.get(k, [0.0])) / max(1, len(fetch.get(k, [0.0]))) * f_factor
        wr = sum(write.get(k, [0.0])) / max(1, len(write.get(k, [0.0]))) * w_factor
        lines.append(f"{k:44s} {calls / b_trace['steps_executed']:13.2f} {total / calls / 1e3:9.1f} {fr:10.0f} {wr:12.0f}")
    lines.append("")
    if sq_dir:
        vals = {c: _per_kernel_counter(sq_dir, c)[0] for c in SQ_COUNTERS}
        lines.append(f"{'kernel':44s} {'valu/wave':>10s} {'salu/wave':>10s} {'lds/wave':>9s} {'lds_conflict/lds_active':>24s} {'wait_any/busy':>14s}")
        for k in sorted(per, key=lambda kk: -per[kk][1]):
            waves = sum(vals["SQ_WAVES"].get(k, [0.0]))
            if waves <= 0:
                continue
            tot = lambda c: sum(vals[c].get(k, [0.0]))
            lds_active = tot("SQ_ACTIVE_INST_LDS")
            busy = tot("SQ_BUSY_CYCLES")
            lines.append(f"{k:44s} {tot('SQ_INSTS_VALU') / waves:10.1f} {tot('SQ_INSTS_SALU') / waves:10.1f} "
                         f"{tot('SQ_INSTS_LDS') / waves:9.1f} {(tot('SQ_LDS_BANK_CONFLICT') / lds_active if lds_active else 0.0):24.4f} "
                         f"{(tot('SQ_WAIT_INST_ANY') / busy if busy else 0.0):14.2f}")
        lines.append("")
    lines += ["[bench_line]", json.dumps(b_trace)]
    return "\n".join(lines) + "\n"


def read_step_traffic(path: str) -> Optional[float]:
    """Measured HBM bytes per step from a counter summary, or None when there is none or it was
    taken on other library code."""
    if not os.path.exists(path):
        return None
    digest = value = None
    with open(path) as fh:
        for raw in fh:
            line = raw.split("#")[0].strip()
            if line.startswith("library_source_sha256"):
                digest = line.split("=")[1].strip()
            elif line.startswith("traffic_bytes_per_step"):
                value = float(line.split("=")[1])
    return value if digest == library_source_digest() else None


def main() -> None:
    ap = argparse.ArgumentParser()
    ap.add_argument("--trace", required=True)
    ap.add_argument("--fetch")
    ap.add_argument("--write")
    ap.add_argument("--sq", help="a --pmc run of the SQ counters (waves, instructions, LDS bank conflicts)")
    ap.add_argument("--bench-json", required=True, help="the bench line of the trace run")
    ap.add_argument("--fetch-json", help="the bench lines of the two counter runs: with them the summary covers "
                                         "every library kernel of the op and the whole step's traffic")
    ap.add_argument("--write-json")
    ap.add_argument("--copy-bytes", type=int, default=1 << 30)
    ap.add_argument("--out", required=True)
    ap.add_argument("--command", action="append", default=[])
    a = ap.parse_args()
    if a.fetch and a.write and a.fetch_json and a.write_json:
        text = summarise_op(a.trace, a.fetch, a.write, (a.bench_json, a.fetch_json, a.write_json), a.copy_bytes, a.command, a.sq)
    elif a.fetch and a.write:
        text = summarise(a.trace, a.fetch, a.write, a.bench_json, a.copy_bytes, a.command, a.sq)
    else:
        text = summarise_trace_only(a.trace, a.bench_json, a.command)
    with open(a.out, "w") as fh:
        fh.write(text)
    print(text)


if __name__ == "__main__":
    main()
