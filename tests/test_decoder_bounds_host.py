"""The index arithmetic of the two stream decoders, checked on the CPU.

fh_huffman_decode and fh_sparse_decode accept streams that no encoder of this library wrote and promise
that such a stream cannot make a kernel read or write outside the buffers it was given.  Here the very
kernels (paper_2510_11400_amd/csrc/fh_huffman.hip, fh_sparse.hip, unchanged) are compiled for the host
against tests/simt_host/hip/hip_runtime.h -- one OS thread per work-item, one workgroup at a time -- and
run under AddressSanitizer and UndefinedBehaviorSanitizer with every buffer allocated to the byte: valid streams must decode to what the
oracle decodes (Section 4.4.1's dense-block path read backwards), and truncated, corrupted and random
streams must run to the end without a report.  Nothing here is a product path: the package never builds
or loads this program."""
from __future__ import annotations

import os
import shutil
import struct
import subprocess

import numpy as np
import pytest

import oracle
from paper_2510_11400_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2510_11400_amd", "csrc")
SHIM = os.path.join(ROOT, "tests", "simt_host")
FH_OK = 0


def _clang():
    for c in ("/opt/rocm/lib/llvm/bin/clang++", shutil.which("clang++")):
        if c and os.path.exists(c):
            return c
    return None


@pytest.fixture(scope="module")
def decoders(tmp_path_factory):
    cxx = _clang()
    if cxx is None:
        pytest.skip("no clang++ (the kernels use clang's vector extensions)")
    out = tmp_path_factory.mktemp("simt")
    flags = ["-std=c++20", "-O1", "-g", "-pthread", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
             "-fno-omit-frame-pointer"]
    objs, jobs = [], []
    for src in ("fh_huffman.hip", "fh_sparse.hip"):
        obj = str(out / (src + ".o"))
        jobs.append(subprocess.Popen([cxx, "-x", "c++", *flags, "-I", SHIM, "-c", os.path.join(CSRC, src), "-o", obj]))
        objs.append(obj)
    for j in jobs:
        assert j.wait() == 0, "the kernels did not compile for the host"
    main_o = str(out / "main.o")
    subprocess.run([cxx, *flags, "-c", os.path.join(SHIM, "coders_main.cpp"), "-o", main_o], check=True)
    exe = str(out / "simt_decoders")
    subprocess.run([cxx, "-pthread", "-fsanitize=address,undefined", main_o, *objs, "-o", exe], check=True)

    def run(cases, timeout=600):
        cf, rf = str(out / "cases.bin"), str(out / "results.bin")
        with open(cf, "wb") as f:
            f.write(struct.pack("<I", len(cases)) + b"".join(cases))
        env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0:halt_on_error=1")
        env.pop("LD_PRELOAD", None)
        r = subprocess.run([exe, cf, rf], capture_output=True, text=True, timeout=timeout, env=env)
        assert r.returncode == 0, f"the CPU build of the decoders failed (rc {r.returncode}):\n{r.stderr[-4000:]}"
        buf, o, results = open(rf, "rb").read(), 0, []
        for _ in cases:
            st, nb = struct.unpack_from("<iQ", buf, o)
            o += 12
            results.append((st, np.frombuffer(buf, np.uint8, nb, o).copy()))
            o += nb
        return results

    return run


def _huffman_case(stream: np.ndarray, n: int, stream_bytes=None) -> bytes:
    s = np.ascontiguousarray(stream, dtype=np.uint8)
    k = s.size if stream_bytes is None else stream_bytes
    return b"H" + struct.pack("<QQQ", n, k, n) + s[:k].tobytes()


def _sparse_case(info, values, indices, dtype, n, maps, h, w, eps) -> bytes:
    return (b"S" + struct.pack("<iiqqqfQQQ", 0 if dtype == "f32" else 1, n, maps, h, w, eps, info.size, values.nbytes,
                               indices.size) + info.tobytes() + values.tobytes() + indices.tobytes())


def _clustered(rng, n, spread):
    return np.clip(np.rint(rng.normal(128.0, spread, n)), 0, 255).astype(np.uint8)


def test_huffman_valid_streams_decode_as_the_oracle_does(decoders):
    rng = np.random.default_rng(5)
    datas = [_clustered(rng, n, s) for n, s in ((1, 3.0), (255, 3.0), (256, 1.0), (257, 6.0), (70_001, 6.0), (300_001, 0.4))]
    datas.append(rng.integers(0, 256, 200_000, dtype=np.uint8))            # 8 bits per symbol: slices too long to stage
    skew = np.minimum(rng.geometric(0.5, 150_000) - 1, 255).astype(np.uint8)  # code lengths up to the limit of 24
    datas.append(skew)
    cases = []
    for d in datas:
        stream, _ = oracle.huffman_encode(d)
        cases.append(_huffman_case(stream, d.size))
    for d, (st, got) in zip(datas, decoders(cases)):
        assert st == FH_OK
        assert np.array_equal(got, d), f"n = {d.size}"


def test_huffman_encoder_on_the_cpu_writes_the_oracles_streams(decoders):
    """The encoder's kernels through the same stand-in (histogram, code construction, count, scan, write): the
    stream and its totals byte for byte, with the buffers sized to the byte."""
    rng = np.random.default_rng(9)
    datas = [_clustered(rng, n, s) for n, s in ((1, 3.0), (255, 3.0), (256, 1.0), (257, 6.0), (4096, 6.0), (70_001, 6.0),
                                                  (300_001, 0.4), (65536 * 3 + 17, 20.0))]
    datas.append(rng.integers(0, 256, 200_000, dtype=np.uint8))
    datas.append(np.minimum(rng.geometric(0.5, 150_000) - 1, 255).astype(np.uint8))
    datas.append(np.full(5000, 7, np.uint8))
    cases = [b"E" + struct.pack("<Q", d.size) + d.tobytes() for d in datas]
    for d, (st, got) in zip(datas, decoders(cases)):
        want, bits = oracle.huffman_encode(d)
        assert st == FH_OK
        assert got[-16:].view(np.uint64).tolist() == [want.size, bits], f"n = {d.size}"
        assert np.array_equal(got[:-16], want), f"n = {d.size}"


def test_huffman_foreign_streams_stay_in_bounds(decoders):
    rng = np.random.default_rng(6)
    n = 200_003                                               # 782 chunks: four workgroups of 256 chunks
    data = _clustered(rng, n, 6.0)
    stream, _ = oracle.huffman_encode(data)
    chunks = (n + 255) // 256
    head = 256 + 4 * (chunks + 1)
    cases = []
    for keep in (head, head + 1, head + 4, head + 1000, stream.size // 2, stream.size - 1, stream.size - 4):
        cases.append(_huffman_case(stream, n, stream_bytes=keep))          # truncated payload
    cases.append(_huffman_case(stream, n, stream_bytes=head - 1))          # not even the offsets: refused on the host
    for fill in (0, 1, 24, 25, 255):                                        # length tables no code has
        s = stream.copy()
        s[:256] = fill
        cases.append(_huffman_case(s, n))
    s = stream.copy()
    s[:256] = rng.integers(0, 32, 256, dtype=np.uint8)
    cases.append(_huffman_case(s, n))
    offsets_at = slice(256, head)
    for kind in ("random", "descending", "huge", "zero", "beyond"):
        s = stream.copy()
        off = s[offsets_at].view(np.uint32)
        if kind == "random":
            off[:] = rng.integers(0, 2 ** 32, off.size, dtype=np.uint64).astype(np.uint32)
        elif kind == "descending":
            off[:] = off[::-1].copy()
        elif kind == "huge":
            off[:] = 0xFFFFFFFF
        elif kind == "zero":
            off[:] = 0
        else:
            off[:] = off + np.uint32((stream.size - head) // 4 - 3)        # slices that start at the very end
        cases.append(_huffman_case(s, n))
    s = stream.copy()
    s[head:] = rng.integers(0, 256, s.size - head, dtype=np.uint8)          # a payload of noise
    cases.append(_huffman_case(s, n))
    cases.append(_huffman_case(rng.integers(0, 256, stream.size, dtype=np.uint8), n))   # noise throughout
    big = rng.integers(0, 256, 256 + 4 * (chunks + 1) + 4 * 192 * chunks, dtype=np.uint8)
    cases.append(_huffman_case(big, n))                                    # noise of the largest size a stream can have
    results = decoders(cases)
    assert results[7][0] != FH_OK
    assert all(st == FH_OK for k, (st, _) in enumerate(results) if k != 7)


def test_huffman_large_launch_uses_the_wide_workgroups(decoders):
    """More than 256 groups of 768 chunks: the launch with workgroups of 768 work-items and 46 staged words per
    chunk; one valid stream -- its second half too wide for a pass to seat 768 chunks -- and the same stream with
    its offsets and payload replaced by noise."""
    rng = np.random.default_rng(7)
    n = 256 * 768 * 256 + 77
    data = np.concatenate([_clustered(rng, n // 2, 6.0), _clustered(rng, n - n // 2, 20.0)])
    stream, _ = oracle.huffman_encode(data)
    head = 256 + 4 * ((n + 255) // 256 + 1)
    noisy = stream.copy()
    noisy[256:] = rng.integers(0, 256, noisy.size - 256, dtype=np.uint8)
    (st, got), (st2, _) = decoders([_huffman_case(stream, n), _huffman_case(noisy, n)], timeout=900)
    assert st == FH_OK and st2 == FH_OK
    assert np.array_equal(got, data)
    assert head < stream.size


SPARSE_SHAPES = [(40, 28, 28, 4, "f32", 0.0), (40, 28, 28, 4, "f32", 0.02), (9, 13, 11, 4, "bf16", 0.0),
                 (9, 13, 11, 4, "bf16", 0.05), (30, 14, 14, 2, "f32", 0.02), (12, 56, 56, 8, "f32", 0.0),
                 (12, 30, 17, 8, "bf16", 0.02), (3, 7, 300, 4, "f32", 0.0)]


def _sparse_input(maps, h, w, dtype, seed):
    x = W.salient_feature_maps(maps, h, w, seed=seed)
    if dtype == "bf16":
        x = (x.view(np.uint32) >> 16).astype(np.uint16)
    return x


def test_sparse_valid_streams_decode_as_the_oracle_does(decoders):
    cases, wants = [], []
    for k, (maps, h, w, n, dtype, eps) in enumerate(SPARSE_SHAPES):
        x = _sparse_input(maps, h, w, dtype, 11 + k)
        info, values, indices, _ = oracle.sparse_encode(x, maps, h, w, n, 0.5, dtype=dtype, eps=eps)
        cases.append(_sparse_case(info, values, indices, dtype, n, maps, h, w, eps))
        wants.append(oracle.sparse_decode(info, values, indices, maps, h, w, n, dtype=dtype, eps=eps))
    for shape, want, (st, got) in zip(SPARSE_SHAPES, wants, decoders(cases)):
        assert st == FH_OK
        assert np.array_equal(got, want.view(np.uint8).reshape(-1)), f"{shape}"


def test_sparse_encoder_on_the_cpu_writes_the_oracles_streams(decoders):
    """The encoder's kernels through the same stand-in: block bytes, totals, and the two streams byte for byte."""
    shapes = SPARSE_SHAPES + [(700, 56, 56, 4, "f32", 0.02)]
    cases, wants = [], []
    for k, (maps, h, w, n, dtype, eps) in enumerate(shapes):
        x = _sparse_input(maps, h, w, dtype, 50 + k)
        cases.append(b"Z" + struct.pack("<iiqqqff", 0 if dtype == "f32" else 1, n, maps, h, w, 0.5, eps) + x.tobytes())
        info, values, indices, totals = oracle.sparse_encode(x, maps, h, w, n, 0.5, dtype=dtype, eps=eps)
        wants.append(np.concatenate([info, totals.view(np.uint8), values.view(np.uint8).reshape(-1), indices]))
    for shape, want, (st, got) in zip(shapes, wants, decoders(cases)):
        assert st == FH_OK
        assert got.size == want.size and np.array_equal(got, want), f"{shape}"


def test_sparse_foreign_streams_stay_in_bounds(decoders):
    rng = np.random.default_rng(8)
    cases = []
    for k, (maps, h, w, n, dtype, eps) in enumerate(SPARSE_SHAPES):
        x = _sparse_input(maps, h, w, dtype, 31 + k)
        info, values, indices, _ = oracle.sparse_encode(x, maps, h, w, n, 0.5, dtype=dtype, eps=eps)
        some = lambda a, share: a[: int(a.size * share)]
        noise_i = rng.integers(0, 256, info.size, dtype=np.uint8)
        noise_x = rng.integers(0, 256, max(1, indices.size), dtype=np.uint8)
        cases += [
            _sparse_case(info, some(values, 0.5), indices, dtype, n, maps, h, w, eps),        # values cut short
            _sparse_case(info, values, some(indices, 0.5), dtype, n, maps, h, w, eps),        # indices cut short
            _sparse_case(info, values[:0], indices[:0], dtype, n, maps, h, w, eps),           # both empty
            _sparse_case(noise_i, values, indices, dtype, n, maps, h, w, eps),                # block bytes of noise
            _sparse_case(info, values, noise_x, dtype, n, maps, h, w, eps),                   # CSR structure / codes of noise
            _sparse_case(noise_i, some(values, 0.3), some(noise_x, 0.3), dtype, n, maps, h, w, eps),
            _sparse_case(np.full(info.size, 0xFF, np.uint8), values, indices, dtype, n, maps, h, w, eps),   # every block dense and full
            _sparse_case(np.full(info.size, 0x7F, np.uint8), values, indices, dtype, n, maps, h, w, eps),   # every block sparse, 127 values
            _sparse_case(info, values, indices, dtype, n, maps, h, w, 0.02 if eps == 0.0 else 0.0),           # read in the other form
        ]
    assert all(st == FH_OK for st, _ in decoders(cases))


def test_sparse_random_shapes_on_the_cpu(decoders):
    """Seeded random shapes, windows, thresholds, error bounds and dtypes (maps narrower or lower than the window,
    single maps, ragged edges): the encoder's streams and the decoder's maps against the oracle's."""
    rng = np.random.default_rng(77)
    specs = []
    for _ in range(40):
        n = int(rng.choice([2, 4, 8]))
        maps, h, w = int(rng.integers(1, 24)), int(rng.integers(1, 45)), int(rng.integers(1, 45))
        dtype = str(rng.choice(["f32", "bf16"]))
        eps = float(rng.choice([0.0, 0.0, 0.02, 0.2]))
        tau = float(rng.choice([0.0, 0.25, 0.5, 1.0]))
        specs.append((maps, h, w, n, dtype, eps, tau))
    enc_cases, dec_cases, enc_wants, dec_wants = [], [], [], []
    for k, (maps, h, w, n, dtype, eps, tau) in enumerate(specs):
        x = _sparse_input(maps, h, w, dtype, 200 + k)
        info, values, indices, totals = oracle.sparse_encode(x, maps, h, w, n, tau, dtype=dtype, eps=eps)
        enc_cases.append(b"Z" + struct.pack("<iiqqqff", 0 if dtype == "f32" else 1, n, maps, h, w, tau, eps) + x.tobytes())
        enc_wants.append(np.concatenate([info, totals.view(np.uint8), values.view(np.uint8).reshape(-1), indices]))
        dec_cases.append(_sparse_case(info, values, indices, dtype, n, maps, h, w, eps))
        dec_wants.append(oracle.sparse_decode(info, values, indices, maps, h, w, n, dtype=dtype, eps=eps))
    results = decoders(enc_cases + dec_cases)
    for spec, want, (st, got) in zip(specs, enc_wants, results[: len(specs)]):
        assert st == FH_OK and got.size == want.size and np.array_equal(got, want), f"encode {spec}"
    for spec, want, (st, got) in zip(specs, dec_wants, results[len(specs):]):
        assert st == FH_OK and np.array_equal(got, want.view(np.uint8).reshape(-1)), f"decode {spec}"


def test_huffman_random_streams_round_trip_on_the_cpu(decoders):
    """Seeded random lengths and byte distributions: the encoder's stream against the oracle's, and the decoder on
    that stream back to the bytes."""
    rng = np.random.default_rng(78)
    datas = []
    for _ in range(24):
        n = int(rng.integers(1, 120_000))
        kind = int(rng.integers(0, 4))
        if kind == 0:
            d = _clustered(rng, n, float(rng.uniform(0.3, 30.0)))
        elif kind == 1:
            d = rng.integers(0, int(rng.integers(1, 257)), n, dtype=np.uint16).astype(np.uint8)
        elif kind == 2:
            d = np.minimum(rng.geometric(float(rng.uniform(0.05, 0.9)), n) - 1, 255).astype(np.uint8)
        else:
            d = rng.choice(np.array([0, 7, 128, 255], np.uint8), n, p=[0.7, 0.2, 0.09, 0.01])
        datas.append(d)
    streams = [oracle.huffman_encode(d) for d in datas]
    cases = [b"E" + struct.pack("<Q", d.size) + d.tobytes() for d in datas]
    cases += [_huffman_case(st, d.size) for d, (st, _) in zip(datas, streams)]
    results = decoders(cases)
    for d, (want, bits), (st, got) in zip(datas, streams, results[: len(datas)]):
        assert st == FH_OK and got[-16:].view(np.uint64).tolist() == [want.size, bits], f"encode n = {d.size}"
        assert np.array_equal(got[:-16], want), f"encode n = {d.size}"
    for d, (st, got) in zip(datas, results[len(datas):]):
        assert st == FH_OK and np.array_equal(got, d), f"decode n = {d.size}"

