"""AddressSanitizer + UndefinedBehaviorSanitizer builds of the host-side code (CPU only).

  * the oracle: tests/host/oracle_sanitize_driver.c includes oracle/mxq_oracle.c and replays the
    hand-derived worked blocks of tests/golden/ plus a battery of shapes (every block size, both
    dtypes, every recipe and scale format, a per-tensor scale, ragged row counts) on exactly sized
    heap buffers; expected bytes for the battery come from the ordinary oracle build;
  * the boundary: tests/host/boundary_sanitize_driver.hip links the C ABI's own validation code
    (paper_2605_08565_amd/csrc/mxq_api.hip) against counting stubs instead of kernel launchers and
    runs the argument-validation battery: every refusal must come before a launch.
The device code cannot be sanitised on the test machines; it is covered by the GPU parity tests."""
import os
import shutil
import struct
import subprocess

import numpy as np
import pytest

from paper_2605_08565_amd import workloads as W

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
FMT = {"e8m0": 0, "e4m3": 1, "ue5m3": 2}
REC = {"absmax": 0, "absmax_pz": 1, "4over6": 2, "4over6_pz": 3, "brute": 4}


def record(x, block, fmt, rec, T, codes, scales, sse):
    dt = 0 if x.dtype == np.uint16 else 1
    head = struct.pack("<6if", dt, x.shape[0], x.shape[1], block, fmt, rec, T)
    return head + x.tobytes() + np.ascontiguousarray(codes, np.uint8).tobytes() + \
        np.ascontiguousarray(scales, np.uint8).tobytes() + np.ascontiguousarray(sse, np.float32).tobytes()


def test_oracle_under_asan_ubsan(tmp_path, oracle):
    recs = []
    # the worked blocks: expected values are the hand-derived ones, not the oracle's
    with open(os.path.join(HERE, "golden", "worked_blocks.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            head, vals, scale, codes, sse = [t.strip() for t in line.split("|")]
            fmt, rec = head.split()
            x = np.array([[float(v) for v in vals.split()]], np.float32)
            recs.append(record(x, 4, FMT[fmt], REC[rec], 1.0, [int(c, 16) for c in codes.split()],
                               [int(scale, 16)], [float(sse)]))
    n_golden = len(recs)
    assert n_golden >= 20
    rng = np.random.default_rng(5)
    for block in (2, 4, 8, 16, 32, 64, 128):
        rows, cols = int(rng.integers(1, 6)), block * int(rng.integers(1, 4))
        x32 = (rng.standard_normal((rows, cols)) * 10.0 ** rng.uniform(-4, 2)).astype(np.float32)
        x32[0, 0] = 0.0
        for x in (x32, W.f32_to_bf16_bits(x32)):
            for fmt, rec in [(0, 0), (0, 4), (1, 0), (1, 1), (1, 2), (1, 3), (1, 4), (2, 0), (2, 3), (2, 4)]:
                for T in (1.0, 0.0371):
                    c, s, e = oracle.quantize(x, block, fmt, rec, tensor_scale=T)
                    recs.append(record(x, block, fmt, rec, float(np.float32(T)), c, s, e))
    cases = tmp_path / "cases.bin"
    cases.write_bytes(struct.pack("<i", len(recs)) + b"".join(recs))
    exe = str(tmp_path / "oracle_sanitize")
    subprocess.run(["gcc", "-O1", "-g", "-std=c11", "-ffp-contract=off", "-fopenmp", "-fsanitize=address,undefined",
                    "-fno-sanitize-recover=all", "-static-libasan", os.path.join(HERE, "host", "oracle_sanitize_driver.c"),
                    "-o", exe, "-lm"], check=True)
    res = subprocess.run([exe, str(cases)], capture_output=True, text=True, timeout=600,
                         env={**os.environ, "ASAN_OPTIONS": "detect_leaks=1:abort_on_error=0", "OMP_NUM_THREADS": "4"})
    print(res.stdout[-2000:], res.stderr[-4000:])
    assert res.returncode == 0
    assert f"oracle_sanitize cases={len(recs)} bad=0" in res.stdout
    assert "ERROR: AddressSanitizer" not in res.stderr and "runtime error" not in res.stderr


def test_boundary_validation_under_asan_ubsan(tmp_path):
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    exe = str(tmp_path / "boundary_sanitize")
    cmd = [hipcc, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17",
           "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=all",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument",
           os.path.join(HERE, "host", "boundary_sanitize_driver.hip"),
           os.path.join(ROOT, "paper_2605_08565_amd", "csrc", "mxq_api.hip"), "-o", exe]
    subprocess.run(cmd, check=True)
    res = subprocess.run([exe], capture_output=True, text=True, timeout=300,
                         env={**os.environ, "ASAN_OPTIONS": "detect_leaks=0"})
    print(res.stdout[-2000:], res.stderr[-4000:])
    assert res.returncode == 0
    assert " bad=0" in res.stdout
    assert "ERROR: AddressSanitizer" not in res.stderr and "runtime error" not in res.stderr
