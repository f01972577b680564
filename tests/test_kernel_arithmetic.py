"""Host-side proof obligations of the HIP kernels (CPU only).

The kernels replace IEEE divisions by cheaper sequences whose rounding DECISIONS must be
unchanged.  Those sequences live in paper_2605_08565_amd/csrc/mxq_arith.hpp, which the kernels
include; tests/host/kernel_arithmetic_check.cpp includes the same header on the host and compares
it with exact arithmetic over (near-)exhaustive input sets: every fp32 mantissa against every
scale mantissa for the element quotient, every bf16 value against every scale code (the exact
ties), every third fp32 mantissa over the whole range of both 8-bit scale formats for the scale
encode, every fifth positive fp32 value for the Eq. 1 code, and for the reciprocal-refined division
by the per-tensor scale 3000 scales against every bf16 value plus random fp32 values, and every
mantissa pair whose exact quotient lies near a rounding midpoint (the only inputs on which that
sequence could fail).

The check is built with the clang that ships with hipcc, i.e. the front end that also compiles the
kernels (g++ rewrites -fma(a, b, -c) as fma(-a, b, c), which flips the sign of a zero result and
is not what the device code does)."""
import os
import shutil
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
CLANG = shutil.which("amdclang++") or "/opt/rocm/llvm/bin/clang++"


def test_kernel_arithmetic_shortcuts_are_decision_exact(tmp_path):
    if "fma" not in open("/proc/cpuinfo").read():
        pytest.skip("host CPU has no FMA instruction; the emulation would take minutes in software")
    exe = str(tmp_path / "kernel_arithmetic_check")
    subprocess.run([CLANG, "-O2", "-std=c++17", "-ffp-contract=off", "-mfma", "-fopenmp", "-Wall", "-Werror",
                    os.path.join(HERE, "host", "kernel_arithmetic_check.cpp"), "-o", exe, "-lm"], check=True)
    res = subprocess.run([exe], capture_output=True, text=True, timeout=900)
    print(res.stdout)
    lines = [l for l in res.stdout.splitlines() if "cases=" in l]
    names = [l.split()[0] for l in lines]
    assert names == ["quotient_decisions", "scale_encode", "pow2_code", "tensor_scale_division",
                     "tensor_scale_division_midpoints", "bf16_quotient_decisions", "scale_decode_and_range"]
    for l in lines:
        cases = int(l.split("cases=")[1].split()[0])
        bad = int(l.split("bad=")[1])
        assert cases > 1_000_000 and bad == 0, l
    assert res.returncode == 0


def test_kernels_are_built_from_the_checked_header():
    """The sequences are defined once: the device header includes mxq_arith.hpp and neither it nor
    the kernel files define them again."""
    csrc = os.path.join(os.path.dirname(HERE), "paper_2605_08565_amd", "csrc")
    dev = open(os.path.join(csrc, "mxq_device.hpp")).read()
    assert '#include "mxq_arith.hpp"' in dev
    for f in os.listdir(csrc):
        if f == "mxq_arith.hpp":
            continue
        text = open(os.path.join(csrc, f)).read()
        for fn in ("make_recip(float", "float quot(", "float div_by_T(", "pow2_code(float", "fast_division_ok(float",
                   "sf_encode_bits(float", "float sixth_of("):
            assert fn not in text, (f, fn)
