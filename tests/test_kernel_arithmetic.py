"""Host-side proof obligations of the HIP kernels (CPU only).

The kernels replace IEEE divisions by cheaper sequences whose rounding DECISIONS must be
unchanged.  tests/host/kernel_arithmetic_check.c re-states those sequences with fmaf on the
host and compares them with exact arithmetic over (near-)exhaustive input sets: every fp32
mantissa against every scale mantissa for the element quotient, every third fp32 mantissa over
the whole range of both 8-bit scale formats for the scale encode, every fifth positive fp32
value for the Eq. 1 code, and for the reciprocal-refined division by the per-tensor scale 3000
scales against every bf16 value plus random fp32 values, and every mantissa pair whose exact
quotient lies near a rounding midpoint (the only inputs on which that sequence could fail)."""
import os
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))


def test_kernel_arithmetic_shortcuts_are_decision_exact(tmp_path):
    if "fma" not in open("/proc/cpuinfo").read():
        pytest.skip("host CPU has no FMA instruction; the emulation would take minutes in software")
    exe = str(tmp_path / "kernel_arithmetic_check")
    subprocess.run(["gcc", "-O2", "-ffp-contract=off", "-mfma", "-fopenmp",
                    os.path.join(HERE, "host", "kernel_arithmetic_check.c"), "-o", exe, "-lm"], check=True)
    res = subprocess.run([exe], capture_output=True, text=True, timeout=600)
    print(res.stdout)
    lines = [l for l in res.stdout.splitlines() if "cases=" in l]
    assert len(lines) == 5
    for l in lines:
        cases = int(l.split("cases=")[1].split()[0])
        bad = int(l.split("bad=")[1])
        assert cases > 1_000_000 and bad == 0, l
    assert res.returncode == 0
