"""Do the pins bite?  (CPU only.)

Each case plants one plausible mistake into a temporary copy of the oracle's source (a wrong
tie rule, a dropped clamp, a swapped nibble, a different summation order, ...), builds it, and
runs a compact battery of the pins on it: the hand-derived worked blocks, the Eq. 1 spot
values, the fp32 tree order, the sign rule and an exhaustive pair search in exact integers.
The unmodified oracle must pass the battery; every mutant must fail it.
"""
import ctypes
import os
import subprocess

import numpy as np
import pytest

from test_oracle_recipes import E2M1, FMT, LATTICE, REC, e4m3_values_from_library, exact_block_search, worked_blocks

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(os.path.dirname(HERE), "oracle", "mxq_oracle.c")

MUTANTS = {
    "e2m1_ties_away_from_even": ("int orc_e2m1_round_mag(float y)\n{", None,
                                 "(d == best_d && (c % 2 == 0) && (best % 2 != 0))", "(d == best_d && (c % 2 != 0))", 2),
    "scale_ties_to_odd": (None, None, "(d == best_d && (c % 2 == 0) && (best % 2 != 0))", "(d == best_d && (c % 2 != 0))", 1),
    "eq1_rounds_up": (None, None, "if (ldexp((double)M, t) <= (double)amax) { k = t; break; }",
                      "if (ldexp((double)M, t - 1) <= (double)amax) { k = t; break; }", 1),
    "sequential_sum": (None, None, "    return a + b;\n}", "    (void)a; (void)b; float acc = 0.0f; for (int i = lo; i < hi; ++i) acc += s[i]; return acc;\n}", 1),
    "sign_dropped_for_zero": (None, None, "int sign = signbit(v[i]) ? 1 : 0;", "int sign = (signbit(v[i]) && mag != 0) ? 1 : 0;", 1),
    "residual_sign": (None, None, "float e = v[i] - qS;", "float e = v[i] + qS;", 1),
    "clamp_dropped": (None, None, "if (pz && orc_scale_decode(fmt, code) < orc_scale_eps(fmt)) {", "if (0) {", 1),
    "four_uses_six": (None, None, "absmax_scale_code(fmt, amax, 4.0f, pz)", "absmax_scale_code(fmt, amax, 6.0f, pz)", 1),
    "four_over_six_prefers_four_on_ties": (None, None,
        "if (less_sel(mode, cand_p, cand_e, best_p, best_e)) {      /* M = 4 only if strictly lower */",
        "if (!less_sel(mode, best_p, best_e, cand_p, cand_e)) {", 1),
    "brute_keeps_highest_code": (None, None, "if (best_code < 0 || less_sel(mode, cand_p, cand_e, best_p, best_e)) {",
                                 "if (best_code < 0 || !less_sel(mode, best_p, best_e, cand_p, cand_e)) {", 1),
    "nibbles_swapped": (None, None, "(uint8_t)(c4[i] | (c4[i + 1] << 4))", "(uint8_t)(c4[i + 1] | (c4[i] << 4))", 1),
    "fused_square": (None, None, "sq[i] = e * e;\n        long double ee", "sq[i] = fmaf(e, e, 0.0f) * 1.0000001f;\n        long double ee", 1),
    "brute_skips_subnormal_scales": (None, None, "if (!(S > 0.0f)) continue;                              /* finite and positive only */",
                                     "if (!(S > 0.0f) || c < 8) continue;", 1),
    "division_by_T_skipped": (None, None, "if (tensor_scale != 1.0f) f = f / tensor_scale;       /* step 0 */", "", 1),
}


def build(src_text, out):
    c = out + ".c"
    with open(c, "w") as f:
        f.write(src_text)
    subprocess.run(["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fopenmp", "-fPIC", "-shared",
                    "-o", out, c, "-lm"], check=True)
    lib = ctypes.CDLL(out)
    i64, i32, f32, vp = ctypes.c_int64, ctypes.c_int, ctypes.c_float, ctypes.c_void_p
    lib.orc_quantize.restype = i32
    lib.orc_quantize.argtypes = [vp, i32, i64, i64, i32, i32, i32, f32, i32, vp, vp, vp, vp]
    lib.orc_pow2_code.restype = i32
    lib.orc_pow2_code.argtypes = [f32, f32]
    lib.orc_scale_decode.restype = f32
    lib.orc_scale_decode.argtypes = [i32, i32]
    return lib


def quantize(lib, x, block, fmt, rec, T=1.0, mode=0):
    x = np.ascontiguousarray(x, np.float32)
    rows, cols = x.shape
    codes = np.empty((rows, cols // 2), np.uint8)
    scales = np.empty((rows, cols // block), np.uint8)
    sse = np.empty((rows, cols // block), np.float32)
    ex = np.empty((rows, cols // block), np.float64)
    rc = lib.orc_quantize(x.ctypes.data, 1, rows, cols, block, fmt, rec, np.float32(T), mode,
                          codes.ctypes.data, scales.ctypes.data, sse.ctypes.data, ex.ctypes.data)
    assert rc == 0
    return codes, scales, sse, ex


def battery(lib):
    """True iff every pin of the compact battery holds for this build of the oracle."""
    ok = True
    for fmt, rec, vals, scale, codes, sse in worked_blocks():                       # hand-derived blocks
        c, s, e, _ = quantize(lib, np.array([vals]), 4, FMT[fmt], REC[rec])
        ok &= s[0, 0] == scale and list(c[0]) == codes and e[0, 0] == np.float32(sse)
    for amax, S in [(6.0, 1.0), (5.99, 0.5), (12.0, 2.0), (1.0, 0.125)]:            # Eq. 1 closed form
        ok &= lib.orc_scale_decode(0, lib.orc_pow2_code(amax, 6.0)) == S
    rng = np.random.default_rng(81)                                                # tree order, no fusion
    v = (rng.standard_normal((1, 32)) * 10 ** rng.uniform(-3, 1, (1, 32))).astype(np.float32)
    c, s, e, _ = quantize(lib, v, 32, 1, 0)
    S = np.float32(lib.orc_scale_decode(1, int(s[0, 0])))
    nib = np.stack([c[0] & 0xF, c[0] >> 4], -1).ravel()
    q = np.array([np.float32(E2M1[n & 7]) * (-1 if n & 8 else 1) for n in nib], np.float32)
    r = (v[0] - q * S).astype(np.float32)
    t = (r * r).astype(np.float32)
    while len(t) > 1:
        t = (t[0::2] + t[1::2]).astype(np.float32)
    ok &= e[0, 0] == t[0]
    z = np.array([[1.0, -0.0, -1e-30, 0.0]], np.float32)                             # sign rule
    c, _, _, _ = quantize(lib, z, 4, 1, 0)
    ok &= list(c[0]) == [0x87, 0x08]
    svals = e4m3_values_from_library()                                             # exhaustive pairs
    lat = LATTICE[::3]
    signed = sorted(set(lat + [-a for a in lat]))
    pairs = np.array([[a, b] for a in signed for b in signed], np.float32)
    c, s, _, ex = quantize(lib, pairs, 2, 1, 4, mode=1)
    for i, (a, b) in enumerate(pairs):
        code, sse_int, mags = exact_block_search([float(a), float(b)], svals, -40)
        ok &= s[i, 0] == code and [c[i, 0] & 7, (c[i, 0] >> 4) & 7] == mags
    x = np.array([[0.5, -0.25, 0.125, 0.75]], np.float32)                            # per-tensor scale
    a = quantize(lib, x, 4, 1, 0, T=0.25)
    b = quantize(lib, x / np.float32(0.25), 4, 1, 0)
    ok &= (a[0] == b[0]).all() and (a[1] == b[1]).all() and (a[2] == b[2]).all()
    # equal-SSE tie in Eq. 4: (3,3,3,3) is exact under M = 6 (S = 0.5) and under M = 4 (S = 0.75)
    ok &= quantize(lib, np.array([[3.0, 3.0, 3.0, 3.0]], np.float32), 4, 1, 2)[1][0, 0] == 0x30
    return bool(ok)


def test_unmodified_oracle_passes_the_battery(tmp_path):
    assert battery(build(open(SRC).read(), str(tmp_path / "orig.so")))


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_mutant_is_caught(tmp_path, name):
    anchor, _, old, new, nth = MUTANTS[name]
    text = open(SRC).read()
    assert text.count(old) >= nth, f"mutation point for {name} not found"
    start = 0
    if anchor is not None:
        start = text.index(anchor)
        idx = text.index(old, start)
    else:
        idx = -1
        for _ in range(nth):
            idx = text.index(old, idx + 1)
    text = text[:idx] + new + text[idx + len(old):]
    assert not battery(build(text, str(tmp_path / f"{name}.so"))), f"no pin notices mutant {name}"
