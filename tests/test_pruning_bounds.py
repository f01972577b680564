"""The two inequalities the pruned brute-force search rests on, checked on the CPU against the
oracle's own block SSE (pinned fp32 arithmetic) for every scale code of many blocks.

The search over all scale codes (Section 2, "brute-force" baseline of the Numerical Study) may skip
a code only if that code cannot be the lowest-code minimiser.  With U the SSE under the abs-max
scale code c_ref (Eq. 2, at least code 1):

  upper side  for a power of two S0, the tree sum of min(fl(v_i^2), fl(fl(S0/2 - |v_i|)^2)) over the
              elements with |v_i| < S0 / 2 is a lower bound of the SSE under every scale >= S0
              (such elements quantise to 0 or to S/2; the rest add >= 0);
  lower side  while 6 S < amax, fl(fl(amax - 6 S)^2) is a lower bound of the SSE under S.

A bound that exceeds U rules the code out.  The kernels apply both per binade of the scale
format; this file re-derives the bounds in numpy float32 and compares them with the SSE of
every code, and checks that the true winner always lies inside the resulting window.
"""
import numpy as np
import pytest

E4M3, UE5M3 = 1, 2
BIAS = {E4M3: 7, UE5M3: 15}
ABSMAX = 0


def tree_sum32(s):
    s = np.asarray(s, np.float32)
    while s.size > 1:
        s = (s[0::2] + s[1::2]).astype(np.float32)
    return np.float32(s[0])


def blocks(kind, b, n, rng):
    if kind == "student":
        return (rng.standard_t(4, size=(n, b)) * 0.02).astype(np.float32)
    if kind == "normal_small":
        return (rng.standard_normal((n, b)) * 0.002).astype(np.float32)
    if kind == "outlier":
        x = rng.standard_normal((n, b)).astype(np.float32)
        x[:, 0] *= 50.0
        return x
    if kind == "flat":                                   # all magnitudes alike: the window's worst case
        return (np.sign(rng.standard_normal((n, b))) * (1.0 + 0.05 * rng.random((n, b)))).astype(np.float32)
    raise ValueError(kind)


@pytest.mark.parametrize("fmt", [E4M3, UE5M3])
@pytest.mark.parametrize("b", [4, 16])
@pytest.mark.parametrize("kind", ["student", "normal_small", "outlier", "flat"])
def test_window_bounds_hold_for_every_code(oracle, fmt, b, kind):
    rng = np.random.default_rng(1000 * fmt + 10 * b + len(kind))
    bias = BIAS[fmt]
    max_code = oracle.scale_max_code(fmt)
    scale = np.array([oracle.scale_decode(fmt, c) for c in range(max_code + 1)], np.float64)
    pruned_hi = pruned_lo = 0
    for v in blocks(kind, b, 24, rng):
        sse = np.array([oracle.block_sse(v, fmt, c)[1] for c in range(max_code + 1)], np.float32)
        _, scales, _ = oracle.quantize(v.reshape(1, b), b, fmt, ABSMAX)
        cref = max(int(scales[0, 0]), 1)
        U = sse[cref]
        winner = 1 + int(np.argmin(sse[1:]))             # lowest code among the minimal ones (code 0 is no candidate)
        amax = np.float32(np.abs(v).max())
        eref = cref >> 3
        vsq = (v * v).astype(np.float32)

        hi = max_code
        for d in range(2, 6):
            ef = eref + d
            s0 = np.float32(2.0 ** (ef - bias))
            gap = (np.float32(0.5) * s0 - np.abs(v)).astype(np.float32)
            terms = np.where(gap > 0, np.minimum(vsq, (gap * gap).astype(np.float32)), np.float32(0))
            bound = tree_sum32(terms)
            above = np.nonzero(scale >= float(s0))[0]
            assert np.all(sse[above] >= bound), (kind, b, fmt, d)
            if bound > U:
                hi = min(hi, (ef << 3) - 1)
                pruned_hi += 1
                break

        lo = 1
        for t in range(1, 4):
            ef = eref - t
            if ef < 0:
                break
            top = (ef << 3) + 7 if ef >= 1 else 7
            lim = np.float32(6.0) * np.float32(scale[top])
            if lim < amax:
                dd = np.float32(amax - lim)
                bound = np.float32(dd * dd)
                below = np.arange(1, top + 1)
                assert np.all(sse[below] >= bound), (kind, b, fmt, t)
                if bound > U:
                    lo = (ef + 1) << 3
                    pruned_lo += 1
                    break
        assert lo <= cref <= hi
        assert lo <= winner <= hi, (kind, b, fmt, lo, winner, hi)
    if kind == "student":
        assert pruned_hi > 0 and pruned_lo > 0           # the bounds do bite on weight-like inputs
