"""Pins for the oracle's appendix diagnostics (CPU only): clipping-only SSE and histograms."""
import os

import numpy as np
import pytest

from paper_2605_08565_amd import workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
FMT = {"e8m0": 0, "e4m3": 1, "ue5m3": 2}


def clip_cases():
    rows = []
    with open(os.path.join(GOLDEN, "worked_blocks_clip.txt")) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                fmt, vals, scale, want = [t.strip() for t in line.split("|")]
                rows.append((fmt, [float(v) for v in vals.split()], int(scale, 16), float(want)))
    return rows


@pytest.mark.parametrize("case", clip_cases(), ids=lambda c: f"{c[0]}-{c[1][0]}-{c[2]:02x}")
def test_clip_sse_worked_blocks(oracle, case):
    fmt, vals, scale, want = case
    x = np.array([vals], np.float32)
    got = oracle.clip_sse(x, np.array([[scale]], np.uint8), 4, FMT[fmt])
    assert got[0, 0] == np.float32(want)


def test_clip_sse_is_part_of_the_sse(oracle):
    """0 <= clip <= SSE per block; equal to the error recomputed from the de-quantised tensor
    restricted to the saturating elements; zero wherever amax <= 6 S."""
    x = W.student_t_weights(48, 512, seed=71)
    xf = W.bf16_bits_to_f32(x).astype(np.float64)
    for fmt, rec in [(1, 0), (1, 2), (1, 4), (0, 0), (2, 1)]:
        for b in (4, 16, 64):
            c, s, e = oracle.quantize(x, b, fmt, rec)
            clip = oracle.clip_sse(x, s, b, fmt)
            assert (clip >= 0).all() and (clip <= e).all()
            S = np.array([oracle.scale_decode(fmt, int(v)) for v in s.ravel()]).reshape(s.shape)
            Sx = np.repeat(S, b, axis=1)
            sat = (np.abs(xf) > 6 * Sx) & (Sx > 0)      # a zero scale zeroes the block: not clipping
            xh = oracle.dequantize(c, s, b, fmt).astype(np.float64)
            want = (((xf - xh) ** 2) * sat).reshape(48, -1, b).sum(-1)
            assert np.allclose(clip, want, rtol=2e-6, atol=0)
            amax = np.abs(xf).reshape(48, -1, b).max(-1)
            assert (clip[(amax <= 6 * S) | (S == 0)] == 0).all()


def test_clipping_error_shrinks_with_4over6_and_brute_force(oracle):
    """Appendix: 4-over-6 and brute force substantially reduce the clipping error at small
    block sizes (Region B), which explains much of the block-size inversion."""
    sigma = 0.008
    x = W.normal_blocks_f32(sigma, 20000, 4, seed=5)
    tot = {}
    for rec in (1, 3, 4):
        s = oracle.quantize(x, 4, 1, rec)[1]
        tot[rec] = float(oracle.clip_sse(x, s, 4, 1).sum(dtype=np.float64))
    assert tot[3] < 0.5 * tot[1] and tot[4] < 0.5 * tot[1]


def test_histograms(oracle):
    x = W.normal_blocks_f32(0.001, 4000, 8, seed=9)
    c, s, _ = oracle.quantize(x, 8, 1, 0)
    eh, sh = oracle.histograms(c, s)
    assert eh.sum() == x.size and sh.sum() == x.size // 8
    # Region A: the abs-max scale is zero for almost every block, so every entry is zero
    assert sh[0] > 0.95 * sh.sum() and eh[0] > 0.95 * eh.sum()
    # brute-force search picks the smallest positive scale there (what prevent-zero picks)
    c, s, _ = oracle.quantize(x, 8, 1, 4)
    _, sh_b = oracle.histograms(c, s)
    assert sh_b[1] > 0.9 * sh_b.sum()
    # independent count of one bin
    nib = np.concatenate([(c & 0xF).ravel(), (c >> 4).ravel()])
    assert oracle.histograms(c, s)[0][3] == int(((nib & 7) == 3).sum())


def test_histograms_hand_counted(oracle):
    """Explicit bytes, counts written out by hand: both nibbles of a byte are counted, the sign
    bit (bit 3 of a nibble) is ignored, scale bytes are counted as they are."""
    codes = np.array([[0x10, 0x92, 0x7F]], np.uint8)      # nibbles 0,1 | 2,9 | 15,7 -> magnitudes 0,1,2,1,7,7
    scales = np.array([[3, 3, 200]], np.uint8)
    eh, sh = oracle.histograms(codes, scales)
    assert list(eh) == [1, 2, 1, 0, 0, 0, 0, 2]
    want = np.zeros(256, np.uint64)
    want[3], want[200] = 2, 1
    assert (sh == want).all()
