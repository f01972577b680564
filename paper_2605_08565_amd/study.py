"""The "Numerical Study" of the paper's Results section on the GPU library: MSE against the standard deviation.

For every sigma of 151 evenly spaced points in [0.0005, 0.05] and every block size in
{4, 8, 16, 32}, 50 000 blocks are drawn from N(0, sigma^2) (seeded) and quantised with E2M1
elements and E4M3 scales under abs-max, prevent-zero, 4-over-6, prevent-zero + 4-over-6 and the
brute-force search -- the five panels of the paper's MSE-vs-sigma figure.  All sigmas of one
block size go through the library as ONE tensor (one block per row), so the whole study is 20
launches.

    python -m paper_2605_08565_amd.study [--out study.json] [--sigmas 151] [--blocks-per-sigma 50000]

Prints / writes JSON: {"sigma": [...], "mse": {recipe: {block: [...]}}}.
"""
from __future__ import annotations

import argparse
import json
import sys

import numpy as np

RECIPES = {"absmax": 0, "prevent_zero": 1, "4over6": 2, "prevent_zero_4over6": 3, "brute_force": 4}
BLOCKS = (4, 8, 16, 32)


def study_sigmas(n: int = 151) -> np.ndarray:
    return np.linspace(0.0005, 0.05, n)


def study_tensor(sigmas: np.ndarray, blocks_per_sigma: int, block: int, seed: int = 2605) -> np.ndarray:
    """fp32 [len(sigmas) * blocks_per_sigma, block]: rows of sigma i are i.i.d. N(0, sigma_i^2)."""
    rng = np.random.Generator(np.random.Philox(seed + block))
    x = rng.standard_normal((len(sigmas), blocks_per_sigma, block), dtype=np.float32)
    x *= sigmas.astype(np.float32)[:, None, None]
    return x.reshape(len(sigmas) * blocks_per_sigma, block)


def run(n_sigmas: int = 151, blocks_per_sigma: int = 50000, scale_fmt: int = 1) -> dict:
    import torch

    from . import mxq

    sig = study_sigmas(n_sigmas)
    out = {"sigma": [float(s) for s in sig], "blocks_per_sigma": blocks_per_sigma, "mse": {}}
    for name in RECIPES:
        out["mse"][name] = {}
    for b in BLOCKS:
        x = mxq.from_bits(study_tensor(sig, blocks_per_sigma, b))
        for name, rec in RECIPES.items():
            _, _, sse = mxq.quantize(x, b, scale_fmt, rec)
            torch.cuda.synchronize()
            per_sigma = sse.view(n_sigmas, blocks_per_sigma).to(torch.float64).sum(1) / (blocks_per_sigma * b)
            out["mse"][name][str(b)] = [float(v) for v in per_sigma.cpu()]
    return out


def timed(n_sigmas: int = 151, blocks_per_sigma: int = 50000, scale_fmt: int = 1, repeats: int = 3) -> list:
    """The same 20 launches timed one by one with events on the launch stream (mean of `repeats`
    launches after one warm-up): rows of {"recipe", "block", "elements", "ms", "gelem_s"}.  Between two timed launches a 512 MB fill
    pushes the input out of the 256 MB Infinity Cache (the b = 4 tensor alone would fit)."""
    import torch

    from . import mxq

    sig = study_sigmas(n_sigmas)
    flush = torch.empty(512 << 20, dtype=torch.uint8, device="cuda")
    rows = []
    for b in BLOCKS:
        x = mxq.from_bits(study_tensor(sig, blocks_per_sigma, b))
        r, c = x.shape
        codes = torch.empty((r, c // 2), dtype=torch.uint8, device="cuda")
        scales = torch.empty((r, c // b), dtype=torch.uint8, device="cuda")
        sse = torch.empty((r, c // b), dtype=torch.float32, device="cuda")
        for name, rec in RECIPES.items():
            total = 0.0
            for it in range(repeats + 1):                     # the first launch is a warm-up
                flush.fill_(1)
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                mxq.quantize(x, b, scale_fmt, rec, codes_out=codes, scales_out=scales, sse_out=sse)
                e1.record()
                e1.synchronize()
                if it > 0:
                    total += e0.elapsed_time(e1)
            ms = total / repeats
            rows.append({"recipe": name, "block": b, "elements": r * c, "ms": round(ms, 5),
                         "gelem_s": round(r * c / ms / 1e6, 1)})
        del x, codes, scales, sse
    return rows


def main() -> None:
    ap = argparse.ArgumentParser()
    ap.add_argument("--out", default="")
    ap.add_argument("--sigmas", type=int, default=151)
    ap.add_argument("--blocks-per-sigma", type=int, default=50000)
    args = ap.parse_args()
    res = run(args.sigmas, args.blocks_per_sigma)
    text = json.dumps(res)
    if args.out:
        with open(args.out, "w") as f:
            f.write(text)
    else:
        sys.stdout.write(text + "\n")


if __name__ == "__main__":
    main()
