#!/usr/bin/env python3
"""Benchmark of the microscaled-FP4 quantisation hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

One *step* is one pass of the whole hot path over the bf16 4096 x 14336 Student-t weight
matrix (the LLM MLP up-projection shape): every streaming recipe at every block size of that
configuration, hierarchical scaling (tensor abs-max + quantise with the per-tensor scale), the
power-of-two and UE5M3 scale formats, the brute-force scale search (E4M3 and UE5M3, block 16
and 4) and one de-quantise.  Inputs are resident in HBM before the timed region; launches
rotate over several copies of the input and of the output buffers so that no launch finds
its data in the 256 MB Infinity Cache.

Prints ONE JSON line: whole-step throughput in GElem/s (element-passes quantised per second),
a per-recipe breakdown, the roofline of the kernel that dominates the step (measured with
events around every launch inside the timed region), the HBM roofline of the streaming
kernel, and the CPU oracle timed on a bounded sample of the same workload.
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

ROWS, COLS = 4096, 14336
N_ELEM = ROWS * COLS
HBM_PEAK_GBS = 8000.0            # MI355X HBM3E
FP32_VECTOR_PEAK_TFLOPS = 157.3  # MI355X fp32 vector (packed FMA) peak
N_SETS = 8                       # rotating buffer sets (8 x ~150-260 MB of traffic each)

E8M0, E4M3, UE5M3 = 0, 1, 2
ABSMAX, ABSMAX_PZ, FOUR6, FOUR6_PZ, BRUTE = 0, 1, 2, 3, 4
REC = {ABSMAX: "absmax", ABSMAX_PZ: "absmax_pz", FOUR6: "4over6", FOUR6_PZ: "4over6_pz", BRUTE: "brute"}
FMT = {E8M0: "e8m0", E4M3: "e4m3", UE5M3: "ue5m3"}
NCAND = {E4M3: 126, UE5M3: 254}


def pass_list():
    """(kind, name, block, fmt, recipe, hierarchical) for every launch of one step."""
    p = []
    for b in (8, 16, 32, 64):
        for r in (ABSMAX, ABSMAX_PZ, FOUR6):
            p.append(("quant", f"{REC[r]}_e4m3_b{b}", b, E4M3, r, False))
    p.append(("absmax", "tensor_absmax", 0, 0, 0, False))
    p.append(("quant", "absmax_e4m3_b16_H", 16, E4M3, ABSMAX, True))
    p.append(("quant", "4over6_e4m3_b16_H", 16, E4M3, FOUR6, True))
    p.append(("quant", "absmax_e8m0_b32", 32, E8M0, ABSMAX, False))
    p.append(("quant", "absmax_ue5m3_b16", 16, UE5M3, ABSMAX, False))
    for fmt in (E4M3, UE5M3):
        for b in (16, 4):
            p.append(("quant", f"brute_{FMT[fmt]}_b{b}", b, fmt, BRUTE, False))
    p.append(("dequant", "dequantize_e4m3_b16_bf16", 16, E4M3, 0, False))
    return p


def algorithmic_bytes(kind, block, in_bytes=2):
    """Bytes one launch must move: input once, codes, scale byte + fp32 SSE per block."""
    if kind == "absmax":
        return N_ELEM * in_bytes
    if kind == "dequant":
        return N_ELEM * (0.5 + 1.0 / block + 2)
    return N_ELEM * (in_bytes + 0.5 + 5.0 / block)


def cpu_baseline(x_np, passes, T, rows):
    """The oracle, as it stands, on the first `rows` rows of the same tensor, same pass list."""
    import numpy as np
    import oracle
    xs = np.ascontiguousarray(x_np[:rows])
    oracle.quantize(xs[:8], 16, E4M3, ABSMAX)            # load the library outside the timing
    t0 = time.perf_counter()
    n_q = 0
    for kind, name, b, fmt, rec, hier in passes:
        if kind == "quant":
            oracle.quantize(xs, b, fmt, rec, tensor_scale=T if hier else 1.0)
            n_q += xs.size
        elif kind == "absmax":
            oracle.tensor_absmax(xs)
        else:
            c, s, _ = oracle.quantize(xs, b, fmt, ABSMAX)
            oracle.dequantize(c, s, b, fmt, 1.0, oracle.DT_BF16)
    dt = time.perf_counter() - t0
    return {"value": n_q / dt / 1e9, "unit": "GElem/s", "cores": oracle.num_threads(),
            "kind": "oracle", "seconds": round(dt, 2),
            "sample": f"first {rows} of {ROWS} rows of the same tensor, same pass list as one step "
                      f"({n_q // xs.size} quantise passes incl. 4 brute-force, 1 abs-max, 1 de-quantise)"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--cpu-rows", type=int, default=384, help="rows of the oracle's timed sample")
    ap.add_argument("--no-cpu", action="store_true", help="skip the oracle timing")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.exit("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
                 "run it with --gpus 1. See DESIGN.md for how the path would shard.")

    import numpy as np
    import torch
    from paper_2605_08565_amd import mxq, workloads as W

    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    mxq.lib()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    x_np = W.config2()
    x0 = mxq.from_bits(x_np)
    xs = [x0] + [x0.clone() for _ in range(N_SETS - 1)]
    nb_max = N_ELEM // 4
    outs = [(torch.empty((ROWS, COLS // 2), dtype=torch.uint8, device=dev),
             torch.empty(nb_max, dtype=torch.uint8, device=dev),
             torch.empty(nb_max, dtype=torch.float32, device=dev)) for _ in range(N_SETS)]
    deq = [torch.empty((ROWS, COLS), dtype=torch.bfloat16, device=dev) for _ in range(2)]
    amax_buf = torch.empty(1, dtype=torch.float32, device=dev)

    A = float(mxq.tensor_absmax(x0).cpu()[0])
    T = mxq.tensor_scale_from_absmax(A, E4M3)
    passes = pass_list()
    n_quant = sum(1 for p in passes if p[0] == "quant")

    # a valid (codes, scales) pair for the de-quantise pass
    dq_codes, dq_scales, _ = mxq.quantize(x0, 16, E4M3, ABSMAX)
    torch.cuda.synchronize()

    counter = [0]

    def launch(p):
        kind, name, b, fmt, rec, hier = p
        k = counter[0] % N_SETS
        counter[0] += 1
        if kind == "quant":
            c, s, e = outs[k]
            nb = N_ELEM // b
            mxq.quantize(xs[k], b, fmt, rec, tensor_scale=T if hier else 1.0, codes_out=c,
                         scales_out=s[:nb].view(ROWS, COLS // b), sse_out=e[:nb].view(ROWS, COLS // b))
        elif kind == "absmax":
            mxq.tensor_absmax(xs[k], out=amax_buf)
        else:
            mxq.dequantize(dq_codes, dq_scales, b, fmt, 1.0, out=deq[k % 2])

    for _ in range(args.warmup):
        for p in passes:
            launch(p)
    torch.cuda.synchronize()

    ev = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
           for _ in passes] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.steps):
        for i, p in enumerate(passes):
            ev[s][i][0].record()
            launch(p)
            ev[s][i][1].record()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0

    ms_per_step = dt / args.steps * 1e3
    value = n_quant * N_ELEM / (dt / args.steps) / 1e9

    kern = []
    for i, p in enumerate(passes):
        kind, name, b, fmt, rec, hier = p
        ms = float(np.mean([ev[s][i][0].elapsed_time(ev[s][i][1]) for s in range(args.steps)]))
        row = {"name": name, "ms": round(ms, 4), "gelem_s": round(N_ELEM / ms / 1e6, 1)}
        if rec == BRUTE and kind == "quant":
            flops = N_ELEM * NCAND[fmt] * 6.0
            row.update(bound="alu", tflop_s=round(flops / ms / 1e9, 2),
                       frac=round(flops / ms / 1e9 / FP32_VECTOR_PEAK_TFLOPS, 4))
        else:
            by = algorithmic_bytes(kind, b)
            row.update(bound="hbm", gb_s=round(by / ms / 1e6, 1),
                       frac=round(by / ms / 1e6 / HBM_PEAK_GBS, 4))
        kern.append(row)

    dom = max(kern, key=lambda r: r["ms"])
    if dom["bound"] == "alu":
        roofline = {"bound": "alu", "kernel": dom["name"], "achieved": dom["tflop_s"],
                    "peak": FP32_VECTOR_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": dom["frac"],
                    "traffic": None, "avg_launch_ms": dom["ms"],
                    "note": "6 flops per (element x candidate): scale, round, residual FMA, square-add FMA"}
    else:
        roofline = {"bound": "hbm", "kernel": dom["name"], "achieved": dom["gb_s"], "peak": HBM_PEAK_GBS,
                    "unit": "GB/s", "frac": dom["frac"], "traffic": None, "avg_launch_ms": dom["ms"]}
    st = next(r for r in kern if r["name"] == "absmax_e4m3_b16")
    roofline_stream = {"bound": "hbm", "kernel": st["name"], "achieved": st["gb_s"], "peak": HBM_PEAK_GBS,
                       "unit": "GB/s", "frac": st["frac"], "traffic": None, "avg_launch_ms": st["ms"],
                       "bytes_per_elem": 2.8125}

    out = {
        "metric": "GElem/s quantized per recipe (absmax, 4-over-6, brute-force); % HBM/VALU roof",
        "value": round(value, 3), "unit": "GElem/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "bf16 4096x14336 Student-t(df=4)*0.02 weights; one step = "
                               f"{n_quant} quantise passes (12 streaming E4M3 b8-64, 2 hierarchical, "
                               "E8M0, UE5M3, 4 brute-force) + tensor abs-max + de-quantise",
                   "elements": N_ELEM, "quantise_passes_per_step": n_quant, "tensor_scale": T},
        "per_recipe_gelem_s": {r["name"]: r["gelem_s"] for r in kern},
        "roofline": roofline,
        "roofline_stream": roofline_stream,
        "kernels": kern,
    }
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(x_np, passes, T, args.cpu_rows)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
