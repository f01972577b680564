#!/usr/bin/env python3
"""Benchmark of the microscaled-FP4 quantisation hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

One *step* is one pass of the whole hot path over a batch of eight bf16 4096 x 14336 Student-t
weight matrices (the LLM MLP up-projection shape): every streaming recipe at every block size
of that configuration, hierarchical scaling (tensor abs-max + quantise with the per-tensor
scale), the power-of-two and UE5M3 scale formats, the brute-force scale search (E4M3 and UE5M3,
block 16 and 4) and one de-quantise.  Inputs are resident in HBM before the timed region; each
pass type runs over the eight matrices back to back, so no launch finds its data in the 256 MB
Infinity Cache and one event pair brackets eight launches of the same kernel.

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
N_SETS = 8                       # matrices in the batch (each launch moves 150-260 MB)

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


KERNEL_OF_PASS = {   # pass name -> kernel instantiation, as rocprofv3 prints it
    "absmax_e4m3_b16": "mxq::stream_kernel<0, 16, 1, false, 0>",
    "absmax_pz_e4m3_b16": "mxq::stream_kernel<0, 16, 1, false, 0>",
    "4over6_e4m3_b16": "mxq::stream_kernel<0, 16, 1, true, 0>",
    "absmax_e4m3_b16_H": "mxq::stream_kernel<0, 16, 1, false, 1>",
    "brute_e4m3_b16": "mxq::brute_kernel<0, 16, 1, false, false>",
    "brute_ue5m3_b16": "mxq::brute_kernel<0, 16, 2, false, false>",
    "brute_e4m3_b4": "mxq::brute_kernel<0, 4, 1, false, false>",
    "brute_ue5m3_b4": "mxq::brute_kernel<0, 4, 2, false, false>",
    "dequantize_e4m3_b16_bf16": "mxq::dequant_bf16_kernel<16>",
    "tensor_absmax": "mxq::absmax_kernel<0>",
}


def measured_traffic(pass_name):
    """HBM bytes per launch from the committed rocprofv3 counter summary (FETCH_SIZE and
    WRITE_SIZE runs, scaled by a plain copy of known size); None if that kernel is not in it."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic_bf16_4096x14336.md")
    kern = KERNEL_OF_PASS.get(pass_name)
    if kern is None or not os.path.exists(path):
        return None
    for line in open(path):
        cells = [c.strip() for c in line.split("|")]
        if len(cells) > 7 and cells[1] == f"`{kern}`":
            return round(float(cells[6]) * 1e6)
    return None


def measured_valu_busy(pass_name):
    """VALU-busy percentage of that kernel from the committed rocprofv3 counter summary."""
    path = os.path.join(ROOT, "profiles", "valu_counters_bf16_4096x14336.md")
    kern = KERNEL_OF_PASS.get(pass_name)
    if kern is None or not os.path.exists(path):
        return None
    for line in open(path):
        cells = [c.strip() for c in line.split("|")]
        if len(cells) > 8 and cells[1] == f"`{kern}`":
            return float(cells[7].rstrip(" %"))
    return None


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
    ap.add_argument("--cpu-rows", type=int, default=1024, help="rows of the oracle's timed sample")
    ap.add_argument("--no-cpu", action="store_true", help="skip the oracle timing")
    ap.add_argument("--only", type=str, default="", help="comma-separated pass names (profiling aid)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run plain device copies of one matrix (known size) for counter calibration")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.exit("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
                 "run it with --gpus 1 (blocks are independent, so rows shard with no exchange; only the "
                 "tensor abs-max of hierarchical scaling would need one 4-byte max-all-reduce).")

    import numpy as np
    import torch
    from paper_2605_08565_amd import mxq, workloads as W

    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    mxq.lib()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    # The batch: N_SETS weight matrices.  Matrix 0 is the seeded tensor; the others are row
    # rotations of it (same distribution, distinct addresses), which keeps start-up short.
    x_np = W.config2()
    x0 = mxq.from_bits(x_np)
    xs = [x0] + [torch.roll(x0, shifts=37 * k, dims=0).contiguous() for k in range(1, N_SETS)]
    nb_max = N_ELEM // 4
    outs = [(torch.empty((ROWS, COLS // 2), dtype=torch.uint8, device=dev),
             torch.empty(nb_max, dtype=torch.uint8, device=dev),
             torch.empty(nb_max, dtype=torch.float32, device=dev)) for _ in range(N_SETS)]
    deq = [torch.empty((ROWS, COLS), dtype=torch.bfloat16, device=dev) for _ in range(N_SETS)]
    amax_buf = torch.empty(N_SETS, dtype=torch.float32, device=dev)

    A = float(mxq.tensor_absmax(x0).cpu()[0])
    T = mxq.tensor_scale_from_absmax(A, E4M3)
    passes = pass_list()
    if args.only:
        keep = set(args.only.split(","))
        passes = [p for p in passes if p[1] in keep]
    n_quant = sum(1 for p in passes if p[0] == "quant")

    # a valid (codes, scales) pair per matrix for the de-quantise pass
    dq = [mxq.quantize(x, 16, E4M3, ABSMAX)[:2] for x in xs]
    torch.cuda.synchronize()

    def launch(p, k):
        kind, name, b, fmt, rec, hier = p
        if kind == "quant":
            c, s, e = outs[k]
            nb = N_ELEM // b
            mxq.quantize(xs[k], b, fmt, rec, tensor_scale=T if hier else 1.0, codes_out=c,
                         scales_out=s[:nb].view(ROWS, COLS // b), sse_out=e[:nb].view(ROWS, COLS // b))
        elif kind == "absmax":
            mxq.tensor_absmax(xs[k], out=amax_buf[k:k + 1])
        else:
            mxq.dequantize(dq[k][0], dq[k][1], b, fmt, 1.0, out=deq[k])

    def step(events=None):
        # one pass of the whole hot path over the batch: every pass type over all matrices;
        # consecutive launches touch different matrices (> 1 GB between re-uses of any buffer)
        for i, p in enumerate(passes):
            if events is not None:
                events[i][0].record()
            for k in range(N_SETS):
                launch(p, k)
            if events is not None:
                events[i][1].record()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    ev = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
           for _ in passes] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.steps):
        step(ev[s])
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0

    # Reported separately, outside the timed step: the bound-pruned brute-force search (same
    # bytes out as the full enumeration, fewer candidates tried).
    extra = []
    if not args.only:
        for fmt in (E4M3, UE5M3):
            for b in (16, 4):
                p = ("quant", f"brute_pruned_{FMT[fmt]}_b{b}", b, fmt, 5, False)
                for k in range(N_SETS):
                    launch(p, k)
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for _ in range(2):
                    for k in range(N_SETS):
                        launch(p, k)
                e1.record()
                torch.cuda.synchronize()
                ms = e0.elapsed_time(e1) / (2 * N_SETS)
                extra.append({"name": p[1], "ms": round(ms, 5), "gelem_s": round(N_ELEM / ms / 1e6, 1),
                              "note": "bit-identical to the full enumeration; not part of the timed step"})

    # Also outside the timed step: hierarchical scaling as an activation tensor meets it (bf16
    # 8192 x 4096, 1 % outlier channels): tensor abs-max, then the quantise pass on the SAME tensor,
    # which takes its per-tensor scale from the abs-max in device memory (no host round trip).
    # "cold": 8 tensors in rotation (750 MB between re-uses); "warm": one tensor over and over, so
    # the second pass finds its 67 MB input in the 256 MB Infinity Cache.
    if not args.only:
        x3 = mxq.from_bits(W.config3())
        r3, c3 = x3.shape
        n3 = r3 * c3
        xs3 = [x3] + [torch.roll(x3, shifts=41 * k, dims=0).contiguous() for k in range(1, N_SETS)]
        t_buf = torch.ones(N_SETS, dtype=torch.float32, device=dev)

        def two_pass(k, rec):
            c, s_, e = outs[k]
            mxq.tensor_absmax(xs3[k], out=amax_buf[k:k + 1])
            mxq.quantize_hier(xs3[k], 16, E4M3, rec, amax_buf[k:k + 1], tensor_scale_out=t_buf[k:k + 1],
                              codes_out=c.view(-1)[:n3 // 2].view(r3, c3 // 2),
                              scales_out=s_[:n3 // 16].view(r3, c3 // 16), sse_out=e[:n3 // 16].view(r3, c3 // 16))

        for rec, rname in ((ABSMAX, "absmax"), (2, "4over6")):
            for mode in ("cold", "warm"):
                order = list(range(N_SETS)) if mode == "cold" else [0] * N_SETS
                for k in order:
                    two_pass(k, rec)
                torch.cuda.synchronize()
                # three short launches per tensor: replayed as one HIP graph so that the host's
                # launch rate does not enter the figure
                g, side = torch.cuda.CUDAGraph(), torch.cuda.Stream()
                with torch.cuda.graph(g, stream=side):
                    for k in order:
                        two_pass(k, rec)
                g.replay()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for _ in range(4):
                    g.replay()
                e1.record()
                torch.cuda.synchronize()
                ms = e0.elapsed_time(e1) / (4 * N_SETS)
                extra.append({"name": f"activations_8192x4096_absmax_then_{rname}_b16_H_{mode}", "ms": round(ms, 5),
                              "gelem_s": round(n3 / ms / 1e6, 1),
                              "note": "two launches + the one-thread clear kernel per tensor, the per-tensor scale derived "
                                      "on the device from the abs-max (mxq_quantize_hier); not part of the timed step"})
        del xs3, x3

    if args.calibrate_copy:
        for k in range(N_SETS):
            deq[k].copy_(xs[k])                       # 117 440 512 bytes read + the same written
        torch.cuda.synchronize()

    ms_per_step = dt / args.steps * 1e3
    value = n_quant * N_SETS * N_ELEM / (dt / args.steps) / 1e9

    kern = []
    for i, p in enumerate(passes):
        kind, name, b, fmt, rec, hier = p
        # average duration of ONE launch: events bracket N_SETS back-to-back launches
        ms = float(np.mean([ev[s][i][0].elapsed_time(ev[s][i][1]) for s in range(args.steps)])) / N_SETS
        row = {"name": name, "ms": round(ms, 5), "gelem_s": round(N_ELEM / ms / 1e6, 1)}
        if rec == BRUTE and kind == "quant":
            flops = N_ELEM * NCAND[fmt] * 6.0
            row.update(bound="alu", tflop_s=round(flops / ms / 1e9, 2),
                       frac=round(flops / ms / 1e9 / FP32_VECTOR_PEAK_TFLOPS, 4))
        else:
            by = algorithmic_bytes(kind, b)
            row.update(bound="hbm", gb_s=round(by / ms / 1e6, 1),
                       frac=round(by / ms / 1e6 / HBM_PEAK_GBS, 4))
        kern.append(row)

    def roof(r, extra=None):
        if r["bound"] == "alu":
            d = {"bound": "alu", "kernel": r["name"], "achieved": r["tflop_s"],
                 "peak": FP32_VECTOR_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": r["frac"], "traffic": measured_traffic(r["name"]),
                 "avg_launch_ms": r["ms"],
                 "frac_of_unpacked_fma_peak": round(r["tflop_s"] / (FP32_VECTOR_PEAK_TFLOPS / 2), 4),
                 "valu_busy_pct_rocprof": measured_valu_busy(r["name"]),
                 "note": "algorithmic work = 6 flops per (element x candidate): scale, round, residual "
                         "FMA, square + add; peak is the packed-FMA fp32 vector peak (packed fp32 is "
                         "not available to this build: the unpacked FMA peak is half of it)"}
        else:
            d = {"bound": "hbm", "kernel": r["name"], "achieved": r["gb_s"], "peak": HBM_PEAK_GBS,
                 "unit": "GB/s", "frac": r["frac"], "traffic": measured_traffic(r["name"]),
                 "avg_launch_ms": r["ms"]}
        if extra:
            d.update(extra)
        return d

    # dominant kernel: the launch with the most algorithmic work (254 candidates); b=16 and b=4
    # take the same time within run-to-run noise, so the choice between them is fixed, not timed
    dom = next((r for r in kern if r["name"] == "brute_ue5m3_b16"), max(kern, key=lambda r: r["ms"]))
    out = {
        "metric": "GElem/s quantized per recipe (absmax, 4-over-6, brute-force); % HBM/VALU roof",
        "value": round(value, 3), "unit": "GElem/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"batch of {N_SETS} bf16 4096x14336 Student-t(df=4)*0.02 weight matrices; "
                               f"one step = {n_quant} quantise passes per matrix (12 streaming E4M3 "
                               "b8-64, 2 hierarchical, E8M0, UE5M3, 4 brute-force) + tensor abs-max + "
                               "de-quantise",
                   "elements_per_matrix": N_ELEM, "matrices": N_SETS,
                   "quantise_passes_per_matrix": n_quant, "tensor_scale": T},
        "per_recipe_gelem_s": {r["name"]: r["gelem_s"] for r in kern},
        "roofline": roof(dom),
        "kernels": kern,
        "extra_kernels": extra,
    }
    st = [r for r in kern if r["name"] == "absmax_e4m3_b16"]
    if st:
        out["roofline_stream"] = roof(st[0], {"bytes_per_elem": 2.8125})
    f6 = [r for r in kern if r["name"] == "4over6_e4m3_b16"]
    if f6:
        out["roofline_4over6"] = roof(f6[0], {"bytes_per_elem": 2.8125})
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(x_np, passes, T, args.cpu_rows)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
