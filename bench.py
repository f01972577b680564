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
kernels, the attainable HBM ceilings measured in the same run (read-only, copy, fill), a
`configs` object with one timed row per configuration / block size of the other workloads
(fp32 matrix, activation tensor with hierarchical scaling, the 32-layer model sweep, the
appendix diagnostics), and the CPU oracle timed on a bounded sample of the step's workload.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

ROWS, COLS = 4096, 14336
N_ELEM = ROWS * COLS
HBM_PEAK_GBS = 8000.0            # MI355X HBM3E
FP32_VECTOR_PEAK_TFLOPS = 157.3  # MI355X fp32 vector (packed FMA) peak
LANE_OPS_PEAK = 256 * 4 * 16 * 2.4e9   # unpacked vector issue: 39.3 T lane-operations / s
N_SETS = 8                       # matrices in the batch (each launch moves 150-260 MB)

E8M0, E4M3, UE5M3 = 0, 1, 2
ABSMAX, ABSMAX_PZ, FOUR6, FOUR6_PZ, BRUTE, BRUTE_PRUNED = 0, 1, 2, 3, 4, 5
REC = {ABSMAX: "absmax", ABSMAX_PZ: "absmax_pz", FOUR6: "4over6", FOUR6_PZ: "4over6_pz", BRUTE: "brute",
       BRUTE_PRUNED: "brute_pruned"}
FMT = {E8M0: "e8m0", E4M3: "e4m3", UE5M3: "ue5m3"}
NCAND = {E8M0: 255, E4M3: 126, UE5M3: 254}

# Workloads (tag -> rows, cols, dtype bytes, number of rotating buffer sets, description)
WORKLOADS = {
    "w2": (4096, 14336, 2, 8, "bf16 4096x14336 Student-t(df=4)*0.02 weights (configs 2 and 4)"),
    "a3": (8192, 4096, 2, 8, "bf16 8192x4096 N(0,1) activations, 1 % outlier channels x50 (config 3)"),
    "f1": (1024, 4096, 4, 16, "fp32 1024x4096 N(0,1) (config 1)"),
    "f2": (4096, 14336, 4, 4, "fp32 4096x14336 (the weights of config 2 widened to fp32)"),
}


def step_passes():
    """(kind, name, block, fmt, recipe, hierarchical) for every launch of one step."""
    # Order: the HBM-bound passes first, then the issue-bound streaming passes, brute force last.
    # For about a millisecond after the brute-force passes the chip runs vector-bound kernels
    # some 20 % slower (measured with the step in both orders: the slow-down follows whichever
    # passes come next, and HBM-bound passes do not notice it), so the passes that would feel it
    # are kept away from the step boundary.
    p = []
    for b in (8, 16, 32, 64):
        for r in (ABSMAX, ABSMAX_PZ):
            p.append(("quant", f"{REC[r]}_e4m3_b{b}", b, E4M3, r, False))
    p.append(("quant", "absmax_e8m0_b32", 32, E8M0, ABSMAX, False))
    p.append(("quant", "absmax_ue5m3_b16", 16, UE5M3, ABSMAX, False))
    p.append(("dequant", "dequantize_e4m3_b16_bf16", 16, E4M3, 0, False))
    p.append(("absmax", "tensor_absmax", 0, 0, 0, False))
    p.append(("quant", "absmax_e4m3_b16_H", 16, E4M3, ABSMAX, True))
    for b in (8, 16, 32, 64):
        p.append(("quant", f"4over6_e4m3_b{b}", b, E4M3, FOUR6, False))
    p.append(("quant", "4over6_e4m3_b16_H", 16, E4M3, FOUR6, True))
    for fmt in (E4M3, UE5M3):
        for b in (16, 4):
            p.append(("quant", f"brute_{FMT[fmt]}_b{b}", b, fmt, BRUTE, False))
    return p


def extra_passes():
    """(workload, kind, name, block, fmt, recipe, hierarchical) timed outside the step, each as a
    HIP graph over all buffer sets of its workload."""
    p = []
    # config-2 tensor: what the step leaves out (b = 2, 4, 128; the pruned search; power-of-two
    # brute force; fp32 de-quantise; the two other abs-max forms; the appendix diagnostics)
    for b in (2, 4, 128):
        for r in (ABSMAX, FOUR6):
            p.append(("w2", "quant", f"{REC[r]}_e4m3_b{b}", b, E4M3, r, False))
    for fmt in (E4M3, UE5M3):
        for b in (16, 4):
            p.append(("w2", "quant", f"brute_pruned_{FMT[fmt]}_b{b}", b, fmt, BRUTE_PRUNED, False))
    p.append(("w2", "quant", "brute_e8m0_b32", 32, E8M0, BRUTE, False))
    # the wider scale format with 4-over-6 and with the per-tensor scale
    p.append(("w2", "quant", "4over6_ue5m3_b16", 16, UE5M3, FOUR6, False))
    p.append(("w2", "quant", "absmax_ue5m3_b16_H", 16, UE5M3, ABSMAX, True))
    p.append(("w2", "quant", "4over6_ue5m3_b16_H", 16, UE5M3, FOUR6, True))
    p.append(("w2", "dequant_f32", "dequantize_e4m3_b16_f32", 16, E4M3, 0, False))
    p.append(("w2", "absmax_2launch", "tensor_absmax_two_launches", 0, 0, 0, False))
    p.append(("w2", "absmax_ws", "tensor_absmax_workspace", 0, 0, 0, False))
    p.append(("w2", "quant_clip", "absmax_e4m3_b16_with_clip_sse", 16, E4M3, ABSMAX, False))
    p.append(("w2", "clip", "clip_sse_e4m3_b16", 16, E4M3, 0, False))
    p.append(("w2", "hist", "histogram_b16", 16, E4M3, 0, False))
    p.append(("w2", "hist", "histogram_b4", 4, E4M3, 0, False))
    # config 1 and its full-size fp32 counterpart
    p.append(("f1", "quant", "config1_f32_1024x4096_absmax_e4m3_b16", 16, E4M3, ABSMAX, False))
    p.append(("f1", "quant_batch", "config1_f32_1024x4096_absmax_e4m3_b16_batched_x16", 16, E4M3, ABSMAX, False))
    for r in (ABSMAX, FOUR6):
        p.append(("f2", "quant", f"f32_4096x14336_{REC[r]}_e4m3_b16", 16, E4M3, r, False))
    p.append(("f2", "absmax", "f32_4096x14336_tensor_absmax", 0, 0, 0, False))
    # config 3: pre-pass alone, then all 10 runs as the two-pass (abs-max + quantise with the scale
    # taken from device memory), cold (8 tensors in rotation) and warm (one tensor over and over)
    p.append(("a3", "absmax", "config3_tensor_absmax", 0, 0, 0, False))
    for b in (4, 8, 16, 32, 64):
        for r in (ABSMAX, FOUR6):
            p.append(("a3", "quant", f"config3_{REC[r]}_e4m3_b{b}_H_quantise_only", b, E4M3, r, True))
            for mode in ("cold", "warm"):
                p.append(("a3", "two_pass_" + mode, f"config3_absmax_then_{REC[r]}_e4m3_b{b}_H_{mode}", b, E4M3, r, True))
    # the search on activations (blocks of very different magnitude share a wavefront)
    for b in (16, 4):
        p.append(("a3", "quant", f"config3_brute_e4m3_b{b}_H", b, E4M3, BRUTE, True))
        p.append(("a3", "quant", f"config3_brute_pruned_e4m3_b{b}_H", b, E4M3, BRUTE_PRUNED, True))
    return p


def algorithmic_bytes(kind, block, n, in_bytes):
    """Bytes one launch must move: input once, codes, scale byte + fp32 SSE per block."""
    if kind.startswith("absmax"):
        return n * in_bytes
    if kind == "dequant":
        return n * (0.5 + 1.0 / block + 2)
    if kind == "dequant_f32":
        return n * (0.5 + 1.0 / block + 4)
    if kind == "clip":
        return n * (in_bytes + 5.0 / block)
    if kind == "hist":
        return n * (0.5 + 1.0 / block)
    if kind == "quant_clip":
        return n * (in_bytes + 0.5 + 9.0 / block)
    if kind.startswith("two_pass"):
        return n * (2 * in_bytes + 0.5 + 5.0 / block)
    return n * (in_bytes + 0.5 + 5.0 / block)


# pass name -> kernel instantiation as rocprofv3 prints it (for the recorded counter figures)
KERNEL_OF_PASS = {
    "absmax_e4m3_b16": "mxq::stream_kernel<0, 16, 1, false, 0, false>",
    "absmax_pz_e4m3_b16": "mxq::stream_kernel<0, 16, 1, false, 0, false>",
    "4over6_e4m3_b16": "mxq::stream_kernel<0, 16, 1, true, 0, false>",
    "4over6_e4m3_b8": "mxq::stream_kernel<0, 8, 1, true, 0, false>",
    "4over6_e4m3_b32": "mxq::stream_kernel<0, 32, 1, true, 0, false>",
    "4over6_e4m3_b64": "mxq::stream_kernel<0, 64, 1, true, 0, false>",
    "absmax_e4m3_b16_H": "mxq::stream_kernel<0, 16, 1, false, 1, false>",
    "4over6_e4m3_b16_H": "mxq::stream_kernel<0, 16, 1, true, 1, false>",
    "brute_e4m3_b16": "mxq::brute_kernel<0, 16, 1, false, false>",
    "brute_ue5m3_b16": "mxq::brute_kernel<0, 16, 2, false, false>",
    "brute_e4m3_b4": "mxq::brute_kernel<0, 4, 1, false, false>",
    "brute_ue5m3_b4": "mxq::brute_kernel<0, 4, 2, false, false>",
    "dequantize_e4m3_b16_bf16": "mxq::dequant_bf16_kernel<16>",
    "tensor_absmax": "mxq::absmax_kernel<0, false>",
}
PROFILE_TRAFFIC = os.path.join(ROOT, "profiles", "hbm_traffic_bf16_4096x14336.md")
PROFILE_VALU = os.path.join(ROOT, "profiles", "valu_counters_bf16_4096x14336.md")
PROFILE_WAIT = os.path.join(ROOT, "profiles", "lds_counters_bf16_4096x14336.md")


def profile_rows(path):
    """{first cell without back-ticks: [other cells]} for every table row of a profile summary,
    and the commit the summary says it was taken at."""
    rows, commit = {}, None
    if not os.path.exists(path):
        return rows, commit
    for line in open(path):
        m = re.search(r"[Tt]aken at commit `?([0-9a-f]{7,40})`?", line)
        if m:
            commit = m.group(1)
        cells = [c.strip() for c in line.strip().strip("|").split("|")]
        if len(cells) > 2 and cells[0].startswith("`"):
            rows[cells[0].strip("`")] = cells[1:]
    return rows, commit


def recorded(pass_name):
    """Counter figures of that pass's kernel from the committed rocprofv3 summaries: HBM bytes per
    launch (FETCH_SIZE + WRITE_SIZE runs, scaled by a plain copy of known size), VALU instructions
    per 8-element chunk, and the shares of resident wavefront time spent waiting for an issue slot
    and waiting for data.  They are RECORDED figures, not measured in this run; the commit they were
    taken at is returned with them."""
    kern = KERNEL_OF_PASS.get(pass_name)
    out = {"traffic": None, "valu_per_chunk": None, "wait_issue_pct": None, "wait_data_pct": None, "commit": None}
    if kern is None:
        return out
    t, c1 = profile_rows(PROFILE_TRAFFIC)
    v, c2 = profile_rows(PROFILE_VALU)
    w, c3 = profile_rows(PROFILE_WAIT)
    out["commit"] = c1 or c2 or c3
    if kern in t:
        out["traffic"] = round(float(t[kern][4]) * 1e6)
    if kern in v:
        out["valu_per_chunk"] = float(v[kern][2])
    if kern in w:
        out["wait_issue_pct"] = float(w[kern][4].rstrip(" %"))
        out["wait_data_pct"] = float(w[kern][5].rstrip(" %"))
    return out


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


class Workload:
    """Rotating buffer sets of one tensor shape, resident on the GPU."""

    def __init__(self, tag, torch, mxq, W, dev):
        rows, cols, in_bytes, n_sets, desc = WORKLOADS[tag]
        self.tag, self.rows, self.cols, self.in_bytes, self.n_sets, self.desc = tag, rows, cols, in_bytes, n_sets, desc
        self.n = rows * cols
        if tag == "w2":
            self.x_np = W.config2()
            x0 = mxq.from_bits(self.x_np)
        elif tag == "a3":
            self.x_np = W.config3()
            x0 = mxq.from_bits(self.x_np)
        elif tag == "f1":
            self.x_np = W.config1()
            x0 = mxq.from_bits(self.x_np)
        else:
            self.x_np = None
            x0 = mxq.from_bits(W.config2()).float()
        # set 0 is the seeded tensor; the others are row rotations of it (same distribution,
        # distinct addresses), which keeps start-up short
        self.xs = [x0] + [torch.roll(x0, shifts=37 * k, dims=0).contiguous() for k in range(1, n_sets)]
        nb_max = self.n // 2
        self.outs = [(torch.empty((rows, cols // 2), dtype=torch.uint8, device=dev),
                      torch.empty(nb_max, dtype=torch.uint8, device=dev),
                      torch.empty(nb_max, dtype=torch.float32, device=dev),
                      torch.empty(nb_max, dtype=torch.float32, device=dev)) for _ in range(n_sets)]
        self.amax = torch.zeros(n_sets, dtype=torch.float32, device=dev)
        self.t_buf = torch.ones(n_sets, dtype=torch.float32, device=dev)
        self.deq = None
        self.dq = None
        self.ws = mxq.absmax_workspace(dev)
        self.eh = torch.empty(8, dtype=torch.int64, device=dev)
        self.sh = torch.empty(256, dtype=torch.int64, device=dev)
        A = float(mxq.tensor_absmax(x0).cpu()[0])
        self.T = mxq.tensor_scale_from_absmax(A, E4M3)
        self.T_by_fmt = {E4M3: self.T, UE5M3: mxq.tensor_scale_from_absmax(A, UE5M3), E8M0: 1.0}

    def views(self, k, b):
        c, s, e, cl = self.outs[k]
        nb = self.n // b
        sh = (self.rows, self.cols // b)
        return c, s[:nb].view(sh), e[:nb].view(sh), cl[:nb].view(sh)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=40)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--cpu-rows", type=int, default=1024, help="rows of the oracle's timed sample")
    ap.add_argument("--no-cpu", action="store_true", help="skip the oracle timing")
    ap.add_argument("--no-configs", action="store_true", help="skip everything outside the timed step")
    ap.add_argument("--only", type=str, default="", help="comma-separated pass names (profiling aid)")
    ap.add_argument("--only-workload", type=str, default="",
                    help="profiling aid: run only the passes of one workload tag (w2, a3, f1, f2), so that every "
                         "kernel instantiation in the trace ran on one tensor shape")
    ap.add_argument("--sweep-layers", type=int, default=2, help="layers of the 32-layer model sweep (config 5) to time")
    ap.add_argument("--no-study", action="store_true", help="skip the timed numerical study (20 launches on fp32 tensors)")
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
    keep = set(args.only.split(",")) if args.only else None
    profiling = bool(keep) or bool(args.only_workload)

    wl_cache = {}

    def workload(tag):
        if tag not in wl_cache:
            wl_cache[tag] = Workload(tag, torch, mxq, W, dev)
        return wl_cache[tag]

    def launch(wl, kind, b, fmt, rec, hier, k, warm=False):
        """One pass on buffer set k of workload wl."""
        x = wl.xs[0 if warm else k]
        if kind == "quant":
            c, s, e, _ = wl.views(k, b)
            if hier == "device":
                mxq.quantize_hier(x, b, fmt, rec, wl.amax[k:k + 1], tensor_scale_out=wl.t_buf[k:k + 1],
                                  codes_out=c, scales_out=s, sse_out=e)
            else:
                mxq.quantize(x, b, fmt, rec, tensor_scale=wl.T_by_fmt[fmt] if hier else 1.0, codes_out=c, scales_out=s,
                             sse_out=e)
        elif kind == "quant_batch":               # all buffer sets in one call (two launches of eight tensors)
            if k == 0:
                mxq.quantize_batch(wl.xs, b, fmt, rec, outs=[wl.views(j, b)[:3] for j in range(wl.n_sets)])
        elif kind == "quant_clip":
            c, s, e, cl = wl.views(k, b)
            mxq.quantize(x, b, fmt, rec, codes_out=c, scales_out=s, sse_out=e, clip_sse_out=cl)
        elif kind == "absmax":                    # running maximum; every call clears the next call's word
            k1 = (k + 1) % wl.n_sets
            mxq.tensor_absmax_acc(x, wl.amax[k:k + 1], clear_word=wl.amax[k1:k1 + 1])
        elif kind == "absmax_2launch":
            mxq.tensor_absmax(x, out=wl.amax[k:k + 1])
        elif kind == "absmax_ws":
            mxq.tensor_absmax(x, out=wl.amax[k:k + 1], workspace=wl.ws)
        elif kind in ("two_pass_cold", "two_pass_warm"):
            c, s, e, _ = wl.views(k, b)
            k1 = (k + 1) % wl.n_sets
            mxq.tensor_absmax_acc(x, wl.amax[k:k + 1], clear_word=wl.amax[k1:k1 + 1])
            mxq.quantize_hier(x, b, fmt, rec, wl.amax[k:k + 1], tensor_scale_out=wl.t_buf[k:k + 1],
                              codes_out=c, scales_out=s, sse_out=e)
        elif kind == "dequant":
            mxq.dequantize(wl.dq[k][0], wl.dq[k][1], b, fmt, 1.0, out=wl.deq[k])
        elif kind == "dequant_f32":
            mxq.dequantize(wl.dq[k][0], wl.dq[k][1], b, fmt, 1.0, out=wl.deq_f32[k % len(wl.deq_f32)])
        elif kind == "clip":
            mxq.clip_sse(x, wl.dq[k][1], b, fmt, out=wl.views(k, b)[3])
        elif kind == "hist":
            mxq.histogram(wl.hq[b][k][0], wl.hq[b][k][1], b, out=(wl.eh, wl.sh))
        else:
            raise ValueError(kind)

    def need_dq(wl):
        if wl.dq is None:                         # a valid (codes, scales) pair per matrix
            wl.dq = [mxq.quantize(x, 16, E4M3, ABSMAX)[:2] for x in wl.xs]
            wl.deq = [torch.empty((wl.rows, wl.cols), dtype=torch.bfloat16, device=dev) for _ in range(wl.n_sets)]
            wl.deq_f32 = [torch.empty((wl.rows, wl.cols), dtype=torch.float32, device=dev) for _ in range(4)]
            wl.hq = {16: wl.dq, 4: [mxq.quantize(x, 4, E4M3, ABSMAX)[:2] for x in wl.xs]}
            torch.cuda.synchronize()

    # ------------------------------------------------------------------ the timed step
    w2 = None
    passes = step_passes()
    if keep is not None:
        passes = [p for p in passes if p[1] in keep]
    if args.only_workload and args.only_workload != "w2":
        passes = []
    out = {}
    if passes:
        w2 = workload("w2")
        need_dq(w2)
        T = w2.T
        n_quant = sum(1 for p in passes if p[0] == "quant")

        def step(events=None):
            # one pass of the whole hot path over the batch: every pass type over all matrices;
            # consecutive launches touch different matrices (> 1 GB between re-uses of any buffer)
            for i, (kind, name, b, fmt, rec, hier) in enumerate(passes):
                if events is not None:
                    events[i][0].record()
                for k in range(N_SETS):
                    launch(w2, kind, b, fmt, rec, hier, k)
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
        ms_per_step = dt / args.steps * 1e3
        value = n_quant * N_SETS * N_ELEM / (dt / args.steps) / 1e9

    # ------------------------------------------------------------------ attainable HBM rates, same run
    # read-only: the library's running-maximum kernel; copy and fill: torch's kernels on the
    # same eight-buffer rotation (a copy moves 2 x 117 MB)
    ceilings = {}
    if passes and not profiling:
        def timed(fn, reps=3):
            for k in range(N_SETS):
                fn(k)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                for k in range(N_SETS):
                    fn(k)
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / (reps * N_SETS)

        by = N_ELEM * 2
        ms_read = timed(lambda k: launch(w2, "absmax", 0, 0, 0, False, k))
        ms_copy = timed(lambda k: w2.deq[k].copy_(w2.xs[(k + 3) % N_SETS]))
        ms_fill = timed(lambda k: w2.deq[k].fill_(1.0))
        ceilings = {"hbm_read_ceiling_gb_s": round(by / ms_read / 1e6, 1),
                    "hbm_copy_ceiling_gb_s": round(2 * by / ms_copy / 1e6, 1),
                    "hbm_fill_ceiling_gb_s": round(by / ms_fill / 1e6, 1),
                    "note": "measured in this run on the step's buffers (117.4 MB per matrix, 8 in rotation): "
                            "read = this library's tensor abs-max kernel, copy / fill = torch's device kernels"}
    copy_gbs = ceilings.get("hbm_copy_ceiling_gb_s")

    def hbm_row(row, by, ms):
        gbs = by / ms / 1e6
        row.update(bound="hbm", gb_s=round(gbs, 1), frac=round(gbs / HBM_PEAK_GBS, 4))
        if copy_gbs:
            row["frac_of_copy"] = round(gbs / copy_gbs, 4)
        return row

    def annotate_valu(row, name):
        """VALU-heavy streaming kernels: the vector-issue time alone, from the recorded counters."""
        r = recorded(name)
        if r["valu_per_chunk"]:
            chunks = N_ELEM / 8
            floor_ms = r["valu_per_chunk"] * chunks * 64 / LANE_OPS_PEAK * 1e3
            row["valu_instr_per_chunk_recorded"] = r["valu_per_chunk"]
            row["valu_issue_floor_ms_at_2p4GHz"] = round(floor_ms, 5)
            row["wait_issue_pct_recorded"] = r["wait_issue_pct"]
            row["wait_data_pct_recorded"] = r["wait_data_pct"]
            row["bound_statement"] = ("limited by vector issue, not by HBM: the recorded counters show more wavefront time "
                                      "waiting for an issue slot than for data, and the vector instructions alone need "
                                      "valu_issue_floor_ms at the nominal clock")

    kern = []
    if passes:
        for i, (kind, name, b, fmt, rec, hier) in enumerate(passes):
            # average duration of ONE launch: events bracket N_SETS back-to-back launches
            ms = float(np.mean([ev[s][i][0].elapsed_time(ev[s][i][1]) for s in range(args.steps)])) / N_SETS
            row = {"name": name, "ms": round(ms, 5), "gelem_s": round(N_ELEM / ms / 1e6, 1)}
            if rec == BRUTE and kind == "quant":
                flops = N_ELEM * NCAND[fmt] * 6.0
                row.update(bound="alu", tflop_s=round(flops / ms / 1e9, 2),
                           frac=round(flops / ms / 1e9 / FP32_VECTOR_PEAK_TFLOPS, 4))
            else:
                hbm_row(row, algorithmic_bytes(kind, b, N_ELEM, 2), ms)
                if rec in (FOUR6, FOUR6_PZ) or hier:
                    annotate_valu(row, name)
            kern.append(row)

    # ------------------------------------------------------------------ passes outside the step
    extra = []
    full_ms = {}
    xp = [] if args.no_configs else extra_passes()
    if keep is not None:
        xp = [p for p in xp if p[2] in keep]
    if args.only_workload:
        xp = [p for p in xp if p[0] == args.only_workload]
    side = torch.cuda.Stream()
    for tag, kind, name, b, fmt, rec, hier in xp:
        wl = workload(tag)
        if kind in ("dequant", "dequant_f32", "clip", "hist"):
            need_dq(wl)
        warm = kind == "two_pass_warm"
        wl.amax.zero_()
        hmode = "device" if (hier and tag == "a3" and kind == "quant" and rec < BRUTE) else hier
        if hmode == "device":                     # the quantise pass alone needs a valid abs-max per set
            for k in range(wl.n_sets):
                wl.amax[k:k + 1].zero_()
                mxq.tensor_absmax_acc(wl.xs[k], wl.amax[k:k + 1])
        order = list(range(wl.n_sets))
        for k in order:
            launch(wl, kind, b, fmt, rec, hmode, k, warm)
        torch.cuda.synchronize()
        reps = 2 if rec in (BRUTE, BRUTE_PRUNED) and kind == "quant" else (20 if tag == "f1" else 4)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        if profiling:
            # under rocprofv3: plain launches, so that every dispatch is traced and counted by itself
            e0.record()
            for _ in range(reps):
                for k in order:
                    launch(wl, kind, b, fmt, rec, hmode, k, warm)
            e1.record()
            torch.cuda.synchronize()
        else:
            # short launches: replayed as one HIP graph so that the host's launch rate does not
            # enter the figure
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=side):
                for k in order:
                    launch(wl, kind, b, fmt, rec, hmode, k, warm)
            g.replay()
            torch.cuda.synchronize()
            e0.record()
            for _ in range(reps):
                g.replay()
            e1.record()
            torch.cuda.synchronize()
            del g
        ms = e0.elapsed_time(e1) / (reps * wl.n_sets)
        row = {"name": name, "workload": tag, "ms": round(ms, 5), "gelem_s": round(wl.n / ms / 1e6, 1)}
        if rec == BRUTE and kind == "quant":
            flops = wl.n * NCAND[fmt] * 6.0
            row.update(bound="alu", tflop_s=round(flops / ms / 1e9, 2),
                       frac=round(flops / ms / 1e9 / FP32_VECTOR_PEAK_TFLOPS, 4))
            full_ms[(tag, b, fmt)] = ms
        elif rec == BRUTE_PRUNED and kind == "quant":
            # no roofline fraction: the variant skips candidates, so the full enumeration's work
            # divided by its time would not be a utilisation
            ref = full_ms.get((tag, b, fmt)) or next((r["ms"] for r in kern if r["name"] == f"brute_{FMT[fmt]}_b{b}"), None)
            row.update(bound="alu", candidates_of_full_search=NCAND[fmt],
                       speedup_vs_full_enumeration=round(ref / ms, 3) if ref else None,
                       note="bit-identical to the full enumeration, fewer candidates tried; reported as a speed-up")
        else:
            hbm_row(row, algorithmic_bytes(kind, b, wl.n, wl.in_bytes), ms)
            row["bytes_per_elem"] = round(algorithmic_bytes(kind, b, wl.n, wl.in_bytes) / wl.n, 4)
        if tag == "f1":
            row["note"] = ("21 MB per launch: bound by launch and ramp-up, not by HBM (reported, no roofline claim)" if kind == "quant"
                           else "mxq_quantize_batch: sixteen such tensors in two launches; time per tensor")
        if warm:
            row["note"] = "same tensor every time: the quantise pass finds its 67 MB input in the 256 MB Infinity Cache"
        extra.append(row)

    # config 5: the 32-layer model sweep, first layers, one HIP graph per (recipe, block size)
    sweep_rows = []
    if not args.no_configs and not profiling and args.sweep_layers > 0:
        for w in list(wl_cache):
            if w != "w2":
                del wl_cache[w]
        torch.cuda.empty_cache()
        from paper_2605_08565_amd import sweep
        res = sweep.run(layer_ids=list(range(args.sweep_layers)), generator="numpy")
        for r in res["rows"]:
            row = {"recipe": r["recipe"], "block": r["block"], "gelem_s": r["gelem_s"], "mse": r["mse"]}
            if r["recipe"] == "e4m3_brute":
                tf = r["gelem_s"] * 1e9 * 126 * 6.0 / 1e12
                row.update(bound="alu", tflop_s=round(tf, 2), frac=round(tf / FP32_VECTOR_PEAK_TFLOPS, 4))
            else:
                gbs = r["gelem_s"] * (2 + 0.5 + 5.0 / r["block"])
                row.update(bound="hbm", gb_s=round(gbs, 1), frac=round(gbs / HBM_PEAK_GBS, 4))
                if copy_gbs:
                    row["frac_of_copy"] = round(gbs / copy_gbs, 4)
            sweep_rows.append(row)

    # the numerical study (MSE against sigma): 20 launches on fp32 tensors of 30 M to 242 M elements
    study_rows = []
    if not args.no_configs and not profiling and not args.no_study:
        for w in list(wl_cache):
            if w != "w2":
                del wl_cache[w]
        torch.cuda.empty_cache()
        from paper_2605_08565_amd import study
        for r in study.timed():
            row = dict(r)
            if r["recipe"] == "brute_force":
                tf = r["gelem_s"] * 1e9 * 126 * 6.0 / 1e12
                row.update(bound="alu", tflop_s=round(tf, 2), frac=round(tf / FP32_VECTOR_PEAK_TFLOPS, 4))
            else:
                gbs = r["gelem_s"] * (4 + 0.5 + 5.0 / r["block"])
                row.update(bound="hbm", gb_s=round(gbs, 1), frac=round(gbs / HBM_PEAK_GBS, 4))
                if copy_gbs:
                    row["frac_of_copy"] = round(gbs / copy_gbs, 4)
            study_rows.append(row)

    if args.calibrate_copy and w2 is not None:
        for k in range(N_SETS):
            w2.deq[k].copy_(w2.xs[k])                 # 117 440 512 bytes read + the same written
        torch.cuda.synchronize()

    if not passes:
        print(json.dumps({"note": "profiling run: no timed step", "extra_kernels": extra}))
        return

    def roof(r, extra_fields=None):
        rec_ = recorded(r["name"])
        if r["bound"] == "alu":
            d = {"bound": "alu", "kernel": r["name"], "achieved": r["tflop_s"],
                 "peak": FP32_VECTOR_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": r["frac"],
                 "traffic": rec_["traffic"], "avg_launch_ms": r["ms"],
                 "frac_of_unpacked_fma_peak": round(r["tflop_s"] / (FP32_VECTOR_PEAK_TFLOPS / 2), 4),
                 "valu_instr_per_chunk_recorded": rec_["valu_per_chunk"],
                 "wait_issue_pct_recorded": rec_["wait_issue_pct"], "wait_data_pct_recorded": rec_["wait_data_pct"],
                 "bound_statement": "issue-bound: %s vector instructions per (8 elements x candidate) "
                                    "against 32 algorithmic ones (recorded counter / 254 candidates); %.2f of the "
                                    "packed-FMA peak, which the instruction set available to this build (no packed "
                                    "fp32) caps at 0.50 even for a pure-FMA stream"
                                    % ("%.1f" % (rec_["valu_per_chunk"] / 254.0) if rec_["valu_per_chunk"] else "about 35",
                                       r["frac"]),
                 "note": "algorithmic work = 6 flops per (element x candidate): scale, round, residual "
                         "FMA, square + add; peak is the packed-FMA fp32 vector peak (packed fp32 is "
                         "not available to this build: the unpacked FMA peak is half of it)"}
        else:
            d = {"bound": "hbm", "kernel": r["name"], "achieved": r["gb_s"], "peak": HBM_PEAK_GBS,
                 "unit": "GB/s", "frac": r["frac"], "traffic": rec_["traffic"], "avg_launch_ms": r["ms"]}
            if "frac_of_copy" in r:
                d["frac_of_copy"] = r["frac_of_copy"]
        d["traffic_is"] = "recorded: committed rocprofv3 summaries under profiles/, not measured in this run"
        d["recorded_at_commit"] = rec_["commit"]
        if extra_fields:
            d.update(extra_fields)
        return d

    # dominant kernel: the launch with the most algorithmic work (254 candidates); b=16 and b=4
    # take the same time within run-to-run noise, so the choice between them is fixed, not timed
    dom = next((r for r in kern if r["name"] == "brute_ue5m3_b16"), max(kern, key=lambda r: r["ms"]))
    by_name = {r["name"]: r for r in extra}
    configs = {
        "config1": [by_name[n] for n in by_name if n.startswith("config1_") or n.startswith("f32_")],
        "config2": {"rows_in": "kernels", "names": [r["name"] for r in kern if re.match(r"(absmax|absmax_pz|4over6)_e4m3_b(8|16|32|64)$", r["name"])]},
        "config3": [by_name[n] for n in by_name if n.startswith("config3_")],
        "config4": {"rows_in": "kernels", "names": [r["name"] for r in kern if r["name"].startswith("brute_")]},
        "config5": {"layers": args.sweep_layers, "generator": "numpy (workloads.layer_matrix: the bytes the parity tests check)",
                    "rows": sweep_rows},
        "numerical_study": {"what": "151 sigmas x 50 000 blocks per block size, fp32 N(0, sigma^2), E4M3 scales; one "
                                    "launch per (recipe, block size), 512 MB flushed through the caches between launches",
                            "rows": study_rows},
        "diagnostics_and_other_blocks": [r for r in extra if r["workload"] == "w2"],
    }
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
        "ceilings": ceilings,
        "kernels": kern,
        "configs": configs,
    }
    st = [r for r in kern if r["name"] == "absmax_e4m3_b16"]
    if st:
        out["roofline_stream"] = roof(st[0], {"bytes_per_elem": 2.8125})
    f6 = [r for r in kern if r["name"] == "4over6_e4m3_b16"]
    if f6:
        out["roofline_4over6"] = roof(f6[0], {"bytes_per_elem": 2.8125})
    if not args.no_cpu and not profiling:
        out["cpu_baseline"] = cpu_baseline(w2.x_np, passes, T, args.cpu_rows)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
