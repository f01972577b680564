"""Model-scale sweep: a synthetic 8B-class decoder (32 layers x {q, k, v, o, gate, up, down},
bf16, 0.02 * Student-t(df=4) with a per-layer, per-matrix seed) quantised with every recipe at
every block size, one layer resident on the GPU at a time.

    python -m paper_2605_08565_amd.sweep [--layers 32] [--out sweep.json]

Recipes: power-of-two MX (E8M0 abs-max), E4M3 abs-max, E4M3 prevent-zero, E4M3 4-over-6,
UE5M3 abs-max, E4M3 brute force; block sizes 2 ... 128.  For every (recipe, block size) the
seven matrices of a layer are quantised in one batched launch (mxq_quantize_batch; the search:
seven launches back to back), 436 MB of input between two touches of a matrix, so the 256 MB
Infinity Cache does not help, as one HIP graph replay with one event pair around it.
Reports GElem/s and the aggregate MSE per (recipe, block size).

Weights come from ``workloads.layer_matrix`` (numpy Philox, drawn on the host one layer ahead of
the GPU and uploaded): the same bytes the parity tests feed to the CPU oracle.  ``--generator
gpu`` draws them with torch's generator on the device instead (faster start-up, same
distribution, but bytes no test compares); the output says which generator produced the figures.
"""
from __future__ import annotations

import argparse
import json
import sys

from concurrent.futures import ThreadPoolExecutor

from .workloads import LAYER_SHAPES, N_LAYERS, layer_matrix

RECIPES = [("pow2_mx", 0, 0), ("e4m3_absmax", 1, 0), ("e4m3_prevent_zero", 1, 1),
           ("e4m3_4over6", 1, 2), ("ue5m3_absmax", 2, 0), ("e4m3_brute", 1, 4)]
BLOCKS = (2, 4, 8, 16, 32, 64, 128)


def host_layer(layer: int) -> dict:
    """The seven matrices of layer `layer` as bf16 bit patterns (numpy uint16), from
    ``workloads.layer_matrix``; the matrices are drawn by parallel threads."""
    names = list(LAYER_SHAPES)
    with ThreadPoolExecutor(max_workers=len(names)) as pool:
        return dict(zip(names, pool.map(lambda n: layer_matrix(layer, n), names)))


def upload_layer(host: dict, mats) -> None:
    """Copy a host layer into the seven resident weight buffers."""
    import torch
    for name, x in mats.items():
        x.view(torch.int16).copy_(torch.from_numpy(host[name].view("int16")))


def draw_layer(layer: int, mats) -> None:
    """Fill the seven resident weight buffers with layer `layer`, drawn on the GPU:
    0.02 * Z / sqrt(chi2_4 / 4)."""
    import torch
    for idx, (name, x) in enumerate(mats.items()):
        g = torch.Generator(device=x.device)
        g.manual_seed(50_000 + 16 * layer + idx)
        z = torch.randn(x.shape, generator=g, device=x.device, dtype=torch.float32)
        chi = torch.zeros(x.shape, device=x.device, dtype=torch.float32)
        for _ in range(4):
            chi += torch.randn(x.shape, generator=g, device=x.device, dtype=torch.float32) ** 2
        x.copy_(0.02 * z / torch.sqrt(chi / 4.0))


def run(layers: int = N_LAYERS, blocks=BLOCKS, recipes=RECIPES, use_graphs: bool = True,
        generator: str = "numpy", layer_ids=None, batched: bool = True, replays: int = 4) -> dict:
    """The smallest matrices (k, v: 4 M elements) quantise in a few microseconds, less than one
    launch through Python costs, so the seven launches of a (recipe, block size) group are
    captured once into a HIP graph over resident buffers and replayed for every layer."""
    import torch

    from . import mxq

    dev = torch.device("cuda:0")
    mats = {name: torch.empty((r, c), dtype=torch.bfloat16, device=dev) for name, (r, c) in LAYER_SHAPES.items()}
    outs = {name: (torch.empty(r * c // 2, dtype=torch.uint8, device=dev),
                   torch.empty(r * c // 2, dtype=torch.uint8, device=dev),
                   torch.empty(r * c // 2, dtype=torch.float32, device=dev))
            for name, (r, c) in LAYER_SHAPES.items()}

    def group(b, fmt, rec):
        views = []
        for name, x in mats.items():
            r, c = x.shape
            co, so, eo = outs[name]
            nb = r * c // b
            views.append((co.view(r, c // 2), so[:nb].view(r, c // b), eo[:nb].view(r, c // b)))
        if rec < mxq.RECIPE_BRUTE and batched:
            # the seven matrices share one launch: k and v hold less work than a launch costs
            mxq.quantize_batch(list(mats.values()), b, fmt, rec, outs=views)
        else:
            for x, (co, so, eo) in zip(mats.values(), views):
                mxq.quantize(x, b, fmt, rec, codes_out=co, scales_out=so, sse_out=eo)

    acc = {(rn, b): {"ms": 0.0, "elements": 0, "sse": 0.0} for rn, _, _ in recipes for b in blocks}
    warm = torch.zeros((8, 256), dtype=torch.bfloat16, device=dev)
    for _, fmt, rec in recipes:                      # untimed: the runtime loads each kernel on first use
        for b in blocks:
            mxq.quantize(warm, b, fmt, rec)
    torch.cuda.synchronize()
    graphs = {}
    if use_graphs:
        for m in mats.values():
            m.zero_()
        side = torch.cuda.Stream()
        for rn, fmt, rec in recipes:
            for b in blocks:
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=side):
                    group(b, fmt, rec)
                graphs[(rn, b)] = g
        torch.cuda.synchronize()

    ids = list(range(layers)) if layer_ids is None else list(layer_ids)
    ahead = ThreadPoolExecutor(max_workers=1)            # the next layer is drawn while this one runs
    pending = ahead.submit(host_layer, ids[0]) if (generator == "numpy" and ids) else None
    for pos, layer in enumerate(ids):
        if generator == "numpy":
            host = pending.result()
            pending = ahead.submit(host_layer, ids[pos + 1]) if pos + 1 < len(ids) else None
            upload_layer(host, mats)
            del host
        else:
            draw_layer(layer, mats)
        torch.cuda.synchronize()
        for rn, fmt, rec in recipes:
            for b in blocks:
                # several replays between one event pair: the latency of submitting a graph (several
                # microseconds, as long as a small matrix takes) is paid once, not per layer pass;
                # a layer's input is 436 MB, so a replay still finds nothing in the Infinity Cache
                reps = 1 if rec >= mxq.RECIPE_BRUTE else replays
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for _ in range(reps):
                    if use_graphs:
                        graphs[(rn, b)].replay()
                    else:
                        group(b, fmt, rec)
                e1.record()
                torch.cuda.synchronize()
                a = acc[(rn, b)]
                a["ms"] += e0.elapsed_time(e1) / reps
                for name, x in mats.items():
                    a["elements"] += x.numel()
                    a["sse"] += float(outs[name][2][: x.numel() // b].to(torch.float64).sum())
    rows = []
    for (rn, b), a in acc.items():
        rows.append({"recipe": rn, "block": b, "gelem_s": round(a["elements"] / a["ms"] / 1e6, 1),
                     "mse": a["sse"] / a["elements"], "elements": a["elements"], "ms": round(a["ms"], 3)})
    ahead.shutdown()
    return {"layers": len(ids), "layer_ids": ids, "graphs": use_graphs, "generator": generator, "batched": batched,
            "parity_checked_bytes": generator == "numpy", "rows": rows}


def main() -> None:
    ap = argparse.ArgumentParser()
    ap.add_argument("--layers", type=int, default=N_LAYERS)
    ap.add_argument("--out", default="")
    ap.add_argument("--no-graphs", action="store_true", help="launch every kernel from Python instead")
    ap.add_argument("--unbatched", action="store_true", help="one launch per matrix instead of one per layer")
    ap.add_argument("--generator", choices=("numpy", "gpu"), default="numpy",
                    help="numpy: workloads.layer_matrix bytes (the parity-checked ones); gpu: torch draws on the device")
    args = ap.parse_args()
    res = run(args.layers, use_graphs=not args.no_graphs, generator=args.generator, batched=not args.unbatched)
    text = json.dumps(res)
    if args.out:
        with open(args.out, "w") as f:
            f.write(text)
    for r in res["rows"]:
        print(f"{r['recipe']:18s} b={r['block']:<4d} {r['gelem_s']:9.1f} GElem/s   mse {r['mse']:.4e}")
    if not args.out:
        sys.stdout.write(text + "\n")


if __name__ == "__main__":
    main()
