#!/usr/bin/env python3
"""Benchmark of the SDGP backward-data path on one MI355X.

Workload of the headline (the largest named configuration that fits one GPU): the whole backward-data pass of a
ResNet-50 at batch 256 and 224 x 224 -- its 53 convolutions and the 2048 -> 1000 classifier, NHWC bf16, every layer's
dL/dO Laplace distributed with a layer-dependent scale 10^-U(3,5) and 20-50 % exact zeros, He-normal weights, 2:4
pruning with the random ranker seeded by the layer index (Sec. IV; Alg. 1).  One "step" is one pass of the hot path
over that batch: 54 calls (rank + prune + backward-data product), last layer first.  All inputs are drawn on the
host by the seeded generators the parity tests use and are resident in HBM before the timed region.

Prints ONE JSON line.  `value` is the effective rate: the FLOPs of the unpruned products divided by the time the
pruned path took.  Extra fields: per distinct ResNet-50 layer shape the dense and the fused times, the ResNet-9 sweep
(speedup at 2:4, 2:8, 2:16), the ResNet-50 bottleneck layers, the standalone prune pass's GB/s, roofline objects and
the CPU oracle timed on a bounded sample.

`--probe` launches a few calls of one kind plus a plain device copy of known size and exits: meant to run under
rocprofv3 (kernel trace, or one --pmc counter per run; the copy calibrates FETCH_SIZE / WRITE_SIZE).  `--summarize`
prints per-kernel averages of a counter_collection.csv.
"""
from __future__ import annotations

import argparse
import collections
import concurrent.futures
import csv
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0
BALANCE_FLOP_PER_BYTE = MFMA_BF16_PEAK_TFLOPS * 1e12 / (HBM_PEAK_GBS * 1e9)   # 312.5
COPY_BYTES = 256 << 20
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "traffic_per_launch.md")
PAPER_CONTEXT = ("the paper reports no measured rate for this path; it estimates a 15-25 % cut of total training time "
                 "assuming 2:4 sparse tensor-core support on an A100 (abstract, Sec. IV-C)")
RANKER_NAMES = ("random", "greedy", "greedy-adjusted")


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--batch", type=int, default=256, help="batch of the ResNet-50 pass (256 is the named configuration)")
    ap.add_argument("--cpu-batch", type=int, default=6, help="batch of the CPU-oracle sample (0 skips it)")
    ap.add_argument("--no-extras", action="store_true", help="only the timed steps and the roofline: no sub-tables, no CPU leg")
    ap.add_argument("--probe", choices=("layer", "prune", "channel", "pass"), default=None)
    ap.add_argument("--workload", choices=("r9", "r50", "r50all"), default="r9", help="--probe layer: which layer list")
    ap.add_argument("--layer", type=int, default=3, help="--probe layer: index into the list")
    ap.add_argument("--n", type=int, default=2)
    ap.add_argument("--m", type=int, default=4)
    ap.add_argument("--ranker", type=int, default=1, help="0 random, 1 greedy, 2 greedy-adjusted")
    ap.add_argument("--reps", type=int, default=3)
    ap.add_argument("--summarize", default=None, metavar="CSV")
    return ap.parse_args()


# ------------------------------------------------------------------------------------------------------ small helpers

def summarize(path):
    rows = list(csv.DictReader(open(path)))
    agg = collections.defaultdict(lambda: [0.0, set()])
    for r in rows:
        key = (r["Kernel_Name"][:70], r["Counter_Name"])
        agg[key][0] += float(r["Counter_Value"])
        agg[key][1].add(r["Dispatch_Id"])
    for (k, c), (v, ids) in sorted(agg.items()):
        print(f"{c:12s} {v / len(ids):14.1f} per dispatch ({len(ids)} dispatches)  {k}")


def traffic_from_profiles(layer_name, setting):
    """HBM bytes per launch as measured with rocprofv3 counters and written down in profiles/traffic_per_launch.md
    (table rows `| layer | setting | ... | bytes |`); None when that file has no row for this call.  The figure is
    not measured by this run."""
    try:
        for line in open(TRAFFIC_FILE):
            cells = [c.strip() for c in line.strip().strip("|").split("|")]
            if len(cells) >= 3 and cells[0] == layer_name and cells[1] == setting:
                m = re.fullmatch(r"([0-9.]+(?:e[0-9]+)?)", cells[-1])
                if m:
                    return float(m.group(1))
    except OSError:
        pass
    return None


def layer_list(workload, batch=None):
    from paper_2202_00774_amd import workloads as wl
    if workload == "r9":
        return wl.resnet9_layers(batch or 512), [(1e-3, 0.3, 2000 + i) for i in range(6)]
    if workload == "r50":
        return wl.resnet50_bottleneck_layers(batch or 128), [(1e-4, 0.4, 3000 + i) for i in range(6)]
    layers = wl.resnet50_all_layers(batch or 256)
    return layers, [wl.resnet50_layer_stats(i) + (5000 + i,) for i in range(len(layers))]


def host_inputs(layers, stats, workers=12):
    """(dO, W) of every layer from the seeded host generators, drawn by a pool of threads."""
    from paper_2202_00774_amd import workloads as wl
    with concurrent.futures.ThreadPoolExecutor(workers) as pool:
        jobs = [pool.submit(wl.layer_inputs, L, s[0], s[1], s[2], wl.BF16) for L, s in zip(layers, stats)]
        return [j.result() for j in jobs]


# -------------------------------------------------------------------------------------------------------------- main

def main():
    args = parse()
    if args.summarize:
        summarize(args.summarize)
        return
    if args.gpus != 1:
        print("bench.py measures one GPU: this build contains no multi-GPU path (every box here has one GPU); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2202_00774_amd as sdgp
    from paper_2202_00774_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    lib = sdgp.binding.load()  # fails loudly when the HIP library is missing
    dev = torch.device("cuda:0")
    rankers = tuple(zip(RANKER_NAMES, (sdgp.RANDOM, sdgp.GREEDY, sdgp.GREEDY_ADJUSTED)))

    def gpu(a):
        return torch.from_numpy(a.view(np.int16)).to(dev).view(torch.bfloat16)

    def resident(layers, stats):
        out = []
        for L, (dO, W) in zip(layers, host_inputs(layers, stats)):
            out.append((L, gpu(dO), gpu(W), torch.empty(L.dD_shape, dtype=torch.bfloat16, device=dev)))
        return out

    scratch = {"buf": torch.empty(64 << 20, dtype=torch.uint8, device=dev)}   # the calls' workspace, grown on demand

    def call(L, dO, W, out, n, m, rk, seed=0):
        need = sdgp.conv_bwd_data_workspace(L.B, L.H, L.Wd, L.C_in, L.C_out, L.R, L.S, L.stride, L.pad, sdgp.BF16, n, m)
        if need > scratch["buf"].numel():
            scratch["buf"] = torch.empty(need, dtype=torch.uint8, device=dev)   # (warm-up calls come first)
        sdgp.sdgp_conv_bwd_data(dO, W, L.H, L.Wd, L.stride, L.pad, n, m, rk, seed, out=out, workspace=scratch["buf"])

    def time_call(fn, reps=10, warm=2):
        """Average duration in ms, HIP events on the stream the kernels are launched on (torch's current stream)."""
        for _ in range(warm):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    if args.probe:
        probe(args, sdgp, wl, torch, np, dev, gpu, call)
        return

    # ------------------------------------------------------------------ headline: the whole ResNet-50 pass at 2:4 random
    r50, r50_stats = layer_list("r50all", args.batch)
    data50 = resident(r50, r50_stats)
    total_flops = sum(L.dense_flops for L in r50)

    def step(n=2, m=4):
        for i in range(len(data50) - 1, -1, -1):
            call(*data50[i], n, m, sdgp.RANDOM, seed=i)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed * 1e3 / args.steps

    result = {
        "metric": "bwd-data effective TFLOP/s + speedup vs dense at 2:4/2:8; prune-pass GB/s",
        "value": round(total_flops / (elapsed / args.steps) / 1e12, 2),
        "unit": "TFLOP/s (effective: dense-equivalent FLOPs / pruned-path time)",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "full ResNet-50 backward-data pass: 53 convolutions + fc, batch %d, 224x224, NHWC bf16, 2:4, "
                               "random ranker seeded per layer (54 sdgp_conv_bwd_data calls per step: one fused kernel each, except that layers "
                               "whose gradient the fused kernel would rank several times over rank and compress it in a pass of their "
                               "own first, and the classifier layer copies gradient and filter into the workspace with its 1000 "
                               "channels padded to 1024)" % args.batch,
                   "n": 2, "m": 4, "batch": args.batch, "ranker": "random"},
        "paper_context": PAPER_CONTEXT,
    }

    # ---- per distinct layer shape: dense, fused 2:4 and 2:8 (random), summed over the 54 layers
    shapes = {}
    for i, (L, dO, W, out) in enumerate(data50):
        key = (L.H, L.Wd, L.C_in, L.C_out, L.R, L.S, L.stride, L.pad)
        if key not in shapes:
            shapes[key] = {"layer": L, "count": 0,
                           "t": {name: time_call(lambda: call(L, dO, W, out, n, m, sdgp.RANDOM, seed=i), reps=5, warm=1)
                                 for name, n, m in (("dense", 4, 4), ("2:4", 2, 4), ("2:8", 2, 8))}}
        shapes[key]["count"] += 1
    tot = {name: sum(s["count"] * s["t"][name] for s in shapes.values()) for name in ("dense", "2:4", "2:8")}

    # ---- roofline of the dominant call of the step: the layer shape whose fused launches take the largest share
    dom = max(shapes.values(), key=lambda s: s["count"] * s["t"]["2:4"])
    result["roofline"] = roofline_entry(dom["layer"], dom["t"]["2:4"], "2:4 random", sparse=True,
                                        share=dom["count"] * dom["t"]["2:4"] / tot["2:4"], launches=dom["count"])
    result["roofline_dense"] = roofline_entry(dom["layer"], dom["t"]["dense"], "dense", sparse=False)

    if args.no_extras:
        print(json.dumps(result))
        return

    # ---- what this GPU sustains with plain kernels (the published peaks are what `frac` divides by; these say how much
    # of them any kernel can reach here)
    nbig = 1 << 29
    pa = torch.empty(nbig, dtype=torch.uint8, device=dev).random_(0, 255)
    pb = torch.empty(nbig, dtype=torch.uint8, device=dev)
    sink = torch.zeros(16384, dtype=torch.uint8, device=dev)
    t_copy = time_call(lambda: sdgp.sdgp_peak_probe(0, pa, pb, nbig), reps=10, warm=2)
    t_read = time_call(lambda: sdgp.sdgp_peak_probe(1, pa, sink, nbig), reps=10, warm=2)
    iters = 20000
    t_dense = time_call(lambda: sdgp.sdgp_peak_probe(2, None, sink, iters=iters), reps=3, warm=1)
    t_sparse = time_call(lambda: sdgp.sdgp_peak_probe(3, None, sink, iters=iters), reps=3, warm=1)
    w_dense = sdgp.sdgp_peak_probe(2, None, sink, iters=1) * iters
    w_sparse = sdgp.sdgp_peak_probe(3, None, sink, iters=1) * iters
    del pa, pb
    peaks = {"hbm_copy_GBs": round(2.0 * nbig / (t_copy * 1e-3) / 1e9, 1), "hbm_read_GBs": round(nbig / (t_read * 1e-3) / 1e9, 1),
             "mfma_bf16_dense_TFLOPs": round(w_dense / (t_dense * 1e-3) / 1e12, 1),
             "smfmac_bf16_dense_equivalent_TFLOPs": round(w_sparse / (t_sparse * 1e-3) / 1e12, 1),
             "note": "sdgp_peak_probe: a 512 MB streaming copy (read + write counted) and read, and register-only loops of "
                     "v_mfma_f32_32x32x16_bf16 / v_smfmac_f32_32x32x32_bf16 (two wavefronts per SIMD, eight independent "
                     "accumulator tiles); the sparse figure counts 2*32*32*32 operations per instruction"}
    result["achievable_peaks"] = peaks
    for key in ("roofline", "roofline_dense"):
        e = result[key]
        e["frac_of_measured_peak"] = round(e["achieved"] / (peaks["mfma_bf16_dense_TFLOPs"] if e["bound"] == "mfma"
                                                            else peaks["hbm_copy_GBs"]), 4)

    result["resnet50_whole"] = {
        "layers": len(r50), "distinct_shapes": len(shapes), "gflop_dense": round(total_flops / 1e9, 1),
        **{"%s_ms" % k: round(v, 3) for k, v in tot.items()},
        "speedup_2:4": round(tot["dense"] / tot["2:4"], 3), "speedup_2:8": round(tot["dense"] / tot["2:8"], 3),
        "effective_tflops_2:4": round(total_flops / tot["2:4"] / 1e9, 1),
        "ideal_ms": round(sum(max(L.bytes_moved() / (HBM_PEAK_GBS * 1e9), L.dense_flops / (MFMA_BF16_PEAK_TFLOPS * 1e12))
                              for L in r50) * 1e3, 3),
        "per_shape": [{"layer": s["layer"].name, "count": s["count"], "gflop_dense": round(s["layer"].dense_flops / 1e9, 2),
                       **{"%s_us" % k: round(v * 1e3, 1) for k, v in s["t"].items()},
                       "hbm_floor_us": round(s["layer"].bytes_moved() / (HBM_PEAK_GBS * 1e9) * 1e6, 1)}
                      for s in shapes.values()],
        "note": "sums of per-layer launch times (HIP events), random ranker seeded with the layer index; ideal = sum over "
                "layers of max(bytes / HBM peak, dense FLOPs / bf16 MFMA peak); per_shape names the first layer of a shape",
    }
    # ---- ranking ahead of the product (one pass writes kept values + positions, the product reads them and ranks
    # nothing) against the fused kernel (the entry point without a workspace runs it: these arrays do not fit its
    # scratch) and the dense kernel, on the ResNet-50 layers where the library takes the pass: strided 3x3 filters
    # and 1x1 filters onto many input channels
    rows = []
    for name in ("l2b0_3x3", "l3b0_3x3", "l4b0_3x3", "l2b1_1x1a", "l3b1_1x1a", "l4b1_1x1a", "l4b0_1x1b"):
        L, dO, W, out = next(d for d in data50 if d[0].name == name)
        row = {"layer": name, "dense_us": round(time_call(lambda: call(L, dO, W, out, 4, 4, sdgp.GREEDY), reps=5) * 1e3, 1)}
        for rname, rk in (("random", sdgp.RANDOM), ("greedy", sdgp.GREEDY)):
            t_a = time_call(lambda: call(L, dO, W, out, 2, 4, rk), reps=5)
            t_f = time_call(lambda: sdgp.sdgp_conv_bwd_data_noalloc(dO, W, L.H, L.Wd, L.stride, L.pad, 2, 4, rk, 0, out=out), reps=5)
            row["2:4_%s_fused_us" % rname] = round(t_f * 1e3, 1)
            row["2:4_%s_ranked_ahead_us" % rname] = round(t_a * 1e3, 1)
        row["speedup_vs_dense_random"] = round(row["dense_us"] / row["2:4_random_ranked_ahead_us"], 3)
        rows.append(row)
    result["ranked_ahead_vs_fused"] = {
        "layers": rows,
        "note": "ranked_ahead = what sdgp_conv_bwd_data runs on these layers given its workspace (for the Magnitude ranker "
                "only where the fused kernel would rank four times or more: otherwise both columns are the fused kernel); "
                "the product kernel alone runs 1.15-1.25x as fast as the dense one (profiles/ranked_ahead_kernel_stats.md)",
    }

    # ---- the 1x1 stride-1 layers are plain GEMMs dD[rows, C_in] = dO[rows, C_out] . W[C_out, C_in]: PyTorch's library GEMM
    # (hipBLASLt) on the same tensors beside this library's dense and fused kernels
    rows = []
    seen = set()
    for L, dO, W, out in data50:
        key = (L.H, L.C_in, L.C_out)
        if L.R != 1 or L.S != 1 or L.stride != 1 or key in seen:
            continue
        seen.add(key)
        a2, w2, o2 = dO.view(-1, L.C_out), W.view(L.C_out, L.C_in), out.view(-1, L.C_in)
        t_lib = time_call(lambda: torch.matmul(a2, w2, out=o2), reps=5, warm=2)
        t_dense = time_call(lambda: call(L, dO, W, out, 4, 4, sdgp.GREEDY), reps=5, warm=1)
        t_fused = time_call(lambda: call(L, dO, W, out, 2, 4, sdgp.RANDOM), reps=5, warm=1)
        rows.append({"layer": L.name, "rows": L.B * L.H * L.Wd, "C_out": L.C_out, "C_in": L.C_in,
                     "library_gemm_us": round(t_lib * 1e3, 1), "dense_us": round(t_dense * 1e3, 1),
                     "2:4_random_us": round(t_fused * 1e3, 1), "dense_vs_library": round(t_lib / t_dense, 2)})
    result["pointwise_vs_library_gemm"] = {
        "layers": rows,
        "note": "library_gemm = torch.matmul(dO[rows, C_out], W[C_out, C_in]) in bf16 on the same tensors (no pruning); "
                "dense_vs_library > 1: this library's dense kernel is the faster one"}
    del data50, shapes

    # ------------------------------------------------------------------ ResNet-9 sweep, batch 512, the three rankers
    r9, r9_stats = layer_list("r9")
    data = resident(r9, r9_stats)
    table = []
    for L, dO, W, out in data:
        t_fused = {name: time_call(lambda rk=rk: call(L, dO, W, out, 2, 4, rk)) for name, rk in rankers}
        t_dense = time_call(lambda: call(L, dO, W, out, 4, 4, sdgp.GREEDY))
        t28 = time_call(lambda: call(L, dO, W, out, 2, 8, sdgp.GREEDY))
        t216 = time_call(lambda: call(L, dO, W, out, 2, 16, sdgp.GREEDY))
        row = {"layer": L.name, "gflop_dense": round(L.dense_flops / 1e9, 2), "dense_us": round(t_dense * 1e3, 1),
               "dense_tflops": round(L.dense_flops / t_dense / 1e9, 1)}
        for name in t_fused:
            row["fused_2:4_%s_us" % name] = round(t_fused[name] * 1e3, 1)
        row["speedup_2:4"] = round(t_dense / t_fused["greedy"], 3)
        row["speedup_2:8"] = round(t_dense / t28, 3)
        row["speedup_2:16"] = round(t_dense / t216, 3)
        row["effective_tflops_2:4"] = round(L.dense_flops / t_fused["greedy"] / 1e9, 1)
        row["hbm_floor_us"] = round(L.bytes_moved() / (HBM_PEAK_GBS * 1e9) * 1e6, 1)
        table.append(row)
    result["resnet9_batch512"] = {
        "layers": table,
        "sweep_ms_2:4_three_rankers": round(sum(sum(r["fused_2:4_%s_us" % n] for n in RANKER_NAMES) for r in table) / 1e3, 4),
        "sweep_effective_tflops": round(3 * sum(L.dense_flops for L in r9) /
                                        sum(sum(r["fused_2:4_%s_us" % n] for n in RANKER_NAMES) for r in table) / 1e6, 1),
    }
    # the slowest single call of the sweep, whatever its ranker, and the dense kernel on the same layer
    worst = max(((r, n) for r in table for n in RANKER_NAMES), key=lambda p: p[0]["fused_2:4_%s_us" % p[1]])
    Lw = next(L for L in r9 if L.name == worst[0]["layer"])
    result["roofline_resnet9"] = roofline_entry(Lw, worst[0]["fused_2:4_%s_us" % worst[1]] / 1e3, "2:4 " + worst[1], sparse=True)
    result["roofline_resnet9_dense"] = roofline_entry(Lw, worst[0]["dense_us"] / 1e3, "dense", sparse=False)

    # general n of m (the accuracy study's settings, Sec. IV-B: Rescaled Magnitude): pruned rows stored dense with zeros
    Lg, dOg, Wg, outg = data[3]
    tg = {"dense": time_call(lambda: call(Lg, dOg, Wg, outg, 4, 4, sdgp.GREEDY))}
    for n_, m_ in ((2, 4), (4, 8), (2, 8), (8, 16), (4, 16), (2, 16), (16, 32), (8, 32), (4, 32)):
        tg["%d:%d" % (n_, m_)] = time_call(lambda: call(Lg, dOg, Wg, outg, n_, m_, sdgp.GREEDY_ADJUSTED))
    result["general_nm_greedy_adjusted"] = {"layer": Lg.name, **{k + "_us": round(v * 1e3, 1) for k, v in tg.items()}}

    # ------------------------------------------------------------------ ResNet-50 bottleneck layers, batch 128
    b50, b50_stats = layer_list("r50")
    table = []
    for L, dO, W, out in resident(b50, b50_stats):
        t = {}
        for name, n, m, rk in (("dense", 4, 4, sdgp.GREEDY), ("2:4_greedy", 2, 4, sdgp.GREEDY),
                               ("2:4_greedy-adjusted", 2, 4, sdgp.GREEDY_ADJUSTED), ("2:8_greedy", 2, 8, sdgp.GREEDY),
                               ("2:16_greedy", 2, 16, sdgp.GREEDY)):
            t[name] = time_call(lambda: call(L, dO, W, out, n, m, rk))
        row = {"layer": L.name, "gflop_dense": round(L.dense_flops / 1e9, 2)}
        row.update({k + "_us": round(v * 1e3, 1) for k, v in t.items()})
        row["speedup_2:4"] = round(t["dense"] / t["2:4_greedy"], 3)
        row["hbm_floor_us"] = round(L.bytes_moved() / (HBM_PEAK_GBS * 1e9) * 1e6, 1)
        row["frac_of_hbm_peak_dense"] = round(L.bytes_moved() / (t["dense"] * 1e-3) / 1e9 / HBM_PEAK_GBS, 3)
        table.append(row)
    result["resnet50_bottleneck_batch128"] = table

    # ---- the compacted-gradient path (K' = (n/m) C_out kept values per pixel, W rows gathered by index, fp32 FMAs) against
    # the fused path (structured-sparse instruction up to m = 16, masked dense instruction at m = 32) and the dense
    # kernel: two HBM-bound pointwise layers and one compute-bound 3x3 layer, Magnitude ranker (Sec. IV-C: ratios 4, 8, 16)
    rows = []
    picks = [(b50[0], b50_stats[0]), (b50[2], b50_stats[2]), (r9[3], r9_stats[3])]
    for (L, dO, W, out) in resident([p[0] for p in picks], [p[1] for p in picks]):
        row = {"layer": L.name, "dense_us": round(time_call(lambda: call(L, dO, W, out, 4, 4, sdgp.GREEDY)) * 1e3, 1)}
        for n_, m_ in ((2, 4), (2, 8), (2, 16), (4, 32), (2, 32)):
            need = int(lib.sdgp_conv_bwd_data_compact_workspace(L.B, L.H, L.Wd, L.C_in, L.C_out, L.R, L.S, L.stride, L.pad,
                                                                sdgp.BF16, n_, m_))
            ws_c = torch.empty(max(need, 16), dtype=torch.uint8, device=dev)
            t_f = time_call(lambda: call(L, dO, W, out, n_, m_, sdgp.GREEDY), reps=5)
            t_c = time_call(lambda: sdgp.sdgp_conv_bwd_data_compact(dO, W, L.H, L.Wd, L.stride, L.pad, n_, m_, sdgp.GREEDY, 0,
                                                                    out=out, workspace=ws_c), reps=3, warm=1)
            row["%d:%d_fused_us" % (n_, m_)] = round(t_f * 1e3, 1)
            row["%d:%d_compact_us" % (n_, m_)] = round(t_c * 1e3, 1)
            del ws_c
        rows.append(row)
    wins = [(r["layer"], k[:-11]) for r in rows for k in r if k.endswith("_compact_us") and r[k] < r[k[:-11] + "_fused_us"]]
    result["compact_vs_fused"] = {
        "layers": rows, "compact_faster_at": wins,
        "note": "compact = prune pass to (values, positions) + one AXPY per kept value on the vector ALUs; fused = the "
                "matrix-core path of sdgp_conv_bwd_data; compact_faster_at lists the (layer, n:m) where the compacted path "
                "wins -- the measured crossover of the sparsity grid",
    }

    # ---- grouped 3x3 layers of RegNetX-400MF (Sec. IV; group width 16, widths 32/64/160/384, batch 256): the stride-2
    # layer that opens each stage and the stride-1 layer of its other blocks
    rows = []
    for C, H, stride in ((32, 112, 2), (64, 56, 2), (64, 28, 1), (160, 28, 2), (160, 14, 1), (384, 14, 2), (384, 7, 1)):
        P = (H + 2 - 3) // stride + 1
        gd = (torch.randn((args.batch, P, P, C), device=dev) * 1e-3).to(torch.bfloat16)
        gw = (torch.randn((C, 3, 3, 16), device=dev) * 0.05).to(torch.bfloat16)
        go = torch.empty((args.batch, H, H, C), dtype=torch.bfloat16, device=dev)
        need = int(lib.sdgp_conv_bwd_data_grouped_workspace(args.batch, H, H, C, C, 3, 3, stride, 1, C // 16, sdgp.BF16, 2, 4))
        gws = torch.empty(max(need, 16), dtype=torch.uint8, device=dev)
        row = {"channels": C, "input": H, "stride": stride, "groups": C // 16,
               "hbm_floor_us": round((gd.numel() + go.numel()) * 2 / (HBM_PEAK_GBS * 1e9) * 1e6, 1)}
        for name, n_, rk in (("dense", 4, sdgp.GREEDY), ("2:4_random", 2, sdgp.RANDOM), ("2:4_greedy-adjusted", 2, sdgp.GREEDY_ADJUSTED)):
            row[name + "_us"] = round(time_call(lambda: sdgp.sdgp_conv_bwd_data_grouped(gd, gw, H, H, stride, 1, C // 16, n_, 4, rk, 0,
                                                                                        out=go, workspace=gws)) * 1e3, 1)
        rows.append(row)
        del gd, gw, go, gws
    result["regnetx400mf_grouped_3x3"] = {
        "layers": rows,
        "note": "sdgp_conv_bwd_data_grouped: a small kernel that re-indexes the filter, then one fused kernel "
                "(v_mfma_f32_16x16x32_bf16, a group's 16 input channels as the rows); times include both launches",
    }

    # ------------------------------------------------------------------ prune pass: tensors beyond the last-level cache
    import ctypes
    nelem = 256 * 112 * 112 * 64
    srcs = [gpu(wl.laplace_with_zeros((nelem // 64, 64), 1e-3, 0.3, seed=9000 + i, dtype=wl.BF16)) for i in range(2)]
    dsts = [torch.empty_like(s) for s in srcs]
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    k = [0]

    def prune_call(n_, m_, rk, dense_out=True, vals=None, idx=None):
        def f():
            s, d = srcs[k[0] % 2], dsts[k[0] % 2]
            k[0] += 1
            rc = lib.sdgp_prune(ctypes.c_void_p(s.data_ptr()), s.shape[0], s.shape[1], sdgp.BF16, n_, m_, rk, 0,
                                ctypes.c_void_p(d.data_ptr()) if dense_out else None,
                                ctypes.c_void_p(vals.data_ptr()) if vals is not None else None,
                                ctypes.c_void_p(idx.data_ptr()) if idx is not None else None, stream)
            assert rc == 0
        return f

    def rate(ms, bytes_per_elem):
        return {"us": round(ms * 1e3, 1), "GB/s": round(bytes_per_elem * nelem / (ms * 1e-3) / 1e9, 1),
                "frac_of_hbm_peak": round(bytes_per_elem * nelem / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}

    prune = {name: rate(time_call(prune_call(2, 4, rk), reps=20, warm=3), 4.0) for name, rk in rankers}
    for n_, m_ in ((2, 8), (2, 16), (4, 16), (8, 16), (2, 32), (4, 32), (8, 32), (16, 32)):
        prune["greedy_%d:%d" % (n_, m_)] = rate(time_call(prune_call(n_, m_, sdgp.GREEDY), reps=10, warm=2), 4.0)
    for n_, m_ in ((4, 16), (4, 32), (16, 32)):
        prune["random_%d:%d" % (n_, m_)] = rate(time_call(prune_call(n_, m_, sdgp.RANDOM), reps=10, warm=2), 4.0)
    vals = torch.empty(nelem // 2, dtype=torch.bfloat16, device=dev)
    idx = torch.empty(nelem // 2, dtype=torch.uint8, device=dev)
    # compact output (values + uint8 positions, no dense-shaped copy): 2 + 3 n/m bytes per element
    prune["greedy_compact_output"] = rate(time_call(prune_call(2, 4, sdgp.GREEDY, False, vals, idx), reps=20, warm=3), 3.5)
    del vals, idx
    result["prune_pass"] = {"tensor": "[%d, 64] bf16 (411 MB), 2:4 unless named, dense-shaped output (4 B per element) unless "
                                      "named" % (nelem // 64), **prune}
    slowest = max(RANKER_NAMES, key=lambda n: prune[n]["us"])
    result["roofline_prune"] = {"bound": "hbm", "kernel": "prune_items (2:4 %s: the slowest ranker)" % slowest,
                                "achieved": prune[slowest]["GB/s"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                "frac": prune[slowest]["frac_of_hbm_peak"],
                                "traffic": traffic_from_profiles("prune_411MB", "2:4 " + slowest),
                                "traffic_source": "profiles/traffic_per_launch.md (counters of an earlier run, not this one)",
                                "algorithmic_bytes": 4.0 * nelem}

    # ---- Rescaled Magnitude with one factor per channel (second reading of Sec. III-B): the sweep that makes the
    # factors (2 bytes per element read), the prune pass with them (4), on the same 411 MB tensors; and the fused
    # call (factors, filter rows times factors, Magnitude product) on the ResNet-9 layers against the per-group one
    ws = torch.empty(int(lib.sdgp_channel_scales_workspace(nelem // 64, 64, sdgp.BF16, 2, 4)), dtype=torch.uint8, device=dev)
    factors = torch.empty(64, dtype=torch.float32, device=dev)

    def sums():
        s = srcs[k[0] % 2]
        k[0] += 1
        rc = lib.sdgp_channel_scales(ctypes.c_void_p(s.data_ptr()), s.shape[0], s.shape[1], sdgp.BF16, 2, 4,
                                     ctypes.c_void_p(factors.data_ptr()), None, ctypes.c_void_p(ws.data_ptr()), ws.numel(), stream)
        assert rc == 0

    def prune_scaled():
        s, d = srcs[k[0] % 2], dsts[k[0] % 2]
        k[0] += 1
        rc = lib.sdgp_prune_channel_rescaled(ctypes.c_void_p(s.data_ptr()), s.shape[0], s.shape[1], sdgp.BF16, 2, 4,
                                             ctypes.c_void_p(factors.data_ptr()), ctypes.c_void_p(d.data_ptr()), stream)
        assert rc == 0
    per_channel = {"channel_scales": rate(time_call(sums, reps=20, warm=3), 2.0),
                   "prune_channel_rescaled": rate(time_call(prune_scaled, reps=20, warm=3), 4.0), "fused_layers": []}
    for L, dO, W, out in data:
        need = int(lib.sdgp_conv_bwd_data_channel_rescaled_workspace(L.B, L.H, L.Wd, L.C_in, L.C_out, L.R, L.S, L.stride,
                                                                     L.pad, sdgp.BF16, 2, 4))
        wsl = torch.empty(need, dtype=torch.uint8, device=dev)
        t_pc = time_call(lambda: sdgp.sdgp_conv_bwd_data_channel_rescaled(dO, W, L.H, L.Wd, L.stride, L.pad, 2, 4, out=out,
                                                                          workspace=wsl))
        t_pg = time_call(lambda: call(L, dO, W, out, 2, 4, sdgp.GREEDY_ADJUSTED))
        per_channel["fused_layers"].append({"layer": L.name, "per_channel_us": round(t_pc * 1e3, 1),
                                            "per_group_us": round(t_pg * 1e3, 1)})
        del wsl
    result["rescaled_per_channel"] = per_channel
    del srcs, dsts, ws

    # ---- where backward-data sits in a training step (Sec. IV-C, Fig. 9: forward, weight gradient and data gradient
    # take about a third each on the paper's hardware): the three passes of the six layers on this library's kernels
    # (forward and weight gradient prune nothing; the weight gradient reads the unpruned dO), with PyTorch's library
    # kernels on the same tensors beside them as context
    split = []
    for i, (L, dO, W, out) in enumerate(data):
        x = gpu(wl.normal(L.dD_shape, 1.0, 7000 + i, wl.BF16))
        y = torch.empty(L.dO_shape, dtype=torch.bfloat16, device=dev)
        dW = torch.empty(L.W_shape, dtype=torch.float32, device=dev)
        geom = (L.B, L.H, L.Wd, L.C_in, L.C_out, L.R, L.S, L.stride, L.pad, sdgp.BF16)
        ws_f = torch.empty(max(int(lib.sdgp_conv_fwd_workspace(*geom)), 16), dtype=torch.uint8, device=dev)
        ws_w = torch.empty(max(int(lib.sdgp_conv_bwd_weight_workspace(*geom)), 16), dtype=torch.uint8, device=dev)
        t_f = time_call(lambda: sdgp.sdgp_conv_fwd(x, W, L.stride, L.pad, out=y, workspace=ws_f))
        t_w = time_call(lambda: sdgp.sdgp_conv_bwd_weight(x, dO, L.R, L.S, L.stride, L.pad, out=dW, workspace=ws_w))
        t_d = time_call(lambda: call(L, dO, W, out, 4, 4, sdgp.GREEDY))
        t_s = time_call(lambda: call(L, dO, W, out, 2, 4, sdgp.GREEDY))
        row = {"layer": L.name, "forward_us": round(t_f * 1e3, 1), "weight_grad_us": round(t_w * 1e3, 1),
               "data_grad_dense_us": round(t_d * 1e3, 1), "data_grad_2:4_us": round(t_s * 1e3, 1)}
        try:   # the library convolution is context, not the product
            xt, wt, gy = x.permute(0, 3, 1, 2), W.permute(0, 3, 1, 2), dO.permute(0, 3, 1, 2)   # NHWC memory
            row["library_forward_us"] = round(time_call(lambda: torch.nn.functional.conv2d(xt, wt, None, L.stride, L.pad), reps=5) * 1e3, 1)
            row["library_weight_grad_us"] = round(time_call(lambda: torch.nn.grad.conv2d_weight(xt, wt.shape, gy, L.stride, L.pad), reps=5) * 1e3, 1)
            row["library_data_grad_us"] = round(time_call(lambda: torch.nn.grad.conv2d_input(xt.shape, wt, gy, L.stride, L.pad), reps=5) * 1e3, 1)
        except Exception as e:
            row["library_error"] = repr(e)[:120]
        split.append(row)
        del x, y, dW, ws_f, ws_w
    tf, tw = sum(r["forward_us"] for r in split), sum(r["weight_grad_us"] for r in split)
    td, ts = sum(r["data_grad_dense_us"] for r in split), sum(r["data_grad_2:4_us"] for r in split)
    result["training_step_split"] = {
        "layers": split, "forward_us": round(tf, 1), "weight_grad_us": round(tw, 1), "data_grad_dense_us": round(td, 1),
        "data_grad_2:4_us": round(ts, 1), "data_grad_share_dense": round(td / (tf + tw + td), 3),
        "step_time_ratio_2:4_vs_dense": round((tf + tw + ts) / (tf + tw + td), 3),
        "note": "all four columns are this library's kernels (ResNet-9 layers, batch 512, bf16; weight gradient written in fp32); "
                "the ratio is the time of the three convolution passes with the fused 2:4 Magnitude data gradient over the "
                "same with the dense one -- the figure the paper's 15-25 % estimate (Sec. IV-C) is about; library_* columns: "
                "PyTorch's kernels on the same tensors",
    }
    if all("library_forward_us" in r for r in split):
        lf, lw, ll = (sum(r[k] for r in split) for k in ("library_forward_us", "library_weight_grad_us", "library_data_grad_us"))
        result["training_step_split"].update({"library_forward_us": round(lf, 1), "library_weight_grad_us": round(lw, 1),
                                              "library_data_grad_us": round(ll, 1),
                                              "library_data_grad_share": round(ll / (lf + lw + ll), 3)})
    del data

    # ------------------------------------------------------------------ the CPU oracle on a bounded sample of the headline
    if args.cpu_batch > 0:
        import oracle
        small, small_stats = layer_list("r50all", args.cpu_batch)
        t_cpu, f_cpu = 0.0, 0.0
        for i, (L, (dO, W)) in enumerate(zip(small, host_inputs(small, small_stats, workers=4))):
            c0 = time.perf_counter()
            pruned = oracle.prune(dO, 2, 4, oracle.RANDOM, seed=i)[0]
            oracle.conv_bwd_data(pruned, W, L.H, L.Wd, L.stride, L.pad)
            t_cpu += time.perf_counter() - c0
            f_cpu += L.dense_flops
        result["cpu_baseline"] = {
            "value": round(f_cpu / t_cpu / 1e12, 6), "unit": "TFLOP/s (effective)", "cores": oracle.threads(), "kind": "oracle",
            "sample": "the same 54 layers at batch %d, 2:4 random, prune + fp64 product, %.1f s" % (args.cpu_batch, t_cpu),
        }

    print(json.dumps(result))


def roofline_entry(L, ms, setting, sparse, share=None, launches=None):
    """Both roofline fractions of one call; `bound` by the intensity test: issued FLOPs per algorithmic byte against
    the chip's balance point (bf16 MFMA peak / HBM peak).  The structured-sparse instruction issues half of the dense
    multiply-adds, so the fused path's issued FLOPs are half the dense count."""
    issued = (0.5 if sparse else 1.0) * L.dense_flops
    nbytes = L.bytes_moved()
    mfma = issued / (ms * 1e-3) / 1e12
    hbm = nbytes / (ms * 1e-3) / 1e9
    bound = "mfma" if issued / nbytes >= BALANCE_FLOP_PER_BYTE else "hbm"
    e = {"bound": bound, "call": "sdgp_conv_bwd_data %s on %s" % (setting, L.name),
         "achieved": round(mfma if bound == "mfma" else hbm, 2),
         "peak": MFMA_BF16_PEAK_TFLOPS if bound == "mfma" else HBM_PEAK_GBS,
         "unit": "TFLOP/s" if bound == "mfma" else "GB/s",
         "frac": round(mfma / MFMA_BF16_PEAK_TFLOPS if bound == "mfma" else hbm / HBM_PEAK_GBS, 4),
         "frac_of_hbm_peak": round(hbm / HBM_PEAK_GBS, 4), "frac_of_mfma_peak": round(mfma / MFMA_BF16_PEAK_TFLOPS, 4),
         "issued_flop_per_byte": round(issued / nbytes, 1), "balance_flop_per_byte": BALANCE_FLOP_PER_BYTE,
         "traffic": traffic_from_profiles(L.name, setting),
         "traffic_source": "profiles/traffic_per_launch.md (counters of an earlier run, not this one); null = no row",
         "algorithmic_bytes": nbytes, "issued_flops": issued, "launch_us": round(ms * 1e3, 2)}
    if share is not None:
        e["share_of_step"] = round(share, 4)
        e["launches_per_step"] = launches
    return e


def probe(args, sdgp, wl, torch, np, dev, gpu, call):
    """A few launches of one kind and a plain device copy of COPY_BYTES (the counters' calibration)."""
    src = torch.zeros(COPY_BYTES, dtype=torch.uint8, device=dev)
    dst = torch.empty_like(src)
    if args.probe in ("prune", "channel"):
        rows = 256 * 112 * 112
        d = gpu(wl.laplace_with_zeros((rows, 64), 1e-3, 0.3, seed=9000, dtype=wl.BF16))
        for _ in range(args.reps):
            if args.probe == "prune":
                for rk in (sdgp.RANDOM, sdgp.GREEDY, sdgp.GREEDY_ADJUSTED):
                    sdgp.sdgp_prune(d, args.n, args.m, rk, 0)
            else:
                scale = sdgp.sdgp_channel_scales(d, 2, 4)
                sdgp.sdgp_prune_channel_rescaled(d, 2, 4, scale=scale)
            dst.copy_(src)
        torch.cuda.synchronize()
        print(args.probe, tuple(d.shape), "algorithmic bytes: prune", 4 * d.numel(), "factor sweep", 2 * d.numel(),
              "copy bytes each way", COPY_BYTES)
        return
    layers, stats = layer_list(args.workload)
    if args.probe == "pass":          # every layer of the list once: dense, then fused n:m
        picks = list(range(len(layers)))
    else:
        picks = [args.layer]
    for i in picks:
        L, s = layers[i], stats[i]
        dO, W = wl.layer_inputs(L, s[0], s[1], s[2], wl.BF16)
        d, w = gpu(dO), gpu(W)
        out = torch.empty(L.dD_shape, dtype=torch.bfloat16, device=dev)
        if args.probe == "layer":
            # each setting back to back, as the timed table launches them (a launch that follows a different kernel
            # or the copy finds colder caches and measures up to 20 % longer)
            for _ in range(args.reps):
                call(L, d, w, out, args.n, args.m, args.ranker, seed=i)
            for _ in range(args.reps):
                call(L, d, w, out, args.m, args.m, args.ranker, seed=i)
            for _ in range(args.reps):
                dst.copy_(src)
        else:
            for _ in range(args.reps):
                call(L, d, w, out, args.n, args.m, args.ranker, seed=i)
                call(L, d, w, out, args.m, args.m, args.ranker, seed=i)
        torch.cuda.synchronize()
        print("layer", i, L.name, "algorithmic bytes", L.bytes_moved(), "copy bytes each way", COPY_BYTES, flush=True)
        del d, w, out


if __name__ == "__main__":
    main()
