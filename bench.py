#!/usr/bin/env python3
"""Benchmark of the SDGP backward-data path on one MI355X.

Workload (the configuration the headline metric is quoted on): the six 3x3
convolutions of a CIFAR ResNet-9 at batch 512, NHWC bf16, dL/dO ~ Laplace(0, 1e-3)
with 30 % exact zeros, He-normal weights, 2:4 pruning with each of the three
rankers.  One "step" is one pass of the whole hot path over that batch: for
every layer and every ranker one fused call (rank + prune + backward-data
product), 18 calls.  Inputs are resident in HBM before the timed region.

Prints ONE JSON line.  `value` is the effective rate: the FLOPs of the unpruned
products divided by the time the pruned path took.  Extra fields give, per
layer, the fused and the dense hand-written kernel's times (speedup at 2:4, 2:8,
2:16), the prune pass's GB/s, a roofline object for the dominant kernel and the
CPU oracle timed on a bounded sample.
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

HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0
# HBM bytes per launch of the fused 2:4 kernel, from two rocprofv3 --pmc runs (FETCH_SIZE, WRITE_SIZE) scaled by what
# the same counters read for a plain 256 MiB device copy (x2.0 and x1.0); see profiles/bwd_row_traffic.md.
MEASURED_TRAFFIC_BYTES = {"r9_128x256_16": 114.0e6, "r9_64x128_32": 228.3e6, "prune_411MB": 822.1e6}
PAPER_CONTEXT = ("the paper reports no measured rate for this path; it estimates a 15-25 % cut of total training time "
                 "assuming 2:4 sparse tensor-core support on an A100 (abstract, Sec. IV-C)")


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--batch", type=int, default=512, help="batch of the ResNet-9 workload (512 is the named config)")
    ap.add_argument("--cpu-batch", type=int, default=128, help="batch of the CPU-oracle sample (0 skips it)")
    ap.add_argument("--no-extras", action="store_true", help="only the timed steps: no per-layer table, no CPU leg")
    return ap.parse_args()


def main():
    args = parse()
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
    sdgp.binding.load()  # fails loudly when the HIP library is missing
    dev = torch.device("cuda:0")

    def gpu(a):
        return torch.from_numpy(a.view(np.int16)).to(dev).view(torch.bfloat16)

    layers = wl.resnet9_layers(args.batch)
    rankers = (("random", sdgp.RANDOM), ("greedy", sdgp.GREEDY), ("greedy-adjusted", sdgp.GREEDY_ADJUSTED))
    data = []
    for i, L in enumerate(layers):
        dO, W = wl.layer_inputs(L, 1e-3, 0.3, seed=2000 + i, dtype=wl.BF16)
        data.append((L, gpu(dO), gpu(W), torch.empty(L.dD_shape, dtype=torch.bfloat16, device=dev)))
    total_flops = sum(L.dense_flops for L in layers) * len(rankers)

    def call(L, dO, W, out, n, m, rk):
        sdgp.sdgp_conv_bwd_data(dO, W, L.H, L.Wd, L.stride, L.pad, n, m, rk, 0, out=out)

    def step():
        for L, dO, W, out in data:
            for _, rk in rankers:
                call(L, dO, W, out, 2, 4, rk)

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
        "config": {"workload": "ResNet-9 conv3x3 backward-data sweep, batch %d, NHWC bf16, 2:4, rankers random+greedy+"
                               "greedy-adjusted (6 layers x 3 rankers per step)" % args.batch,
                   "n": 2, "m": 4, "batch": args.batch},
        "paper_context": PAPER_CONTEXT,
    }

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

    # ---- roofline of the dominant kernel: the fused sparse kernel of the layer that takes the largest share
    per_layer = []
    for L, dO, W, out in data:
        t_fused = {name: time_call(lambda rk=rk: call(L, dO, W, out, 2, 4, rk)) for name, rk in rankers}
        per_layer.append((L, t_fused))
    dom_i = max(range(len(layers)), key=lambda i: sum(per_layer[i][1].values()))
    Ld, td = per_layer[dom_i]
    dom_ms = td["greedy"]
    issued = 0.5 * Ld.dense_flops  # the structured-sparse instruction issues half of the dense multiply-adds
    result["roofline"] = {
        "bound": "mfma", "kernel": "bwd_row (fused 2:4 greedy, structured-sparse MFMA) on %s" % Ld.name,
        "achieved": round(issued / (dom_ms * 1e-3) / 1e12, 2), "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
        "frac": round(issued / (dom_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
        "traffic": MEASURED_TRAFFIC_BYTES.get(Ld.name),
        "algorithmic_bytes": Ld.bytes_moved(),
        "launch_us": round(dom_ms * 1e3, 2),
        "note": "achieved = FLOPs actually issued per launch (half the dense count: one 2:4 sparse MFMA per two dense "
                "ones) / mean launch time from HIP events; effective rate is twice that; traffic in bytes per launch",
    }
    # the dense hand-written kernel (n == m) on the same layer: all of its FLOPs are issued
    dense_ms = time_call(lambda: call(*data[dom_i], 4, 4, sdgp.GREEDY))
    result["roofline_dense"] = {
        "bound": "mfma", "kernel": "bwd_row (dense, n == m) on %s" % Ld.name,
        "achieved": round(Ld.dense_flops / (dense_ms * 1e-3) / 1e12, 2), "peak": MFMA_BF16_PEAK_TFLOPS,
        "unit": "TFLOP/s", "frac": round(Ld.dense_flops / (dense_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
        "launch_us": round(dense_ms * 1e3, 2),
    }

    if not args.no_extras:
        table = []
        for (L, dO, W, out), (_, t_fused) in zip(data, per_layer):
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
        result["layers"] = table

        # ---- the other named workloads, timed only (their parity is the business of the GPU tests): inputs drawn on
        # the GPU, Laplace magnitudes with exact zeros
        def gpu_inputs(L, scale, zero_frac):
            g = torch.Generator(device=dev)
            g.manual_seed(7)
            mag = torch.empty(L.dO_shape, device=dev).exponential_(generator=g) * scale
            u = torch.rand(L.dO_shape, device=dev, generator=g)
            x = torch.where(u < zero_frac, torch.zeros_like(mag), torch.where(u < zero_frac + (1 - zero_frac) / 2, -mag, mag))
            w = torch.randn(L.W_shape, device=dev, generator=g) * (2.0 / (L.R * L.S * L.C_in)) ** 0.5
            return x.to(torch.bfloat16), w.to(torch.bfloat16), torch.empty(L.dD_shape, dtype=torch.bfloat16, device=dev)

        table = []
        for L in wl.resnet50_bottleneck_layers(128):
            dO, W, out = gpu_inputs(L, 1e-4, 0.4)
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
            del dO, W, out
        result["resnet50_bottleneck_batch128"] = table

        # general n of m (the accuracy study's settings, Sec. IV-B: Rescaled Magnitude): pruned rows stored dense with zeros
        Lg, dOg, Wg, outg = data[3]
        tg = {"dense": time_call(lambda: call(Lg, dOg, Wg, outg, 4, 4, sdgp.GREEDY))}
        for n_, m_ in ((2, 4), (4, 8), (2, 8), (8, 16), (4, 16), (2, 16), (16, 32), (8, 32), (4, 32)):
            tg["%d:%d" % (n_, m_)] = time_call(lambda: call(Lg, dOg, Wg, outg, n_, m_, sdgp.GREEDY_ADJUSTED))
        result["general_nm_greedy_adjusted"] = {"layer": Lg.name, **{k + "_us": round(v * 1e3, 1) for k, v in tg.items()}}

        # the whole ResNet-50 at batch 256 and 224 x 224: every layer once per distinct shape, summed over the 54 layers
        seen, tot = {}, {"dense": 0.0, "2:4_random": 0.0, "2:8_random": 0.0}
        r50 = wl.resnet50_all_layers(256)
        for i, L in enumerate(r50):
            key = (L.H, L.Wd, L.C_in, L.C_out, L.R, L.S, L.stride, L.pad)
            if key not in seen:
                scale, zero_frac = wl.resnet50_layer_stats(i)
                dO, W, out = gpu_inputs(L, scale, zero_frac)
                seen[key] = {name: time_call(lambda: sdgp.sdgp_conv_bwd_data(dO, W, L.H, L.Wd, L.stride, L.pad, n, m, sdgp.RANDOM,
                                                                             i, out=out), reps=5, warm=1)
                             for name, n, m in (("dense", 4, 4), ("2:4_random", 2, 4), ("2:8_random", 2, 8))}
                del dO, W, out
            for name in tot:
                tot[name] += seen[key][name]
        flops = sum(L.dense_flops for L in r50)
        result["resnet50_whole_batch256"] = {
            "layers": len(r50), "distinct_shapes": len(seen), "gflop_dense": round(flops / 1e9, 1),
            **{k + "_ms": round(v, 3) for k, v in tot.items()},
            "speedup_2:4": round(tot["dense"] / tot["2:4_random"], 3), "speedup_2:8": round(tot["dense"] / tot["2:8_random"], 3),
            "effective_tflops_2:4": round(flops / tot["2:4_random"] / 1e9, 1),
            "ideal_ms": round(sum(max(L.bytes_moved() / (HBM_PEAK_GBS * 1e9), L.dense_flops / (MFMA_BF16_PEAK_TFLOPS * 1e12))
                                  for L in r50) * 1e3, 3),
            "note": "sum of per-layer launch times (random ranker seeded with the layer index); ideal = sum over layers of "
                    "max(bytes / HBM peak, dense FLOPs / bf16 MFMA peak)",
        }

        # ---- prune pass: dense-shaped output, tensors too large for the 256 MB last-level cache, rotated
        nelem = 256 * 112 * 112 * 64
        srcs = [gpu(wl.laplace_with_zeros((nelem // 64, 64), 1e-3, 0.3, seed=9000 + i, dtype=wl.BF16)) for i in range(2)]
        dsts = [torch.empty_like(s) for s in srcs]
        lib = sdgp.binding.load()
        import ctypes
        stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
        k = [0]
        prune = {}
        for name, rk in rankers:
            def f(rk=rk):
                s, d = srcs[k[0] % 2], dsts[k[0] % 2]
                k[0] += 1
                rc = lib.sdgp_prune(ctypes.c_void_p(s.data_ptr()), s.shape[0], s.shape[1], sdgp.BF16, 2, 4, rk, 0,
                                    ctypes.c_void_p(d.data_ptr()), None, None, stream)
                assert rc == 0
            ms = time_call(f, reps=20, warm=3)
            prune[name] = {"us": round(ms * 1e3, 1), "GB/s": round(4.0 * nelem / (ms * 1e-3) / 1e9, 1),
                           "frac_of_hbm_peak": round(4.0 * nelem / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
        for n_, m_ in ((2, 8), (2, 16)):
            def g(n_=n_, m_=m_):
                s, d = srcs[k[0] % 2], dsts[k[0] % 2]
                k[0] += 1
                rc = lib.sdgp_prune(ctypes.c_void_p(s.data_ptr()), s.shape[0], s.shape[1], sdgp.BF16, n_, m_, sdgp.GREEDY, 0,
                                    ctypes.c_void_p(d.data_ptr()), None, None, stream)
                assert rc == 0
            ms = time_call(g, reps=20, warm=3)
            prune["greedy_%d:%d" % (n_, m_)] = {"us": round(ms * 1e3, 1), "GB/s": round(4.0 * nelem / (ms * 1e-3) / 1e9, 1),
                                                "frac_of_hbm_peak": round(4.0 * nelem / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
        # compact output (values + uint8 positions, no dense-shaped copy): 2 + 3 n/m bytes per element
        vals = torch.empty(nelem // 2, dtype=torch.bfloat16, device=dev)
        idx = torch.empty(nelem // 2, dtype=torch.uint8, device=dev)

        def compact():
            s = srcs[k[0] % 2]
            k[0] += 1
            rc = lib.sdgp_prune(ctypes.c_void_p(s.data_ptr()), s.shape[0], s.shape[1], sdgp.BF16, 2, 4, sdgp.GREEDY, 0, None,
                                ctypes.c_void_p(vals.data_ptr()), ctypes.c_void_p(idx.data_ptr()), stream)
            assert rc == 0
        ms = time_call(compact, reps=20, warm=3)
        prune["greedy_compact_output"] = {"us": round(ms * 1e3, 1), "GB/s": round(3.5 * nelem / (ms * 1e-3) / 1e9, 1),
                                          "frac_of_hbm_peak": round(3.5 * nelem / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
        del vals, idx
        result["prune_pass"] = {"tensor": "[%d, 64] bf16 (411 MB), 2:4 unless named, dense-shaped output (4 B per element) unless "
                                          "named" % (nelem // 64), **prune}
        result["roofline_prune"] = {"bound": "hbm", "kernel": "prune_items (2:4 greedy)",
                                    "achieved": prune["greedy"]["GB/s"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                    "frac": prune["greedy"]["frac_of_hbm_peak"],
                                    "traffic": MEASURED_TRAFFIC_BYTES["prune_411MB"], "algorithmic_bytes": 4.0 * nelem}
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
        ms_s, ms_p = time_call(sums, reps=20, warm=3), time_call(prune_scaled, reps=20, warm=3)
        per_channel = {
            "channel_scales": {"us": round(ms_s * 1e3, 1), "GB/s": round(2.0 * nelem / (ms_s * 1e-3) / 1e9, 1),
                               "frac_of_hbm_peak": round(2.0 * nelem / (ms_s * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)},
            "prune_channel_rescaled": {"us": round(ms_p * 1e3, 1), "GB/s": round(4.0 * nelem / (ms_p * 1e-3) / 1e9, 1),
                                       "frac_of_hbm_peak": round(4.0 * nelem / (ms_p * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)},
            "fused_layers": [],
        }
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
        # take about a third each on the paper's hardware): forward and weight gradient by PyTorch's library kernels
        # (outside this library's path; context only), data gradient by this library, same layers, same layout
        try:
            split = []
            for L, dO, W, out in data:
                x = torch.randn(L.B, L.H, L.Wd, L.C_in, device=dev, dtype=torch.bfloat16).permute(0, 3, 1, 2)  # NHWC memory
                wt = W.permute(0, 3, 1, 2)                      # [K, C, R, S] view of the KRSC filter
                gy = dO.permute(0, 3, 1, 2)
                t_f = time_call(lambda: torch.nn.functional.conv2d(x, wt, None, L.stride, L.pad), reps=5, warm=2)
                t_w = time_call(lambda: torch.nn.grad.conv2d_weight(x, wt.shape, gy, L.stride, L.pad), reps=5, warm=2)
                t_l = time_call(lambda: torch.nn.grad.conv2d_input(x.shape, wt, gy, L.stride, L.pad), reps=5, warm=2)
                t_d = time_call(lambda: call(L, dO, W, out, 4, 4, sdgp.GREEDY), reps=5)
                t_s = time_call(lambda: call(L, dO, W, out, 2, 4, sdgp.GREEDY), reps=5)
                split.append({"layer": L.name, "forward_us": round(t_f * 1e3, 1), "weight_grad_us": round(t_w * 1e3, 1),
                              "data_grad_library_us": round(t_l * 1e3, 1), "data_grad_dense_us": round(t_d * 1e3, 1),
                              "data_grad_2:4_us": round(t_s * 1e3, 1)})
                del x
            tf, tw = sum(r["forward_us"] for r in split), sum(r["weight_grad_us"] for r in split)
            td, ts = sum(r["data_grad_dense_us"] for r in split), sum(r["data_grad_2:4_us"] for r in split)
            tl = sum(r["data_grad_library_us"] for r in split)
            result["training_step_split"] = {
                "layers": split, "data_grad_share_library": round(tl / (tf + tw + tl), 3),
                "data_grad_share_dense": round(td / (tf + tw + td), 3),
                "step_time_ratio_2:4_vs_dense": round((tf + tw + ts) / (tf + tw + td), 3),
                "step_time_ratio_2:4_vs_library": round((tf + tw + ts) / (tf + tw + tl), 3),
                "note": "forward, weight gradient and data_grad_library: torch (library kernels, bf16 channels-last), not part "
                        "of this library; data_grad_dense and data_grad_2:4: this library (n == m, and fused 2:4 greedy); the "
                        "ratios are what the three convolution passes of these six layers would take with the fused 2:4 data "
                        "gradient instead of this library's dense one / instead of the library's",
            }
        except Exception as e:  # the library convolution is context, not the product: report and go on
            result["training_step_split"] = {"error": repr(e)[:200]}

        # ---- the CPU oracle on a bounded sample of the same workload
        if args.cpu_batch > 0:
            import oracle
            t_cpu, f_cpu = 0.0, 0.0
            for i, L in enumerate(wl.resnet9_layers(args.cpu_batch)):
                dO, W = wl.layer_inputs(L, 1e-3, 0.3, seed=2000 + i, dtype=wl.BF16)
                c0 = time.perf_counter()
                pruned = oracle.prune(dO, 2, 4, oracle.GREEDY, seed=0)[0]
                oracle.conv_bwd_data(pruned, W, L.H, L.Wd, L.stride, L.pad)
                t_cpu += time.perf_counter() - c0
                f_cpu += L.dense_flops
            result["cpu_baseline"] = {
                "value": round(f_cpu / t_cpu / 1e12, 6), "unit": "TFLOP/s (effective)", "cores": oracle.threads(),
                "kind": "oracle",
                "sample": "the same six layers at batch %d, 2:4 greedy, prune + fp64 product, %.1f s" % (args.cpu_batch, t_cpu),
            }

    print(json.dumps(result))


if __name__ == "__main__":
    main()
