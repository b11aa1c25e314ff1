"""Launches one fused backward-data call of a ResNet-9 (or ResNet-50 bottleneck) layer, or the standalone prune pass,
and one plain device copy of known size.

Meant to run under ``rocprofv3 --pmc FETCH_SIZE`` (and again with ``WRITE_SIZE``): the copy calibrates what the
counter reads per byte, the ratio scales the kernel's reading into HBM bytes.  Usage::

    rocprofv3 --pmc FETCH_SIZE -d out -o fetch --output-format csv -- python3 -m paper_2202_00774_amd.traffic_probe --layer 3

``--workload r50`` takes the layer from the ResNet-50 bottleneck list (batch 128); ``--prune`` launches the prune pass
(2:4, all three rankers) on a [3211264, 64] bf16 tensor instead; ``--channel`` launches, on the same tensor, the sweep
that makes the per-channel rescaling factors and the prune pass that applies them.
``--summarize out/fetch_counter_collection.csv`` prints the per-dispatch averages of a finished run.
"""
from __future__ import annotations

import argparse
import collections
import csv
import sys

COPY_BYTES = 256 << 20


def run_prune(reps: int) -> None:
    import numpy as np
    import torch

    import paper_2202_00774_amd as sdgp
    from paper_2202_00774_amd import workloads as wl

    dev = torch.device("cuda:0")
    rows = 256 * 112 * 112
    dO = wl.laplace_with_zeros((rows, 64), 1e-3, 0.3, seed=9000, dtype=wl.BF16)
    d = torch.from_numpy(dO.view(np.int16)).to(dev).view(torch.bfloat16)
    src = torch.zeros(COPY_BYTES, dtype=torch.uint8, device=dev)
    dst = torch.empty_like(src)
    for _ in range(reps):
        for ranker in (sdgp.RANDOM, sdgp.GREEDY, sdgp.GREEDY_ADJUSTED):
            sdgp.sdgp_prune(d, 2, 4, ranker, 0)
        dst.copy_(src)
    torch.cuda.synchronize()
    print("prune pass", tuple(d.shape), "algorithmic bytes", 4 * d.numel(), "copy bytes each way", COPY_BYTES)


def run_channel(reps: int) -> None:
    import numpy as np
    import torch

    import paper_2202_00774_amd as sdgp
    from paper_2202_00774_amd import workloads as wl

    dev = torch.device("cuda:0")
    rows = 256 * 112 * 112
    dO = wl.laplace_with_zeros((rows, 64), 1e-3, 0.3, seed=9000, dtype=wl.BF16)
    d = torch.from_numpy(dO.view(np.int16)).to(dev).view(torch.bfloat16)
    src = torch.zeros(COPY_BYTES, dtype=torch.uint8, device=dev)
    dst = torch.empty_like(src)
    for _ in range(reps):
        scale = sdgp.sdgp_channel_scales(d, 2, 4)
        sdgp.sdgp_prune_channel_rescaled(d, 2, 4, scale=scale)
        dst.copy_(src)
    torch.cuda.synchronize()
    print("per-channel rescale", tuple(d.shape), "algorithmic bytes: factors", 2 * d.numel(), "prune", 4 * d.numel(),
          "copy bytes each way", COPY_BYTES)


def run(workload: str, layer_index: int, n: int, m: int, ranker: int, reps: int) -> None:
    import numpy as np
    import torch

    import paper_2202_00774_amd as sdgp
    from paper_2202_00774_amd import workloads as wl

    dev = torch.device("cuda:0")
    L = (wl.resnet9_layers(512) if workload == "r9" else wl.resnet50_bottleneck_layers(128))[layer_index]
    dO, W = wl.layer_inputs(L, 1e-3, 0.3, seed=2000 + layer_index, dtype=wl.BF16)
    d = torch.from_numpy(dO.view(np.int16)).to(dev).view(torch.bfloat16)
    w = torch.from_numpy(W.view(np.int16)).to(dev).view(torch.bfloat16)
    out = torch.empty(L.dD_shape, dtype=torch.bfloat16, device=dev)
    src = torch.zeros(COPY_BYTES, dtype=torch.uint8, device=dev)
    dst = torch.empty_like(src)
    for _ in range(reps):
        sdgp.sdgp_conv_bwd_data(d, w, L.H, L.Wd, L.stride, L.pad, n, m, ranker, 0, out=out)
        sdgp.sdgp_conv_bwd_data(d, w, L.H, L.Wd, L.stride, L.pad, m, m, ranker, 0, out=out)
        dst.copy_(src)
    torch.cuda.synchronize()
    print("layer", L.name, "algorithmic bytes", L.bytes_moved(), "copy bytes each way", COPY_BYTES)


def summarize(path: str) -> None:
    rows = list(csv.DictReader(open(path)))
    agg = collections.defaultdict(lambda: [0.0, set()])
    for r in rows:
        key = (r["Kernel_Name"][:70], r["Counter_Name"])
        agg[key][0] += float(r["Counter_Value"])
        agg[key][1].add(r["Dispatch_Id"])
    for (k, c), (v, ids) in sorted(agg.items()):
        print(f"{c:12s} {v / len(ids):14.1f} per dispatch ({len(ids)} dispatches)  {k}")


if __name__ == "__main__":
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", choices=("r9", "r50"), default="r9")
    ap.add_argument("--prune", action="store_true")
    ap.add_argument("--channel", action="store_true")
    ap.add_argument("--layer", type=int, default=3)
    ap.add_argument("--n", type=int, default=2)
    ap.add_argument("--m", type=int, default=4)
    ap.add_argument("--ranker", type=int, default=1)
    ap.add_argument("--reps", type=int, default=3)
    ap.add_argument("--summarize", default=None)
    a = ap.parse_args()
    if a.summarize:
        summarize(a.summarize)
        sys.exit(0)
    if a.channel:
        run_channel(a.reps)
    elif a.prune:
        run_prune(a.reps)
    else:
        run(a.workload, a.layer, a.n, a.m, a.ranker, a.reps)
