"""Per-layer timings for the benchmark configurations other than the headline one
(bench.py covers configs[2]), and the two sweeps of the paper's evaluation that a
format parameter makes cheap: time against block size (Sec. VI-A, the figure behind
the 128 x 128 choice) and against the pruning level (the uniform 70/80/90 % models).
Prints one JSON line per (layer, block, density, path, batch).

    python -m paper_1711_00244_amd.measure --config 4          # AlexNet conv layers
    python -m paper_1711_00244_amd.measure --config 2          # AlexNet fc6, batch 1 and 8
    python -m paper_1711_00244_amd.measure --config 6          # VGG-16 convolutions
    python -m paper_1711_00244_amd.measure --config 2 --batches 16 256 \
        --blocks 16x16 32x32 64x64 128x128 256x256 512x512 1024x1024 4096x9216
    python -m paper_1711_00244_amd.measure --config 2 --batches 1 16 64 256 \
        --densities 0.3 0.2 0.1 0.05 --paths sparse mfma
"""
from __future__ import annotations

import argparse
import json
import sys

import numpy as np

from . import binding as cl
from . import workloads as wl


def time_ms(fn, reps, warmup):
    import torch
    for _ in range(warmup):
        fn()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    e1.synchronize()
    return e0.elapsed_time(e1) / reps


def main(argv=None):
    import torch
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", type=int, required=True, choices=[1, 2, 3, 4, 5, 6])
    ap.add_argument("--reps", type=int, default=30)
    ap.add_argument("--block", type=int, nargs=2, default=[128, 128])
    ap.add_argument("--blocks", nargs="+", default=None, help="block sizes to sweep, as HxW")
    ap.add_argument("--batches", type=int, nargs="+", default=None, help="override the configuration's batch sizes")
    ap.add_argument("--densities", type=float, nargs="+", default=[None], help="override the fraction of non-zeros")
    ap.add_argument("--paths", nargs="+", default=["auto"], choices=["auto", "sparse", "mfma", "bf16"])
    ap.add_argument("--layers", type=int, nargs="+", default=None, help="layer indices (default: all)")
    args = ap.parse_args(argv)
    cfg = wl.CONFIGS[args.config]
    paths = {"auto": cl.PATH_AUTO, "sparse": cl.PATH_SPARSE, "mfma": cl.PATH_MFMA_F32, "bf16": cl.PATH_MFMA_BF16}
    blocks = [tuple(int(t) for t in b.lower().split("x")) for b in args.blocks] if args.blocks else [tuple(args.block)]
    for li, spec0 in enumerate(cfg["layers"]):
        if args.layers is not None and li not in args.layers:
            continue
        for density in args.densities:
            spec, W = wl.layer_weights(args.config, li, density=density)
            for bh, bw in blocks:
                if spec.conv is not None:
                    bh = cl.conv_block_h(spec.conv["OC"], spec.conv["groups"], bh)
                L = cl.compress_layer(W, spec.r, spec.k, bh, bw, upload=True)
                st = L.stats()
                for B in (args.batches or cfg["batches"]):
                    X = torch.from_numpy(wl.activations(args.config, B, layer_index=li)).cuda()
                    for pname in args.paths:
                        path = paths[pname]
                        try:
                            if spec.conv is not None:
                                g = spec.conv
                                ws = torch.empty(max(256, cl.conv_workspace_bytes(L, g, B, path)), dtype=torch.uint8, device="cuda")
                                P = (g["H"] + 2 * g["pad"] - g["R"]) // g["stride"] + 1
                                out = torch.empty((B, g["OC"], P, P), device="cuda")
                                ms = time_ms(lambda: cl.compressed_conv_forward(L, g, X, relu=True, path=path, out=out, workspace=ws), args.reps, 3)
                                n_cols = B * P * P
                            else:
                                ws = torch.empty(max(256, cl.fc_workspace_bytes(L, B, path)), dtype=torch.uint8, device="cuda")
                                out = torch.empty((B, spec.M), device="cuda")
                                ms = time_ms(lambda: cl.compressed_fc_forward(L, X, out=out, path=path, workspace=ws), args.reps, 3)
                                n_cols = B
                        except cl.CLError as e:
                            print(json.dumps(dict(config=args.config, layer=spec.name, batch=B, block=[bh, bw], path=pname,
                                                  density=spec.density, unsupported=str(e))), flush=True)
                            continue
                        print(json.dumps(dict(config=args.config, layer=spec.name, batch=B, block=[bh, bw], path=pname,
                                              density=spec.density, ms=round(ms, 5),
                                              images_per_s=round(B / (ms * 1e-3), 1), model_bytes=st["model_bytes"], nnz=st["nnz"],
                                              bits_per_nnz=round(8.0 * st["model_bytes"] / max(1, st["nnz"]), 2),
                                              compressed_GBps=round(st["model_bytes"] / (ms * 1e-3) / 1e9, 2),
                                              dense_TFLOPs=round(2.0 * spec.M * spec.K * n_cols / (ms * 1e-3) / 1e12, 3),
                                              useful_TFLOPs=round(2.0 * st["nnz"] * n_cols / (ms * 1e-3) / 1e12, 3))), flush=True)
                L.free()
    return 0


if __name__ == "__main__":
    sys.exit(main())
