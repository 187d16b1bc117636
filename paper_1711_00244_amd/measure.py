"""Per-layer timings for the benchmark configurations other than the headline one
(bench.py covers configs[2]), and the two sweeps of the paper's evaluation that a
format parameter makes cheap: time against block size (Sec. VI-A, the figure behind
the 128 x 128 choice) and against the pruning level (the uniform 70/80/90 % models).
Prints one JSON line per (layer, block, density, path, batch); with --decode also one
per (layer, block, density) with the time of the decoding alone (cl_decode_layer:
Huffman decode of both arrays and the prefix sums, symbols written out) and of the
decoding with the dense matrix rebuilt - the decode / compute / total split of the
paper's block-size figure: the forward kernels fuse the three, so the split is the
decode-only launch beside the fused total, not a sum.

    python -m paper_1711_00244_amd.measure --config 4          # AlexNet conv layers
    python -m paper_1711_00244_amd.measure --config 2          # AlexNet fc6, batch 1 and 8
    python -m paper_1711_00244_amd.measure --config 6          # VGG-16 convolutions
    python -m paper_1711_00244_amd.measure --config 2 --batches 16 256 \
        --blocks 16x16 32x32 64x64 128x128 256x256 512x512 1024x1024 4096x9216
    python -m paper_1711_00244_amd.measure --config 2 --batches 1 16 64 256 \
        --densities 0.3 0.2 0.1 0.05 --paths sparse mfma wide
    python -m paper_1711_00244_amd.measure --config 2 --batches 16 256 --decode --markdown \
        --blocks 16x16 32x32 64x64 128x128 256x256 512x512 1024x1024 2048x2048 4096x4096
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
    ap.add_argument("--paths", nargs="+", default=["auto"], choices=["auto", "sparse", "mfma", "bf16", "wide"])
    ap.add_argument("--decode", action="store_true", help="also time the decoding alone, per layer, block size and density")
    ap.add_argument("--markdown", action="store_true", help="after the JSON lines, the same figures as a markdown table")
    ap.add_argument("--layers", type=int, nargs="+", default=None, help="layer indices (default: all)")
    args = ap.parse_args(argv)
    cfg = wl.CONFIGS[args.config]
    paths = {"auto": cl.PATH_AUTO, "sparse": cl.PATH_SPARSE, "mfma": cl.PATH_MFMA_F32, "bf16": cl.PATH_MFMA_BF16,
             "wide": cl.PATH_SPARSE_WIDE}
    names = {v: k for k, v in paths.items()}
    rows = []

    def emit(rec):
        rows.append(rec)
        print(json.dumps(rec), flush=True)
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
                if args.decode:
                    import ctypes as C
                    val = torch.empty(st["entries"], dtype=torch.uint8, device="cuda")
                    idx = torch.empty(st["entries"], dtype=torch.uint8, device="cuda")
                    dense = torch.empty((spec.M, spec.K), dtype=torch.float32, device="cuda")
                    stream = C.c_void_p(torch.cuda.current_stream().cuda_stream)

                    def decode(with_dense):
                        rc = cl.lib().cl_decode_layer(L.handle, C.c_void_p(val.data_ptr()), C.c_void_p(idx.data_ptr()), None,
                                                      C.c_void_p(dense.data_ptr()) if with_dense else None, stream)
                        assert rc == 0, rc
                    emit(dict(config=args.config, layer=spec.name, block=[bh, bw], density=spec.density, entries=st["entries"],
                              chunks=st["n_chunks"], bits_per_nnz=round(8.0 * st["model_bytes"] / max(1, st["nnz"]), 2),
                              decode_ms=round(time_ms(lambda: decode(False), args.reps, 3), 5),
                              decode_and_rebuild_ms=round(time_ms(lambda: decode(True), args.reps, 3), 5)))
                    del val, idx, dense
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
                            emit(dict(config=args.config, layer=spec.name, batch=B, block=[bh, bw], path=pname,
                                      density=spec.density, unsupported=str(e)))
                            continue
                        ran = pname if spec.conv is not None else names[cl.fc_resolved_path(L, B, path)]
                        emit(dict(config=args.config, layer=spec.name, batch=B, block=[bh, bw], path=pname, ran=ran,
                                              density=spec.density, ms=round(ms, 5),
                                              images_per_s=round(B / (ms * 1e-3), 1), model_bytes=st["model_bytes"], nnz=st["nnz"],
                                              bits_per_nnz=round(8.0 * st["model_bytes"] / max(1, st["nnz"]), 2),
                                              compressed_GBps=round(st["model_bytes"] / (ms * 1e-3) / 1e9, 2),
                                              dense_TFLOPs=round(2.0 * spec.M * spec.K * n_cols / (ms * 1e-3) / 1e12, 3),
                                              useful_TFLOPs=round(2.0 * st["nnz"] * n_cols / (ms * 1e-3) / 1e12, 3)))
                L.free()
    if args.markdown:
        print()
        keys = sorted({(r["layer"], r["density"], tuple(r["block"])) for r in rows}, key=lambda k: (k[0], -k[1], k[2][0] * k[2][1]))
        cols = sorted({(r["batch"], r["path"]) for r in rows if "batch" in r})
        head = ["layer", "density", "block", "bits/nnz", "decode ms", "decode+rebuild ms"] + [f"B={b} {p} ms" for b, p in cols]
        print("| " + " | ".join(head) + " |")
        print("|" + "---|" * len(head))
        for layer, density, block in keys:
            mine = [r for r in rows if r["layer"] == layer and r["density"] == density and tuple(r["block"]) == block]
            dec = next((r for r in mine if "decode_ms" in r), {})
            bits = next((r["bits_per_nnz"] for r in mine if "bits_per_nnz" in r), "")
            cells = [layer, f"{density:g}", f"{block[0]}x{block[1]}", str(bits), str(dec.get("decode_ms", "")), str(dec.get("decode_and_rebuild_ms", ""))]
            for b, pth in cols:
                r = next((r for r in mine if r.get("batch") == b and r.get("path") == pth), None)
                cells.append("" if r is None else "unsupported" if "unsupported" in r else f"{r['ms']} ({r['ran']})")
            print("| " + " | ".join(cells) + " |")
    return 0


if __name__ == "__main__":
    sys.exit(main())
