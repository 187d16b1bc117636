#!/usr/bin/env python3
"""Benchmark: images/s through the compressed AlexNet FC6-8 stack on one MI355X.

A step is one forward pass of the whole hot path - Huffman decode of both entry
arrays, position prefix sums, codebook lookup, sparse-weight x dense-activation
product, bias/ReLU - through fc6 -> fc7 -> fc8 for one batch of synthetic images,
with the compressed layers and the input batch already resident in HBM.

Prints ONE JSON line (see README for the fields).
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

PAPER_FC_STACK_IMAGES_PER_S = {16: 1000.0 * 16 / 82.49, 256: 1000.0 * 256 / 181.84}   # Table IV, Xeon E5-2697, MKL 4 threads
HBM_PEAK_GBS = 8000.0
FP32_VECTOR_PEAK_TFLOPS = 157.3
LDS_PEAK_TBS = 256 * 128 * 2.4e9 / 1e12            # 256 CUs x 128 bytes per clock x 2.4 GHz
FP32_MFMA_PEAK_TFLOPS = 157.3
BLOCK = (128, 128)


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--batch", type=int, default=256, help="headline batch size")
    ap.add_argument("--path", choices=["auto", "sparse", "mfma", "bf16", "wide"], default="auto")
    ap.add_argument("--min-warmup-ms", type=float, default=60.0,
                    help="keep running untimed steps after the --warmup ones until this much time has passed (clocks settle)")
    ap.add_argument("--no-sweep", action="store_true", help="skip the batch sweep 1,4,16,64,256")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-bf16", action="store_true", help="skip the extra run on the bf16-tile path")
    ap.add_argument("--no-cold-pool", action="store_true", help="skip the batch-1 steady-state run over separately uploaded copies")
    ap.add_argument("--no-conv", action="store_true", help="skip the side measurement of the AlexNet convolutions")
    ap.add_argument("--conv-batch", type=int, default=64)
    ap.add_argument("--cold-copies", type=int, default=128)
    ap.add_argument("--cpu-batch", type=int, default=256, help="batch of the CPU-oracle sample")
    ap.add_argument("--counter-run", type=int, default=None, metavar="LAYER",
                    help="profiling aid: only run 25 forward calls of this layer of the stack (0 = fc6) at --batch on --path, "
                         "so that a rocprofv3 --pmc run sees the dispatches of one layer; prints a short JSON line")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a 256 MiB device copy a few times (reference kernel of known traffic for rocprofv3 --pmc)")
    return ap.parse_args()


def main():
    args = parse_args()
    if args.gpus != 1:
        print(f"bench.py: this build runs on one GPU only (asked for {args.gpus}); "
              "the compressed model is replicated per GPU when sharded by request, see DESIGN.md", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_1711_00244_amd as cl
    from paper_1711_00244_amd import binding, counters, workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(3)
    torch.cuda.set_device(0)
    path = {"auto": cl.PATH_AUTO, "sparse": cl.PATH_SPARSE, "mfma": cl.PATH_MFMA_F32, "bf16": cl.PATH_MFMA_BF16,
            "wide": cl.PATH_SPARSE_WIDE}[args.path]
    path_names = {cl.PATH_SPARSE: "sparse", cl.PATH_MFMA_F32: "mfma", cl.PATH_MFMA_BF16: "bf16", cl.PATH_SPARSE_WIDE: "wide"}

    # ---- the workload: configs[2], synthetic AlexNet fc6/fc7/fc8 -------------
    cfg = 3
    specs, layers, stats, dense_host = [], [], [], []
    for li in range(3):
        spec, W = wl.layer_weights(cfg, li)
        L = cl.compress_layer(W, spec.r, spec.k, BLOCK[0], BLOCK[1], upload=True)
        specs.append(spec)
        layers.append(L)
        stats.append(L.stats())
        dense_host.append(W)
    model_bytes = sum(s["model_bytes"] for s in stats)
    nnz = [s["nnz"] for s in stats]

    sweep_batches = sorted(set(([] if args.no_sweep else [1, 4, 16, 64, 256]) + [args.batch]))
    batches = sorted(set(sweep_batches + [1]))      # batch 1 always: its kernel gets a roofline entry of its own
    bufs = {}
    for B in batches:
        X = torch.from_numpy(wl.activations(cfg, B)).cuda()
        ys = [torch.empty((B, s.M), dtype=torch.float32, device="cuda") for s in specs]
        ws = [torch.empty(max(1, cl.fc_workspace_bytes(L, B, path)), dtype=torch.uint8, device="cuda") for L in layers]
        bufs[B] = (X, ys, ws)
    stack_ws = {B: torch.empty(max(256, cl.fc_stack_workspace_bytes(layers, B, path)), dtype=torch.uint8, device="cuda")
                for B in batches}

    def step(B):
        # the whole stack through the library's stack entry point: fc6 -> ReLU -> fc7 -> ReLU -> fc8
        X, ys, ws = bufs[B]
        return cl.compressed_fc_stack_forward(layers, X, relu_hidden=True, relu_last=False, path=path, out=ys[-1],
                                              workspace=stack_ws[B])

    def timed(B, steps, warmup):
        # the asked-for warm-up steps, then more of them until min-warmup-ms have passed: a
        # handful of sub-millisecond steps does not bring the clocks up
        t_w = time.perf_counter()
        for _ in range(warmup):
            step(B)
        torch.cuda.synchronize()
        while (time.perf_counter() - t_w) * 1e3 < args.min_warmup_ms:
            for _ in range(10):
                step(B)
            torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            step(B)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / steps

    if args.copy_calibration:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()

    if args.counter_run is not None:
        li, B = args.counter_run, args.batch
        X, ys, ws = bufs[B]
        a = X if li == 0 else torch.rand((B, specs[li].K), device="cuda")
        for _ in range(25):
            cl.compressed_fc_forward(layers[li], a, relu=(li < 2), path=path, out=ys[li], workspace=ws[li])
        torch.cuda.synchronize()
        print(json.dumps({"counter_run": specs[li].name, "batch": B, "path": path_names[cl.fc_resolved_path(layers[li], B, path)],
                          "source_hash": counters.source_hash()}))
        return

    ms = timed(args.batch, args.steps, args.warmup)
    value = args.batch / (ms * 1e-3)

    sweep = {}
    for B in sweep_batches:
        if B == args.batch:
            sweep[str(B)] = {"ms_per_step": round(ms, 5), "images_per_s": round(value, 1)}
            continue
        m = timed(B, max(20, args.steps // 4), max(5, args.warmup // 2))
        sweep[str(B)] = {"ms_per_step": round(m, 5), "images_per_s": round(B / (m * 1e-3), 1)}
    for B in sweep_batches:
        sweep[str(B)]["compressed_GBps"] = round(model_bytes / (sweep[str(B)]["ms_per_step"] * 1e-3) / 1e9, 2)

    # ---- roofline of the dominant kernel (fc6's main kernel), live HIP events ----
    # The library brackets the first main-kernel launch of a forward call with HIP
    # events on the call's stream; fc6 carries 63 % of the stack's entries.
    def kernel_time(li, B, p, reps=50):
        X, ys, _ = bufs[B]
        a = X if li == 0 else ys[li - 1]
        w = torch.empty(max(1, cl.fc_workspace_bytes(layers[li], B, p)), dtype=torch.uint8, device="cuda")
        binding.set_kernel_timing(True)
        ts = []
        for i in range(reps + 10):
            cl.compressed_fc_forward(layers[li], a, relu=(li < 2), path=p, out=ys[li], workspace=w)
            t, n = binding.last_kernel_ms()
            if i >= 10:
                ts.append(t / n)
        binding.set_kernel_timing(False)
        return float(np.mean(ts))

    def traffic_of(kind, B):
        """HBM bytes of the fc6 launch from the counter runs recorded in profiles/counters.json
        (FETCH_SIZE / WRITE_SIZE, scaled by the reference copy's reading), and whether the
        kernel sources have changed since they were taken."""
        fig, stale = counters.lookup(f"{kind}/fc6/{B}")
        if not fig or "fetch_bytes" not in fig or "write_bytes" not in fig:
            return None, None, fig
        return fig["fetch_bytes"] + fig["write_bytes"], stale, fig

    def kernel_roofline(kind, B):
        """fc6's main kernel on the named path at batch B against the roof that bounds it."""
        p = {"sparse": cl.PATH_SPARSE, "mfma": cl.PATH_MFMA_F32, "wide": cl.PATH_SPARSE_WIDE}[kind]
        ms_launch = kernel_time(0, B, p)
        s0, sp = stats[0], specs[0]
        useful = 2.0 * s0["nnz"] * B                      # the method's own work: one multiply-add per surviving weight and image
        traffic, stale, fig = traffic_of(kind, B)
        if kind == "mfma":
            Bp = -(-B // 32) * 32
            executed = 2.0 * sp.M * sp.K * Bp            # every tile product the kernel issues
            r = {"bound": "mfma", "achieved": round(executed / (ms_launch * 1e-3) / 1e12, 3), "peak": FP32_MFMA_PEAK_TFLOPS,
                 "unit": "TFLOP/s", "kernel": "fc_mfma_kernel", "flops_counted": "executed dense-tile flops 2*M*K*B"}
        elif kind == "wide":
            r = {"bound": "alu", "achieved": round(useful / (ms_launch * 1e-3) / 1e12, 3), "peak": FP32_VECTOR_PEAK_TFLOPS,
                 "unit": "TFLOP/s", "kernel": "wide_mul_kernel",
                 "flops_counted": "2*nnz*B, all of them useful",
                 "peak_note": "157.3 = 256 CUs x 128 lanes x 2 flops x 2.4 GHz needs packed fp32; this build issues unpacked "
                              "multiply-adds, whose ceiling is 78.6"}
        else:
            imgs = min(B, 16)                            # the sparse kernel takes batch tiles of up to 16 images
            alg_bytes = s0["model_bytes"] + imgs * (sp.K + sp.M) * 4
            useful = 2.0 * s0["nnz"] * imgs
            r = {"bound": "hbm", "achieved": round(alg_bytes / (ms_launch * 1e-3) / 1e9, 2), "peak": HBM_PEAK_GBS,
                 "unit": "GB/s", "kernel": "fc_sparse_kernel", "algorithmic_bytes_per_launch": int(alg_bytes),
                 "images_per_launch": imgs}
        r["frac"] = round(r["achieved"] / r["peak"], 5)
        r["useful_TFLOPs"] = round(useful / (ms_launch * 1e-3) / 1e12, 4)
        r["frac_useful"] = round(useful / (ms_launch * 1e-3) / 1e12 / (FP32_MFMA_PEAK_TFLOPS if kind == "mfma" else FP32_VECTOR_PEAK_TFLOPS), 5)
        r["traffic"] = traffic
        if traffic is not None:
            r["traffic_stale"] = bool(stale)
        r.update({"layer": "fc6", "batch": B, "launch_ms": round(ms_launch, 5), "path": kind})
        if kind == "wide":
            # what binds this kernel in practice: every surviving weight reads its column's activations for the
            # image tile from LDS once (4 bytes per multiply-add) through a port of 128 bytes per clock and CU
            lds_bytes = 4.0 * s0["nnz"] * B
            r["lds"] = {"achieved": round(lds_bytes / (ms_launch * 1e-3) / 1e12, 2), "peak": LDS_PEAK_TBS, "unit": "TB/s",
                        "frac": round(lds_bytes / (ms_launch * 1e-3) / 1e12 / LDS_PEAK_TBS, 4),
                        "note": "4 bytes of activations from LDS per multiply-add; 256 CUs x 128 B/clk x 2.4 GHz"}
        if kind == "wide":
            r["other_launches"] = "wide_expand_kernel decodes the layer once per call before this kernel (its duration: profiles/)"
        return r, fig

    def roofline_for(B):
        kind = path_names[cl.fc_resolved_path(layers[0], B, path)]
        if kind == "bf16":
            kind = "mfma"
        return kernel_roofline(kind, B)

    headline, _ = roofline_for(args.batch)
    b1, b1_fig = roofline_for(1)
    # both large-batch kernels at the headline batch, so that the choice between them shows
    side = {}
    if args.batch > 4:
        for kind in ("mfma", "wide"):
            try:
                side[kind] = headline if headline["path"] == kind else kernel_roofline(kind, args.batch)[0]
            except cl.CLError as e:
                side[kind] = {"error": str(e)}

    def cold_pool(copies, n_streams, rounds=3):
        """Steady state at batch 1: `copies` separately uploaded copies of fc6 (together
        larger than the 256 MB last-level cache, so every launch reads its layer from
        HBM), one forward each, round robin over n_streams streams of equal priority.
        Returns the compressed bytes per second over all launches."""
        blob = layers[0].serialize()
        pool = [binding.layer_deserialize(blob).upload() for _ in range(copies)]
        streams = [torch.cuda.Stream() for _ in range(n_streams)]
        x1 = bufs[1][0]
        outs = [torch.empty((1, specs[0].M), device="cuda") for _ in range(n_streams)]
        wss = [torch.empty(max(256, cl.fc_workspace_bytes(pool[0], 1, cl.PATH_SPARSE)), dtype=torch.uint8, device="cuda")
               for _ in range(n_streams)]

        def one_round():
            for i, L in enumerate(pool):
                j = i % n_streams
                with torch.cuda.stream(streams[j]):
                    cl.compressed_fc_forward(L, x1, path=cl.PATH_SPARSE, out=outs[j], workspace=wss[j])
        if n_streams == 0:
            # the same pool in one grid (cl_compressed_fc_group_forward): one launch for the
            # decode-and-multiply of all copies, one for the finishing
            group = cl.LayerGroup(pool)
            gout = torch.empty((copies, 1, specs[0].M), device="cuda")
            gws = torch.empty(max(256, group.workspace_bytes(1)), dtype=torch.uint8, device="cuda")

            def one_round():                                           # noqa: F811
                group.forward(x1, out=gout, workspace=gws)
        one_round()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(rounds):
            one_round()
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / (rounds * copies)
        if n_streams == 0:
            group.free()
        for L in pool:
            L.free()
        alg_bytes = stats[0]["model_bytes"] + (specs[0].K + specs[0].M) * 4
        if n_streams == 0:
            return {"copies": copies, "one_grid": True, "us_per_layer": round(dt * 1e6, 3),
                    "achieved": round(alg_bytes / dt / 1e9, 2), "unit": "GB/s", "frac": round(alg_bytes / dt / 1e9 / HBM_PEAK_GBS, 5)}
        return {"copies": copies, "streams": n_streams, "us_per_launch_pair": round(dt * 1e6, 3),
                "achieved": round(alg_bytes / dt / 1e9, 2), "unit": "GB/s", "frac": round(alg_bytes / dt / 1e9 / HBM_PEAK_GBS, 5)}

    # ---- the same step on the bf16-tile path (three bf16 products per fp32 product) ----
    def bf16_tiles(B):
        pb = cl.PATH_MFMA_BF16
        X, ys, _ = bufs[B]
        ysb = [torch.empty_like(y) for y in ys]
        wsb = [torch.empty(max(1, cl.fc_workspace_bytes(L, B, pb)), dtype=torch.uint8, device="cuda") for L in layers]

        wss = torch.empty(max(256, cl.fc_stack_workspace_bytes(layers, B, pb)), dtype=torch.uint8, device="cuda")

        def stepb():
            return cl.compressed_fc_stack_forward(layers, X, relu_hidden=True, relu_last=False, path=pb, out=ysb[2], workspace=wss)
        for _ in range(args.warmup):
            stepb()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            stepb()
        torch.cuda.synchronize()
        msb = (time.perf_counter() - t0) * 1e3 / args.steps
        step(B)
        torch.cuda.synchronize()
        diff = float((ysb[2] - ys[2]).abs().max() / ys[2].abs().max())
        binding.set_kernel_timing(True)
        ts = []
        for i in range(30):
            cl.compressed_fc_forward(layers[0], X, relu=True, path=pb, out=ysb[0], workspace=wsb[0])
            t, n = binding.last_kernel_ms()
            if i >= 5:
                ts.append(t / n)
        binding.set_kernel_timing(False)
        kms = float(np.mean(ts))
        Bp = -(-B // 32) * 32
        executed = 3 * 2.0 * specs[0].M * specs[0].K * Bp         # three bf16 tile products per fp32 one
        return {"value": round(B / (msb * 1e-3), 1), "unit": "images/s", "ms_per_step": round(msb, 5), "batch": B, "dtype": "bf16 x3, f32 accumulate",
                "max_abs_diff_vs_f32_path_over_max_abs": diff,
                "roofline": {"bound": "mfma", "kernel": "fc_mfma_bf16_kernel", "layer": "fc6", "launch_ms": round(kms, 5),
                             "achieved": round(executed / (kms * 1e-3) / 1e12, 1), "peak": 2500.0, "unit": "TFLOP/s",
                             "frac": round(executed / (kms * 1e-3) / 1e12 / 2500.0, 4),
                             "flops_counted": "executed bf16 tile flops 3*2*M*K*B",
                             "fp32_equivalent_TFLOPs": round(executed / 3 / (kms * 1e-3) / 1e12, 1)}}

    # The batch-1 kernel against what binds it: vector-ALU issue.  Peak = 256 CUs x 4 SIMDs x
    # 2.4 GHz / 4 cycles per wavefront instruction; the instruction count of the fc6 launch is
    # the SQ_INSTS_VALU counter recorded in profiles/counters.json.
    if b1_fig and "SQ_INSTS_VALU" in b1_fig:
        valu_insts = b1_fig["SQ_INSTS_VALU"]
        b1["alu"] = {"bound": "alu", "achieved": round(valu_insts / (b1["launch_ms"] * 1e-3) / 1e9, 1), "peak": 614.4,
                     "unit": "G wavefront VALU instructions/s", "valu_instructions_per_launch": int(valu_insts),
                     "stale": bool(counters.lookup("sparse/fc6/1")[1])}
        b1["alu"]["frac"] = round(b1["alu"]["achieved"] / b1["alu"]["peak"], 4)

    if not args.no_cold_pool:
        b1["steady_state_cold"] = [cold_pool(args.cold_copies, 1), cold_pool(args.cold_copies, 4), cold_pool(args.cold_copies, 0)]

    out = {
        "metric": "images/sec through compressed AlexNet FC6-8",
        "value": round(value, 1),
        "unit": "images/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": round(value / PAPER_FC_STACK_IMAGES_PER_S[args.batch], 2) if args.batch in PAPER_FC_STACK_IMAGES_PER_S else None,
        "baseline_note": "paper Table IV fc6+fc7+fc8, Xeon E5-2697, MKL 4 threads, real AlexNet weights (another machine: context only)",
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": "configs[2]: AlexNet FC stack 9216-4096-4096-1000, densities 9/9/25 %, 5-bit codebook, "
                               "4-bit relative index, Huffman-coded, 128x128 blocks, ReLU between layers",
                   "batch": args.batch, "path": args.path, "block": list(BLOCK),
                   "compressed_model_bytes": int(model_bytes), "nnz": nnz},
        "sweep": sweep,
        "roofline": headline,
        "roofline_batch1": b1,
        "large_batch_kernels": side,
    }
    if not args.no_bf16 and args.path == "auto":
        out["bf16_tiles"] = bf16_tiles(args.batch)

    # ---- beside the metric: the five AlexNet convolutions (configs[3]) through cl_compressed_conv_forward ----
    if not args.no_conv and args.path == "auto":
        Bc, per_layer = args.conv_batch, {}
        for li in range(5):
            cspec, cW = wl.layer_weights(4, li)
            g = cspec.conv
            Lc = cl.compress_layer(cW, cspec.r, cspec.k, cl.conv_block_h(g["OC"], g["groups"]), 128, upload=True)
            Xc = torch.from_numpy(wl.activations(4, Bc, layer_index=li)).cuda()
            P = (g["H"] + 2 * g["pad"] - g["R"]) // g["stride"] + 1
            Yc = torch.empty((Bc, g["OC"], P, P), device="cuda")
            wsc = torch.empty(max(256, cl.conv_workspace_bytes(Lc, g, Bc)), dtype=torch.uint8, device="cuda")
            for _ in range(5):
                cl.compressed_conv_forward(Lc, g, Xc, relu=True, out=Yc, workspace=wsc)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(20):
                cl.compressed_conv_forward(Lc, g, Xc, relu=True, out=Yc, workspace=wsc)
            torch.cuda.synchronize()
            per_layer[cspec.name] = round((time.perf_counter() - t0) * 1e3 / 20, 5)
            Lc.free()
        total = sum(per_layer.values())
        out["conv_alexnet"] = {"workload": "configs[3]: AlexNet conv1-5 at 84/38/35/37/37 % density, 8-bit codebook and relative index, ReLU",
                               "batch": Bc, "ms_per_layer": per_layer, "ms_total": round(total, 5),
                               "images_per_s": round(Bc / (total * 1e-3), 1), "dtype": "f32"}

    # ---- the CPU oracle on the host cores, same workload, bounded sample -----
    if not args.no_cpu_baseline:
        import oracle
        Bc = args.cpu_batch
        Xc = wl.activations(cfg, Bc)
        try:
            ncores = len(os.sched_getaffinity(0))
        except AttributeError:
            ncores = os.cpu_count() or 1
        ncores = max(1, min(ncores, int(os.environ.get("OMP_NUM_THREADS", ncores) or ncores)))
        t_all0 = time.perf_counter()
        models = [oracle.compress_layer(W, spec.r, spec.k, BLOCK[0], BLOCK[1]) for spec, W in zip(specs, dense_host)]   # offline, not timed
        t_dec = t_rec = 0.0
        dense = []
        for m in models:
            t0 = time.perf_counter()
            v3, i3, bp = oracle.decode_layer(m)          # Algorithm 2 steps 3-6, block by block (one thread: a bit-serial walk)
            t_dec += time.perf_counter() - t0
            t0 = time.perf_counter()
            dense.append(oracle.dense_weights(m, v3, i3, bp))
            t_rec += time.perf_counter() - t0

        def products(nthreads):
            a, t = Xc, 0.0
            for li, Wd in enumerate(dense):
                t0 = time.perf_counter()
                y = oracle.fc_forward(Wd, a, None, relu=(li < 2), nthreads=nthreads)
                t += time.perf_counter() - t0
                a = y.astype(np.float32)
            return t
        t_mm_all = products(ncores)
        t_mm_one = products(1)
        t_cpu = t_dec + t_rec + t_mm_all
        out["cpu_baseline"] = {
            "value": round(Bc / t_cpu, 2), "unit": "images/s", "cores": ncores, "kind": "oracle",
            "sample": f"one pass of the same FC6-8 stack at batch {Bc}: bit-serial Huffman decode {t_dec:.2f} s + dense "
                      f"rebuild {t_rec:.2f} s (one thread each) + triple-loop fp64 product {t_mm_all:.2f} s on {ncores} threads "
                      f"(compression not timed)",
            "one_thread": {"value": round(Bc / (t_dec + t_rec + t_mm_one), 2), "unit": "images/s", "cores": 1,
                           "product_s": round(t_mm_one, 2)},
            "host_cpus": os.cpu_count(), "wall_s": round(time.perf_counter() - t_all0, 1)}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
