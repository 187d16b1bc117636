"""A whole network with per-layer batch sizes (Sec. V and VI-B of the paper): the
thirteen layers of the AlexNet runs of Table IV - conv1, norm1, pool1, conv2,
norm2, pool2, conv3, conv4, conv5, pool5, fc6, fc7, fc8, ReLU folded into the layer
before it - over synthetic compressed weights of the benchmark configurations.

Host-side control only: the layers run in the library's kernels, the per-layer batch
sizes come from the library's dynamic program, and the fixed-batch baseline of
Sec. VI-B (the single batch size that fits every layer and is fastest) is picked from
the same measured Time(i, B) table.

    python -m paper_1711_00244_amd.network                     # K = 32, 64, 128; budgets in model sizes
"""
from __future__ import annotations

import argparse
import json
import sys

import numpy as np

from . import binding as cl
from . import workloads as wl
from .scheduler import Plan, StackRunner


class FcOp:
    def __init__(self, name, layer, relu, block):
        self.name, self.layer, self.relu, self.block = name, layer, relu, tuple(block)
        self._ws = {}

    def out_shape(self, in_shape):
        return (self.layer.M,)

    def ws_bytes(self, B, in_shape):
        return cl.fc_workspace_bytes(self.layer, B)

    def forward(self, X, out=None):
        import torch
        B = X.shape[0]
        X = X.reshape(B, -1)
        if B not in self._ws:
            self._ws[B] = torch.empty(max(256, cl.fc_workspace_bytes(self.layer, B)), dtype=torch.uint8, device="cuda")
        return cl.compressed_fc_forward(self.layer, X, relu=self.relu, out=out, workspace=self._ws[B])


class ConvOp:
    """compact: run with the least scratch the library works with (filter groups one
    after the other, blocks decoded inside the multiply kernel) instead of the fast form."""

    def __init__(self, name, layer, geom, block, relu=True, compact=False):
        self.name, self.layer, self.geom, self.relu, self.block = name, layer, geom, relu, tuple(block)
        self.compact = compact
        self._ws = {}

    def out_shape(self, in_shape):
        g = self.geom
        P = (g["H"] + 2 * g["pad"] - g["R"]) // g["stride"] + 1
        Q = (g["W"] + 2 * g["pad"] - g["S"]) // g["stride"] + 1
        return (g["OC"], P, Q)

    def ws_bytes(self, B, in_shape):
        return cl.conv_workspace_bytes(self.layer, self.geom, B, compact=self.compact)

    def forward(self, X, out=None):
        import torch
        B = X.shape[0]
        if B not in self._ws:
            self._ws[B] = torch.empty(max(256, self.ws_bytes(B, None)), dtype=torch.uint8, device="cuda")
        return cl.compressed_conv_forward(self.layer, self.geom, X, relu=self.relu, out=out, workspace=self._ws[B])


class LrnOp:
    def __init__(self, name, n=5, alpha=1e-4, beta=0.75, k=1.0):
        self.name, self.args = name, (n, alpha, beta, k)

    def out_shape(self, in_shape):
        return tuple(in_shape)

    def ws_bytes(self, B, in_shape):
        return 0

    def forward(self, X, out=None):
        return cl.lrn_forward(X, *self.args, out=out)


class PoolOp:
    def __init__(self, name, size=3, stride=2):
        self.name, self.size, self.stride = name, size, stride

    def out_shape(self, in_shape):
        c, h, w = in_shape
        return (c, (h - self.size) // self.stride + 1, (w - self.size) // self.stride + 1)

    def ws_bytes(self, B, in_shape):
        return 0

    def forward(self, X, out=None):
        return cl.maxpool_forward(X, self.size, self.stride, out=out)


class NetworkRunner(StackRunner):
    """StackRunner over heterogeneous layers (anything with forward / out_shape /
    ws_bytes)."""

    def __init__(self, ops, in_shape):
        self.layers = list(ops)
        self.in_shape = tuple(in_shape)
        self.shapes = [self.in_shape]
        for op in self.layers:
            self.shapes.append(tuple(op.out_shape(self.shapes[-1])))

    def layer_forward(self, li, X, out=None):
        return self.layers[li].forward(X.contiguous(), out)

    def measure_times(self, batch_set, reps=10, warmup=2, graphs=False):
        """Time(i, B) in ms.  graphs: the `reps` calls of a layer are captured in a graph
        and replayed, which leaves the caller's per-call cost (Python, ctypes: 10-20 us,
        more than the kernels of a small layer take) out of the figure."""
        import torch
        t = np.zeros((len(self.layers), len(batch_set)))
        for j, B in enumerate(batch_set):
            a = torch.rand((B,) + self.in_shape, device="cuda")
            for li in range(len(self.layers)):
                for _ in range(warmup):
                    out = self.layer_forward(li, a)
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                if graphs:
                    torch.cuda.synchronize()
                    graph = torch.cuda.CUDAGraph()
                    with torch.cuda.graph(graph):
                        for _ in range(reps):
                            out = self.layer_forward(li, a, out)
                    graph.replay()
                    e0.record()
                    graph.replay()
                    e1.record()
                else:
                    e0.record()
                    for _ in range(reps):
                        out = self.layer_forward(li, a, out)
                    e1.record()
                e1.synchronize()
                t[li, j] = e0.elapsed_time(e1) / reps
                a = out
        return t

    def memory_model(self, batch_set):
        """IN, OUT per image and the layer's working memory.  The library's device
        scratch grows with the batch (transposed activations, partial tiles), so its
        per-image share goes with IN and WS(i) is left at zero."""
        inb, outb = [], []
        for li, op in enumerate(self.layers):
            ws_img = max(op.ws_bytes(B, self.shapes[li]) / B for B in batch_set)
            inb.append(int(np.prod(self.shapes[li])) * 4 + int(np.ceil(ws_img)))
            outb.append(int(np.prod(self.shapes[li + 1])) * 4)
        return inb, outb, [0] * len(self.layers)

    def plan(self, batch_set, tot_bytes, mem_step_bytes=100 * 1024, latency_cap_ms=None, time_ms=None):
        time_ms = self.measure_times(batch_set) if time_ms is None else np.asarray(time_ms, float)
        inb, outb, ws = self.memory_model(batch_set)
        ms, bpl = cl.plan_batches(time_ms, batch_set, inb, outb, ws, tot_bytes, mem_step_bytes, latency_cap_ms)
        if bpl is None:
            return None
        return Plan(bpl, ms, list(batch_set), time_ms, ws, int(tot_bytes))

    def fixed_batch(self, batch_set, tot_bytes, time_ms):
        """The baseline of Sec. VI-B: one batch size for all layers that violates the
        memory limit in none of them; among those the one with the best throughput."""
        inb, outb, ws = self.memory_model(batch_set)
        best = None
        for j, B in enumerate(batch_set):
            if all(B * (i + o) + w <= tot_bytes for i, o, w in zip(inb, outb, ws)):
                ms = float(time_ms[:, j].sum()) / B
                if best is None or ms < best[0]:
                    best = (ms, B)
        return best


def compact_copy(net):
    """The same network (the same compressed layers) with its convolutions in the compact form."""
    ops = [ConvOp(op.name, op.layer, op.geom, op.block, op.relu, compact=True) if isinstance(op, ConvOp) else op for op in net.layers]
    return NetworkRunner(ops, net.in_shape)


def alexnet(block=(128, 128), density=None):
    """The AlexNet of Table IV with synthetic compressed layers: configs[3]'s
    convolutions and configs[2]'s FC stack.  density overrides every layer's fraction
    of non-zeros (the uniformly pruned models of Sec. VI-B: 0.3, 0.2, 0.1)."""
    ops = []

    def conv(li):
        spec, W = wl.layer_weights(4, li, density=density)
        g = spec.conv
        bh = cl.conv_block_h(g["OC"], g["groups"], block[0])
        return ConvOp(spec.name, cl.compress_layer(W, spec.r, spec.k, bh, block[1], upload=True), g, (bh, block[1]))

    def fc(li, relu):
        spec, W = wl.layer_weights(3, li, density=density)
        return FcOp(spec.name, cl.compress_layer(W, spec.r, spec.k, block[0], block[1], upload=True), relu, block)

    ops += [conv(0), LrnOp("norm1"), PoolOp("pool1"), conv(1), LrnOp("norm2"), PoolOp("pool2"),
            conv(2), conv(3), conv(4), PoolOp("pool5"), fc(0, True), fc(1, True), fc(2, False)]
    return NetworkRunner(ops, (3, 227, 227))


def main(argv=None):
    import torch
    ap = argparse.ArgumentParser()
    ap.add_argument("--images", type=int, nargs="+", default=[32, 64, 128], help="K: images per request")
    ap.add_argument("--budgets", type=float, nargs="+", default=[1.5, 2.0, 2.5, 8.0, 32.0],
                    help="memory besides the model, in multiples of the compressed model size")
    ap.add_argument("--check", action="store_true", help="run the plan for K images and compare with one-batch execution")
    ap.add_argument("--density", type=float, default=None, help="uniform fraction of non-zeros for all layers")
    ap.add_argument("--graphs", action="store_true", help="time the layers from replayed graphs (no per-call cost of the caller)")
    ap.add_argument("--layer-times", type=int, default=None, metavar="B",
                    help="only time every layer at batch B (fast form) and print ms per layer")
    args = ap.parse_args(argv)
    fast = alexnet(density=args.density)
    if args.layer_times:
        t = fast.measure_times([args.layer_times], graphs=args.graphs)[:, 0]
        print(json.dumps(dict(batch=args.layer_times, density=args.density, timed_from_graphs=args.graphs,
                              ms_per_layer={op.name: round(float(x), 5) for op, x in zip(fast.layers, t)},
                              ms_total=round(float(t.sum()), 4))), flush=True)
        return 0
    nets = {"fast": fast, "compact": compact_copy(fast)}
    model_bytes = sum(op.layer.stats()["model_bytes"] for op in fast.layers if hasattr(op, "layer"))
    for K in args.images:
        batch_set = [b for b in range(1, K + 1) if K % b == 0]
        times = {name: n.measure_times(batch_set, graphs=args.graphs) for name, n in nets.items()}
        for mult in args.budgets:
            tot = int(mult * model_bytes)
            # the convolutions' scratch is part of the budget: both forms of the network are
            # planned, the faster feasible plan (and the faster feasible fixed batch) is reported
            plans = {name: n.plan(batch_set, tot, time_ms=times[name]) for name, n in nets.items()}
            fixeds = {name: n.fixed_batch(batch_set, tot, times[name]) for name, n in nets.items()}
            form = min((nm for nm in nets if plans[nm] is not None), key=lambda nm: plans[nm].ms_per_image, default=None)
            fform = min((nm for nm in nets if fixeds[nm] is not None), key=lambda nm: fixeds[nm][0], default=None)
            plan = plans[form] if form else None
            fixed = fixeds[fform] + (fform,) if fform else None
            net = nets[form] if form else fast
            rec = dict(images=K, density=args.density, timed_from_graphs=args.graphs, budget_x_model=mult, budget_bytes=tot, model_bytes=model_bytes,
                       layers=[op.name for op in net.layers], conv_form=form)
            if plan is None or fixed is None:
                rec["infeasible"] = True
            else:
                rec.update(plan=plan.batch_per_layer, plan_ms_total=round(plan.ms_per_image * K, 4),
                           fixed_batch=fixed[1], fixed_ms_total=round(fixed[0] * K, 4), fixed_conv_form=fixed[2],
                           gain_percent=round(100.0 * (fixed[0] / plan.ms_per_image - 1.0), 1))
                if args.check:
                    X = torch.rand((K, 3, 227, 227), device="cuda")
                    ya = net.run(X, plan.batch_per_layer)
                    yb = net.run(X, None)
                    rec["max_abs_diff_vs_one_batch"] = float((ya - yb).abs().max())
            print(json.dumps(rec), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
