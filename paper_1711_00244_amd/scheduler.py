"""Variable batch sizes for a stack of compressed layers (Sec. V-C/D of the paper)
and a request scheduler around it.

Host-side control only: the per-layer batch sizes come from the library's dynamic
program (``cl_plan_batches``), every layer runs in the library's kernels.

* ``measure_times``  - Time(i, B): "obtained once for a given compressed model".
* ``plan``           - the dynamic program under a memory budget TOT and a latency
                       threshold; WS(i) is the device scratch the library asks for.
* ``StackRunner.run``- runs K images with per-layer batch sizes: to run layer i once
                       at batch B, the layers before it run B / b times at batch b,
                       their outputs parked until B of them are there.
* ``simulate``       - single-image requests arriving as a Poisson stream; batches
                       are formed under a per-request latency cap.  The GPU work of
                       every dispatched batch is real; the clock advances either by
                       the cost the dynamic program assigns to the per-layer batch
                       sizes that were dispatched (``clock="model"``, reproducible)
                       or by the duration of the dispatch measured with HIP events
                       (``clock="measured"``).
"""
from __future__ import annotations

import argparse
import json
import sys
from dataclasses import dataclass

import numpy as np

from . import binding as cl


@dataclass
class Plan:
    batch_per_layer: list
    ms_per_image: float
    batch_set: list
    time_ms: np.ndarray          # [layer][batch index]
    ws_bytes: list
    tot_bytes: int

    def dispatch_ms(self, bpl) -> float:
        """Cost of running bpl[-1] images with per-layer batch sizes bpl (a monotone
        divisor chain of members of batch_set): the recurrence of Sec. V-C,
        cost(i) = Time(i, bpl[i]) + (bpl[i] / bpl[i-1]) cost(i-1) - every earlier
        layer is repeated until the later layer's batch is full."""
        cost = 0.0
        for i, b in enumerate(bpl):
            reps = 1 if i == 0 else b // bpl[i - 1]
            cost = float(self.time_ms[i, self.batch_set.index(b)]) + reps * cost
        return cost

    def bpl_for(self, B: int) -> list:
        """Per-layer batch sizes for a dispatch of B images (B in batch_set): the plan's,
        capped at B; a size that does not divide B gives way to B."""
        bpl = [min(b, B) for b in self.batch_per_layer]
        return [b if B % b == 0 else B for b in bpl]


class StackRunner:
    """fc -> ReLU -> fc -> ... -> fc over compressed layers."""

    def __init__(self, layers, path=cl.PATH_AUTO):
        self.layers = list(layers)
        self.path = path
        self._ws = {}

    def _workspace(self, li, B):
        import torch
        key = (li, B)
        if key not in self._ws:
            n = cl.fc_workspace_bytes(self.layers[li], B, self.path)
            self._ws[key] = torch.empty(max(n, 256), dtype=torch.uint8, device="cuda")
        return self._ws[key]

    def layer_forward(self, li, X, out=None):
        relu = li + 1 < len(self.layers)
        return cl.compressed_fc_forward(self.layers[li], X, relu=relu, path=self.path, out=out,
                                        workspace=self._workspace(li, X.shape[0]))

    def run(self, X, batch_per_layer=None):
        """All rows of X through the stack.  batch_per_layer must be a monotone
        divisor chain (what the dynamic program returns); None = one batch."""
        import torch
        n = X.shape[0]
        f = len(self.layers)
        bpl = [n] * f if batch_per_layer is None else list(batch_per_layer)
        top = bpl[-1]
        outs = []
        for s in range(0, n, top):                      # a remainder smaller than the plan's top batch runs as one batch
            xs = X[s:s + top]
            if xs.shape[0] == top:
                outs.append(self._run_level(f - 1, xs, bpl))
            else:
                a = xs
                for li in range(f):
                    a = self.layer_forward(li, a)
                outs.append(a)
        return torch.cat(outs, 0)

    def _run_level(self, li, xs, bpl):
        """Output of layer li for the rows xs (len(xs) == bpl[li]): the earlier
        layers run in phases of bpl[li - 1] rows whose outputs are parked."""
        import torch
        if li == 0:
            return self.layer_forward(0, xs.contiguous())
        b = bpl[li - 1]
        parked = [self._run_level(li - 1, xs[s:s + b], bpl) for s in range(0, xs.shape[0], b)]
        a = parked[0] if len(parked) == 1 else torch.cat(parked, 0)
        return self.layer_forward(li, a)

    # ------------------------------------------------------------------ #
    def measure_times(self, batch_set, reps=20, warmup=3):
        """Time(i, B) in ms with HIP events on the current stream."""
        import torch
        t = np.zeros((len(self.layers), len(batch_set)))
        for j, B in enumerate(batch_set):
            a = torch.rand((B, self.layers[0].K), device="cuda")
            for li, L in enumerate(self.layers):
                out = torch.empty((B, L.M), device="cuda")
                for _ in range(warmup):
                    self.layer_forward(li, a, out)
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for _ in range(reps):
                    self.layer_forward(li, a, out)
                e1.record()
                e1.synchronize()
                t[li, j] = e0.elapsed_time(e1) / reps
                a = out
        return t

    def plan(self, batch_set, tot_bytes, mem_step_bytes=100 * 1024, latency_cap_ms=None, time_ms=None):
        """The dynamic program over batch_set.  WS(i) is one figure per layer - the most
        scratch the layer asks for at any candidate batch size - so a candidate whose
        scratch alone breaks the budget would rule out every plan: the largest candidates
        are dropped one by one until a plan exists (None if not even the smallest fits)."""
        batch_set = list(batch_set)
        time_ms = self.measure_times(batch_set) if time_ms is None else np.asarray(time_ms, float)
        inb = [L.K * 4 for L in self.layers]
        outb = [L.M * 4 for L in self.layers]
        for cut in range(len(batch_set), 0, -1):
            bs = batch_set[:cut]
            ws = [max(cl.fc_workspace_bytes(L, B, self.path) for B in bs) for L in self.layers]
            ms, bpl = cl.plan_batches(time_ms[:, :cut], bs, inb, outb, ws, tot_bytes, mem_step_bytes, latency_cap_ms)
            if bpl is not None:
                return Plan(bpl, ms, bs, time_ms[:, :cut], ws, int(tot_bytes))
        return None


def simulate(runner: StackRunner, plan: Plan, arrivals_s, inputs, latency_cap_ms, clock="model"):
    """Serve single-image requests arriving at arrivals_s (ascending, seconds).

    When the GPU is idle and requests wait, the largest candidate batch B <= queue
    is dispatched as soon as (i) the queue has reached the plan's batch, or (ii)
    waiting for the next larger candidate would push the oldest request past the
    cap (its wait so far + the cost of that larger dispatch), or no more requests
    will come.  A dispatch of B images runs with the per-layer batch sizes
    plan.bpl_for(B) and is charged plan.dispatch_ms of exactly those sizes
    (clock="model") or its measured duration (clock="measured": HIP events around
    the dispatch, the device idle before it).  Returns (outputs in request order,
    stats)."""
    import torch
    assert clock in ("model", "measured")
    n = len(arrivals_s)
    bs = [b for b in plan.batch_set if b <= plan.batch_per_layer[-1]] or [plan.batch_set[0]]
    target = bs[-1]
    cap_s = latency_cap_ms * 1e-3
    done = np.zeros(n)
    outputs = [None] * n
    now, head, served = 0.0, 0, 0
    predicted_ms = charged_ms = 0.0
    batches = []
    while served < n:
        if head <= served:                                   # nobody waiting: jump to the next arrival
            now = max(now, arrivals_s[served])
        while head < n and arrivals_s[head] <= now:
            head += 1
        q = head - served
        B = max(b for b in bs if b <= q)
        if q < target and head < n:
            nxt = min(b for b in bs if b > B)                # next larger candidate
            t_fill = arrivals_s[served + nxt - 1] if served + nxt - 1 < n else np.inf
            # keep waiting only if the oldest request would still meet the cap with the larger batch
            if t_fill + plan.dispatch_ms(plan.bpl_for(nxt)) * 1e-3 - arrivals_s[served] <= cap_s:
                now = t_fill
                continue
        idx = list(range(served, served + B))
        X = torch.stack([inputs[i] for i in idx], 0)
        bpl = plan.bpl_for(B)
        if clock == "measured":
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            Y = runner.run(X, bpl)
            e1.record()
            e1.synchronize()
            spent_ms = e0.elapsed_time(e1)
        else:
            Y = runner.run(X, bpl)
            spent_ms = plan.dispatch_ms(bpl)
        predicted_ms += plan.dispatch_ms(bpl)
        charged_ms += spent_ms
        now += spent_ms * 1e-3
        for k, i in enumerate(idx):
            outputs[i] = Y[k]
            done[i] = now
        batches.append(B)
        served += B
    lat = (done - np.asarray(arrivals_s)) * 1e3
    stats = dict(requests=n, batches=len(batches), mean_batch=float(np.mean(batches)), p50_ms=float(np.percentile(lat, 50)),
                 p99_ms=float(np.percentile(lat, 99)), max_ms=float(lat.max()), span_s=float(done.max() - arrivals_s[0]),
                 images_per_s=float(n / (done.max() - arrivals_s[0])), over_cap=int((lat > latency_cap_ms + 1e-9).sum()),
                 clock=clock, gpu_ms_charged=charged_ms, gpu_ms_predicted=predicted_ms)
    return outputs, stats


def main(argv=None):
    """configs[4]: VGG-16 FC stack, decoded-buffer / activation budget and latency
    cap, Poisson stream of single-image requests."""
    import torch
    from . import workloads as wl
    ap = argparse.ArgumentParser()
    ap.add_argument("--rate", type=float, default=20000.0, help="requests per second")
    ap.add_argument("--requests", type=int, default=4096)
    ap.add_argument("--budget-mb", type=float, default=64.0)
    ap.add_argument("--latency-cap-ms", type=float, default=10.0)
    ap.add_argument("--scale", type=float, default=1.0)
    ap.add_argument("--clock", choices=["model", "measured"], default="measured")
    args = ap.parse_args(argv)
    layers = []
    for li in range(3):
        spec, W = wl.layer_weights(5, li, scale=args.scale)
        layers.append(cl.compress_layer(W, spec.r, spec.k, 128, 128, upload=True))
    runner = StackRunner(layers)
    batch_set = wl.CONFIGS[5]["batches"]
    plan = runner.plan(batch_set, int(args.budget_mb * 2 ** 20), latency_cap_ms=args.latency_cap_ms)
    if plan is None:
        print(json.dumps({"error": "no feasible plan"}))
        return 1
    arrivals = wl.poisson_arrivals(args.requests, args.rate, wl.BASE_SEED + 5000)
    X = torch.from_numpy(wl.activations(5, args.requests, K=layers[0].K)).cuda()
    _, stats = simulate(runner, plan, arrivals, [X[i] for i in range(args.requests)], args.latency_cap_ms, clock=args.clock)
    stats.update(rate=args.rate, plan=plan.batch_per_layer, plan_ms_per_image=plan.ms_per_image,
                 budget_bytes=plan.tot_bytes, ws_bytes=plan.ws_bytes,
                 time_ms={str(b): [round(float(t), 4) for t in plan.time_ms[:, j]] for j, b in enumerate(plan.batch_set)})
    print(json.dumps(stats))
    return 0


if __name__ == "__main__":
    sys.exit(main())
