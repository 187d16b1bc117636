"""Variable batch sizes and the request scheduler on the GPU (configs[4] shape,
scaled down so that the oracle side stays quick)."""
import numpy as np
import pytest

import oracle
import paper_1711_00244_amd as cl
from paper_1711_00244_amd import scheduler, workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def vgg_stack():
    import torch
    assert torch.cuda.is_available()
    layers, dense = [], []
    K = None
    for li in range(3):
        spec, W = wl.layer_weights(5, li, scale=0.125)
        if K is not None and W.shape[1] != K:           # chain the scaled shapes: inputs of layer i = outputs of layer i-1
            W = wl.pruned_weights(W.shape[0], K, spec.density, spec.sigma, 7 + li)
        K = W.shape[0]
        layers.append(cl.compress_layer(W, spec.r, spec.k, 128, 128, upload=True))
        dense.append(oracle.dense_weights(oracle.compress_layer(W, spec.r, spec.k, 128, 128)))
    return layers, dense


def oracle_stack(dense, X):
    a = X
    for li, W in enumerate(dense):
        y = oracle.fc_forward(W, a, relu=(li + 1 < len(dense)), nthreads=8)
        a = y.astype(np.float32)
    return y


def test_variable_batch_run_matches_oracle(vgg_stack):
    import torch
    layers, dense = vgg_stack
    runner = scheduler.StackRunner(layers)
    X = wl.activations(5, 48, K=layers[0].K)
    ref = oracle_stack(dense, X)
    Xd = torch.from_numpy(X).cuda()
    for bpl in (None, [4, 8, 16], [1, 1, 16], [16, 16, 16], [2, 4, 4]):
        Y = runner.run(Xd, bpl).cpu().numpy()
        # activations pass through fp32 between layers on both sides; allow the chain a little more room
        assert np.abs(Y - ref).max() / np.abs(ref).max() <= 3e-5, bpl


def test_plan_and_poisson_stream(vgg_stack):
    import torch
    layers, dense = vgg_stack
    runner = scheduler.StackRunner(layers)
    batch_set = [1, 2, 4, 8, 16, 32, 64]
    times = runner.measure_times(batch_set, reps=5, warmup=2)
    assert times.shape == (3, len(batch_set)) and (times > 0).all()
    budget = 64 << 20
    plan = runner.plan(batch_set, budget, latency_cap_ms=10.0, time_ms=times)
    assert plan is not None
    bpl = plan.batch_per_layer
    assert all(a <= b and b % a == 0 for a, b in zip(bpl, bpl[1:]))
    # the plan respects the budget: activations in/out of the largest layer call plus its scratch
    for li, L in enumerate(layers):
        assert bpl[li] * (L.K + L.M) * 4 + plan.ws_bytes[li] <= budget
    # an impossible budget yields no plan
    assert runner.plan(batch_set, 1024, latency_cap_ms=10.0, time_ms=times) is None
    # a latency cap below the fastest single image yields no plan either
    assert runner.plan(batch_set, budget, latency_cap_ms=1e-6, time_ms=times) is None

    n = 256
    arrivals = wl.poisson_arrivals(n, 20000.0, 99)
    X = wl.activations(5, n, K=layers[0].K)
    Xd = torch.from_numpy(X).cuda()
    outs, stats = scheduler.simulate(runner, plan, arrivals, [Xd[i] for i in range(n)], 10.0)
    assert stats["requests"] == n and stats["over_cap"] == 0 and stats["max_ms"] <= 10.0
    assert 1 <= stats["mean_batch"] <= bpl[-1]
    Y = torch.stack(outs, 0).cpu().numpy()
    ref = oracle_stack(dense, X)
    assert np.abs(Y - ref).max() / np.abs(ref).max() <= 3e-5


def test_config5_full_size_plan_and_stream():
    """configs[4] at full size: the VGG-16 FC stack (fc6 is 4096 x 25088) planned over
    the batch sizes 1..256 under the 64 MB decoded-buffer / activation budget and the
    10 ms latency cap, then one seeded Poisson stream of 256 single-image requests
    served with that plan, the clock advancing by the measured duration of every
    dispatch.  Outputs of sampled requests against the oracle's chain on its own decode
    (layer by layer in fp64, activations handed on in fp32 as the device does)."""
    import torch
    layers, dense = [], []
    for li in range(3):
        spec, W = wl.layer_weights(5, li)
        layers.append(cl.compress_layer(W, spec.r, spec.k, 128, 128, upload=True))
        dense.append(oracle.dense_weights(oracle.compress_layer(W, spec.r, spec.k, 128, 128)))
        del W
    runner = scheduler.StackRunner(layers)
    batch_set = wl.CONFIGS[5]["batches"]
    assert batch_set[0] == 1 and batch_set[-1] == 256
    budget, cap = 64 << 20, 10.0
    plan = runner.plan(batch_set, budget, latency_cap_ms=cap)
    assert plan is not None
    bpl = plan.batch_per_layer
    assert all(a <= b and b % a == 0 for a, b in zip(bpl, bpl[1:]))
    for li, L in enumerate(layers):
        assert bpl[li] * (L.K + L.M) * 4 + plan.ws_bytes[li] <= budget
    assert abs(plan.dispatch_ms(bpl) / bpl[-1] - plan.ms_per_image) <= 1e-9 * plan.ms_per_image
    assert plan.dispatch_ms(bpl) <= cap
    n = 256
    arrivals = wl.poisson_arrivals(n, 20000.0, wl.BASE_SEED + 5000)
    X = wl.activations(5, n, K=layers[0].K)
    Xd = torch.from_numpy(X).cuda()
    outs, stats = scheduler.simulate(runner, plan, arrivals, [Xd[i] for i in range(n)], cap, clock="measured")
    print({k: (round(v, 3) if isinstance(v, float) else v) for k, v in stats.items()}, "plan", bpl, end=" ")
    assert stats["requests"] == n and stats["over_cap"] == 0 and stats["max_ms"] <= cap
    assert 1 <= stats["mean_batch"] <= bpl[-1]
    Y = torch.stack(outs, 0).cpu().numpy()
    sample = np.sort(np.random.default_rng(5).choice(n, size=12, replace=False))
    ref = oracle_stack(dense, X[sample])
    assert np.abs(Y[sample] - ref).max() / np.abs(ref).max() <= 3e-5
    for L in layers:
        L.free()


def test_alexnet_whole_network_with_per_layer_batches():
    """The thirteen layers of Table IV end to end on the device with per-layer batch
    sizes (small early, larger late, as in Table V), against the oracle's chain of
    direct convolutions, normalisations, poolings and dense products in fp64 on its
    own decode of the same compressed layers.  Eight layers with arithmetic compound
    their 1e-5 each, so the logits are held to 2e-4 of their largest magnitude."""
    import torch
    from paper_1711_00244_amd import network
    net = network.alexnet()
    K = 4
    rng = np.random.default_rng(77)
    X = rng.random((K, 3, 227, 227), dtype=np.float32)
    Y = net.run(torch.from_numpy(X).cuda(), [1, 1, 1, 2, 2, 2, 2, 2, 2, 4, 4, 4, 4]).cpu().numpy()
    Y1 = net.run(torch.from_numpy(X).cuda(), None).cpu().numpy()
    a = X
    for op in net.layers:
        if isinstance(op, network.ConvOp) or isinstance(op, network.FcOp):
            cfg, names = (4, [s.name for s in wl.CONFIGS[4]["layers"]]) if isinstance(op, network.ConvOp) else (3, ["fc6", "fc7", "fc8"])
            spec, W = wl.layer_weights(cfg, names.index(op.name))
            m = oracle.compress_layer(W, spec.r, spec.k, op.block[0], op.block[1])
            oW = oracle.dense_weights(m)
            if isinstance(op, network.ConvOp):
                a = oracle.conv_forward(oW, a.astype(np.float32), op.geom, relu=True, nthreads=8)
            else:
                a = oracle.fc_forward(oW, a.reshape(K, -1).astype(np.float32), relu=op.relu, nthreads=8)
        elif isinstance(op, network.LrnOp):
            a = oracle.lrn_forward(a.astype(np.float32), *op.args)
        else:
            a = oracle.maxpool_forward(a.astype(np.float32), op.size, op.stride)
    scale = np.abs(a).max()
    assert np.abs(Y - a).max() <= 2e-4 * scale
    assert np.abs(Y1 - a).max() <= 2e-4 * scale
    for op in net.layers:
        if hasattr(op, "layer"):
            op.layer.free()
