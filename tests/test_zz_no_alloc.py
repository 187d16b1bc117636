"""The entry point that allocates nothing (scratch in the library's static device
array) against the entry point it is a variant of, through the C ABI: two calls in a
row, the second with a smaller input, on the run-to-run identical dense-tile path (bit
for bit) and on the sparse path (whose own results differ in the last bits from call
to call: both within the gates of the oracle, and of each other within 1e-5)."""
import numpy as np
import pytest

import oracle
import paper_1711_00244_amd as cl
from paper_1711_00244_amd import binding
from gates import TOL, assert_close, fc_ref

pytestmark = pytest.mark.gpu


def _layer(rng, M, K, d):
    W = (rng.standard_normal((M, K)) * 0.02).astype(np.float32)
    W *= rng.random((M, K)) < d
    W[W == 0] = 0.0
    L = cl.compress_layer(W, 5, 4, 128, 128, upload=True)
    return L, oracle.dense_weights(oracle.compress_layer(W, 5, 4, 128, 128))


def test_static_scratch_entry_point_matches_the_workspace_one():
    import torch
    assert torch.cuda.is_available()
    rng = np.random.default_rng(31)
    big, big_W = _layer(rng, 700, 900, 0.1)
    small, small_W = _layer(rng, 130, 260, 0.2)
    for path, exact in ((cl.PATH_MFMA_F32, True), (cl.PATH_SPARSE, False)):
        # the larger call first, then a smaller one into the same static scratch
        for L, oW, B in ((big, big_W, 48 if exact else 4), (small, small_W, 7 if exact else 2)):
            X = np.maximum(rng.standard_normal((B, L.K)), 0).astype(np.float32)
            bias = (rng.standard_normal(L.M) * 0.1).astype(np.float32)
            Xd, bd = torch.from_numpy(X).cuda(), torch.from_numpy(bias).cuda()
            want = cl.compressed_fc_forward(L, Xd, bd, relu=True, path=path)
            out = torch.full((B, L.M), -7.0, device="cuda")
            got = cl.compressed_fc_forward_static(L, Xd, out, bd, relu=True, path=path)
            torch.cuda.synchronize()
            assert got.data_ptr() == out.data_ptr()
            ref = fc_ref(oW, X, bias)
            assert_close(got.cpu().numpy(), ref, True)
            assert_close(want.cpu().numpy(), ref, True)
            if exact:
                assert torch.equal(got, want), (path, B)
            else:
                scale = float(np.abs(ref.pre).max())
                assert float((got - want).abs().max()) <= TOL * scale, (path, B)
    # a call whose scratch exceeds the static area is refused, nothing is launched
    B = 4096
    assert cl.fc_workspace_bytes(big, B, cl.PATH_MFMA_F32) > cl.STATIC_SCRATCH_BYTES
    out = torch.full((B, big.M), -7.0, device="cuda")
    with pytest.raises(cl.CLError) as e:
        cl.compressed_fc_forward_static(big, torch.zeros((B, big.K), device="cuda"), out, path=cl.PATH_MFMA_F32)
    assert e.value.code == binding.CL_EUNSUPPORTED
    torch.cuda.synchronize()
    assert bool((out == -7.0).all())
    big.free()
    small.free()
