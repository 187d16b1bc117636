"""Pins for the CPU oracle: every check here compares the oracle with something
that is NOT the oracle - the paper's worded examples and table values
(tests/golden), closed forms, brute force over tiny inputs written independently
in this file, or a library routine on a special case."""
import heapq
import itertools
import math
import os

import numpy as np
import pytest

import oracle
from oracle import dp as odp

GOLD = os.path.join(os.path.dirname(__file__), "golden")


# --------------------------------------------------------------------------- #
# independent restatements used as pins (pure Python, written from the text)
# --------------------------------------------------------------------------- #
def py_entries_of_sequence(seq, k):
    """Relative-index entries of one flattened block, from the rule in words:
    z zeros precede each stored element; a k-bit field holds at most 2^k - 1, so
    a longer run is broken by stored zeros each preceded by 2^k - 1 zeros."""
    R = 1 << k
    out = []
    run = 0
    for s in seq:
        if s == 0:
            run += 1
            continue
        while run >= R:            # R-1 zeros, then one stored zero = R positions
            out.append((0, R - 1))
            run -= R
        out.append((int(s), run))
        run = 0
    return out


def py_positions(entries):
    pos, p = [], -1
    for v, z in entries:
        p += int(z) + 1
        pos.append(p)
    return pos


def py_blocks(M, K, bh, bw):
    """(row_id, col_id, bh', bw') in the order Algorithm 2 visits them."""
    nbw = -(-K // bw)
    nbh = -(-M // bh)
    for i in range(nbh * nbw):
        row_id, col_id = (i // nbw) * bh, (i % nbw) * bw
        yield row_id, col_id, min(bh, M - row_id), min(bw, K - col_id)


def py_entries(q, bh, bw, k, colmajor=False):
    M, K = q.shape
    val, idx, bp = [], [], [0]
    for row_id, col_id, bhp, bwp in py_blocks(M, K, bh, bw):
        blk = q[row_id:row_id + bhp, col_id:col_id + bwp]
        seq = blk.T.reshape(-1) if colmajor else blk.reshape(-1)
        for v, z in py_entries_of_sequence(seq.tolist(), k):
            val.append(v)
            idx.append(z)
        bp.append(len(val))
    return np.array(val, np.uint8), np.array(idx, np.uint8), np.array(bp, np.int64)


def heap_huffman_cost(counts):
    """Total coded bits of an optimal prefix code = sum of all merged weights."""
    h = [int(c) for c in counts if c > 0]
    if len(h) == 1:
        return h[0]
    heapq.heapify(h)
    cost = 0
    while len(h) > 1:
        a, b = heapq.heappop(h), heapq.heappop(h)
        cost += a + b
        heapq.heappush(h, a + b)
    return cost


def rand_pruned(rng, M, K, d, sigma=0.02):
    W = (rng.standard_normal((M, K)) * sigma).astype(np.float32)
    W[W == 0] = 1e-3
    W *= rng.random((M, K)) < d
    W[W == 0] = 0.0
    return W


# --------------------------------------------------------------------------- #
# the paper's worded examples
# --------------------------------------------------------------------------- #
def _parse_k2_fixture():
    k, cases, row = None, [], None
    for line in open(os.path.join(GOLD, "relative_index_k2_example.txt")):
        t = line.split()
        if not t or t[0].startswith("#"):
            continue
        if t[0] == "k":
            k = int(t[1])
        elif t[0] == "row":
            row = [int(x) for x in t[1:]]
        elif t[0] == "entries":
            cases.append((row, [(x.split(":")[0] == "pad", int(x.split(":")[1])) for x in t[1:]]))
    return k, cases


def test_paper_k2_padding_example():
    k, cases = _parse_k2_fixture()
    assert k == 2
    for row, expect in cases:
        q = np.array([row], np.uint8)
        val, idx, bp = oracle.build_entries(q, 1, len(row), k, colmajor=False)
        got = [(int(v) == 0, int(z)) for v, z in zip(val, idx)]
        assert got == expect
    # the sentence itself: first non-zero beyond column 4 -> a padded zero that
    # stands at the fourth location (0-based position 3)
    q = np.zeros((2, 8), np.uint8)
    q[0, 1] = 1
    q[1, 6] = 2
    val, idx, bp = oracle.build_entries(q, 1, 8, 2, colmajor=False)
    second = slice(bp[1], bp[2])
    assert val[second].tolist() == [0, 2]
    assert py_positions(list(zip(val[second], idx[second])))[0] == 3


def test_paper_8x8_blocking_example():
    """Sec. IV-A: an 8x8 matrix in 4x4 blocks becomes a 4x16 matrix whose row i
    holds block i contiguously; that matrix is then stored as relative-indexed
    CSR.  Algorithm 2's row_id/col_id formulas place block i back."""
    rng = np.random.default_rng(5)
    q = (rng.integers(1, 4, (8, 8)) * (rng.random((8, 8)) < 0.4)).astype(np.uint8)
    relaid = q.reshape(2, 4, 2, 4).transpose(0, 2, 1, 3).reshape(4, 16)   # row i = block i, row-major inside
    val, idx, bp = oracle.build_entries(q, 4, 4, 3, colmajor=False)
    val2, idx2, bp2 = oracle.build_entries(relaid, 1, 16, 3, colmajor=False)   # plain CSR rows of the 4x16
    assert val.tolist() == val2.tolist() and idx.tolist() == idx2.tolist() and bp.tolist() == bp2.tolist()
    a_rows, bw, bh = 8, 4, 4
    for i, (row_id, col_id, _, _) in enumerate(py_blocks(8, 8, 4, 4)):
        assert col_id == (i % (a_rows // bw)) * bw and row_id == (i // (a_rows // bw)) * bh
    cb = np.arange(8, dtype=np.float32)
    Wd = oracle.reconstruct(val, idx, bp, cb, 8, 8, 4, 4, 3, colmajor=False)
    assert np.array_equal(Wd, q.astype(np.float32))


# --------------------------------------------------------------------------- #
# brute force on tiny inputs
# --------------------------------------------------------------------------- #
@pytest.mark.parametrize("k", [1, 2])
def test_bruteforce_all_1x6(k):
    R = 1 << k
    for seq in itertools.product([0, 1, 2], repeat=6):
        q = np.array([seq], np.uint8)
        val, idx, bp = oracle.build_entries(q, 1, 6, k, colmajor=False)
        # entry count by an independent one-liner: nnz + sum floor(gap / 2^k)
        nzpos = [i for i, s in enumerate(seq) if s]
        gaps = [b - a - 1 for a, b in zip([-1] + nzpos[:-1], nzpos)]
        assert len(val) == len(nzpos) + sum(g // R for g in gaps)
        assert list(zip(val.tolist(), idx.tolist())) == py_entries_of_sequence(seq, k)
        assert idx.max(initial=0) < R
        cb = np.array([0, 1.5, -2.5, 0], np.float32)
        Wd = oracle.reconstruct(val, idx, bp, cb, 1, 6, 1, 6, k, colmajor=False)
        assert np.array_equal(Wd[0], cb[list(seq)])


@pytest.mark.parametrize("bh,bw,colmajor", [(3, 3, True), (3, 3, False), (2, 2, True), (1, 3, True), (3, 1, True), (2, 3, False)])
def test_bruteforce_all_3x3_binary(bh, bw, colmajor):
    cb = np.array([0, 2.0], np.float32)
    for bits in range(512):
        q = np.array([(bits >> i) & 1 for i in range(9)], np.uint8).reshape(3, 3)
        val, idx, bp = oracle.build_entries(q, bh, bw, 1, colmajor)
        pv, pi, pb = py_entries(q, bh, bw, 1, colmajor)
        assert val.tolist() == pv.tolist() and idx.tolist() == pi.tolist() and bp.tolist() == pb.tolist()
        Wd = oracle.reconstruct(val, idx, bp, cb, 3, 3, bh, bw, 1, colmajor)
        assert np.array_equal(Wd, 2.0 * q)


# --------------------------------------------------------------------------- #
# round trips and mask invariants over the parameter space
# --------------------------------------------------------------------------- #
SHAPES = [(1, 1, 1, 1), (1, 37, 1, 37), (40, 1, 40, 1), (64, 48, 64, 1), (64, 48, 16, 16),
          (100, 70, 32, 24), (33, 129, 128, 128), (50, 50, 7, 50)]


@pytest.mark.parametrize("M,K,bh,bw", SHAPES)
@pytest.mark.parametrize("d", [0.0, 0.004, 0.09, 0.25, 0.84, 1.0])
def test_round_trip_and_mask(M, K, bh, bw, d):
    rng = np.random.default_rng(M * 1000 + K + int(d * 100))
    for r, k in [(5, 4), (8, 8), (1, 1), (3, 2), (5, 5)]:
        W = rand_pruned(rng, M, K, d)
        if d == 0.004 and not W.any():
            W[M // 2, K // 2] = 0.01          # "one entry" case
        m = oracle.compress_layer(W, r, k, bh, bw, keep=True)
        val, idx, bp = oracle.decode_layer(m)
        assert np.array_equal(val, m.extra["val"]) and np.array_equal(idx, m.extra["idx"])
        assert np.array_equal(bp, m.extra["block_ptr"])
        v2, i2 = oracle.decode_layer_whole(m)
        assert np.array_equal(v2, val) and np.array_equal(i2, idx)
        # independent entry builder
        pv, pi, pb = py_entries(m.extra["q"], bh, bw, k)
        assert np.array_equal(pv, val) and np.array_equal(pi, idx) and np.array_equal(pb, bp)
        # mask invariants
        assert int((val != 0).sum()) == int((W != 0).sum())
        Wd, qd = oracle.reconstruct(val, idx, bp, m.codebook, M, K, bh, bw, k, want_q=True)
        assert np.array_equal(qd, m.extra["q"])
        assert np.array_equal(Wd != 0, (m.codebook[m.extra["q"]] != 0))
        assert np.array_equal((qd != 0), (W != 0))
        for b, (row_id, col_id, bhp, bwp) in enumerate(py_blocks(M, K, bh, bw)):
            e = list(zip(val[bp[b]:bp[b + 1]].tolist(), idx[bp[b]:bp[b + 1]].tolist()))
            pos = [p for p, (v, z) in zip(py_positions(e), e) if v]
            mask = (W[row_id:row_id + bhp, col_id:col_id + bwp] != 0).reshape(-1)
            assert pos == np.flatnonzero(mask).tolist()
        # quantisation error bound of a linear codebook: half a step
        if W.any() and r > 1:
            nzv = W[W != 0]
            step = (float(nzv.max()) - float(nzv.min())) / ((1 << r) - 2)
            assert np.abs(Wd - W).max() <= step / 2 * (1 + 1e-5) + 1e-12


def test_csc_block_ptr_is_column_pointer():
    rng = np.random.default_rng(11)
    W = rand_pruned(rng, 200, 30, 0.1)
    m = oracle.compress_layer(W, 5, 4, 200, 1, keep=True)
    bp = m.extra["block_ptr"]
    R = 16
    for j in range(30):
        nz = np.flatnonzero(W[:, j])
        gaps = np.diff(np.concatenate([[-1], nz])) - 1
        assert bp[j + 1] - bp[j] == len(nz) + int((gaps // R).sum())


# --------------------------------------------------------------------------- #
# quantisation
# --------------------------------------------------------------------------- #
def test_quantize_against_numpy_argmin():
    rng = np.random.default_rng(3)
    W = rand_pruned(rng, 60, 70, 0.5)
    for r in (1, 2, 5, 8):
        cb = oracle.linear_codebook(W, r)
        n = (1 << r) - 1
        nz = W[W != 0].astype(np.float64)
        assert cb[0] == 0 and cb.size == n + 1
        if n > 1:
            assert cb[1] == np.float32(nz.min()) and cb[n] == np.float32(nz.max())
            assert np.allclose(np.diff(cb[1:].astype(np.float64)), (nz.max() - nz.min()) / (n - 1), rtol=1e-4)
        q = oracle.quantize(W, r, cb)
        d = np.abs(W.astype(np.float64)[..., None] - cb[1:].astype(np.float64))
        ref = np.where(W != 0, d.argmin(-1) + 1, 0)     # argmin returns the first (lowest) minimiser
        assert np.array_equal(q, ref)


def test_quantize_ties_and_supplied_codebook():
    cb = np.array([0, -1.0, 1.0, 3.0], np.float32)
    W = np.array([[0.0, 0.0, 2.0, -5.0, 1e-30, 1.0]], np.float32)
    W[0, 0] = 0.0
    q = oracle.quantize(W, 2, cb)
    # 2.0 is equidistant from 1.0 and 3.0 -> lower index; tiny non-zero is equidistant from -1, 1 -> index 1
    assert q.tolist() == [[0, 0, 2, 1, 1, 2]]
    with pytest.raises(oracle.OracleError):
        oracle.quantize(np.array([np.nan], np.float32), 2, cb)


# --------------------------------------------------------------------------- #
# Huffman
# --------------------------------------------------------------------------- #
@pytest.mark.parametrize("seed", range(12))
def test_huffman_invariants(seed):
    rng = np.random.default_rng(seed)
    nsym = int(rng.integers(1, 40))
    kind = seed % 4
    if kind == 0:
        counts = rng.integers(0, 50, nsym)
    elif kind == 1:
        counts = (1000 * 0.5 ** np.arange(nsym)).astype(np.int64)          # geometric
    elif kind == 2:
        counts = np.array([int(1.6180339 ** i) + 1 for i in range(nsym)])   # Fibonacci-like: deep tree
    else:
        counts = np.ones(nsym, np.int64) * 7
    counts = np.asarray(counts, np.int64)
    if not counts.any():
        counts[0] = 3
    ln, code = oracle.huffman_code(counts)
    used = counts > 0
    assert (ln[~used] == 0).all() and (ln[used] > 0).all()
    total = int((counts * ln).sum())
    if used.sum() == 1:
        assert ln[used][0] == 1
    else:
        assert sum(2.0 ** -int(l) for l in ln[used]) == 1.0                 # Kraft equality
        assert total == heap_huffman_cost(counts)                            # optimal cost
        p = counts[used] / counts.sum()
        H = float(-(p * np.log2(p)).sum())
        assert H - 1e-9 <= total / counts.sum() < H + 1
    # prefix-freeness, checked here bit by bit on the strings
    words = ["".join(str((int(code[s]) >> j) & 1) for j in range(ln[s])) for s in np.flatnonzero(used)]
    for a, b in itertools.permutations(words, 2):
        assert not b.startswith(a)
    # encode / bit-serial decode
    sym = rng.choice(np.flatnonzero(used), size=300).astype(np.uint8)
    buf, nbits = oracle.huffman_encode(sym, ln, code)
    assert nbits == int(ln[sym].sum())
    # stream convention: bit b = bit (b mod 8) of byte b // 8, codeword bits in walk order
    bits = "".join(words[list(np.flatnonzero(used)).index(s)] for s in sym)
    got = "".join(str((buf[b >> 3] >> (b & 7)) & 1) for b in range(nbits))
    assert got == bits
    out, end, pos = oracle.huffman_decode_serial(buf, nbits, 0, sym.size, ln, code, want_bitpos=True)
    assert np.array_equal(out, sym) and end == nbits
    assert np.array_equal(pos, np.concatenate([[0], np.cumsum(ln[sym])[:-1]]))
    assert np.array_equal(oracle.huffman_decode_span(buf, 0, nbits, ln, code), sym)


def test_huffman_decoder_rejects_bad_input():
    ln = np.array([1, 2, 2], np.uint8)
    code = np.array([0, 1, 3], np.uint64)           # 0, 10, 11
    buf, nbits = oracle.huffman_encode(np.array([0, 1, 2, 0], np.uint8), ln, code)
    with pytest.raises(oracle.OracleError):          # truncated
        oracle.huffman_decode_serial(buf, nbits - 1, 0, 4, ln, code)
    with pytest.raises(oracle.OracleError):          # not a prefix code: 0 and 01
        oracle.huffman_decode_serial(buf, nbits, 0, 1, np.array([1, 2], np.uint8), np.array([0, 2], np.uint64))
    with pytest.raises(oracle.OracleError):          # incomplete code, walk leaves the tree
        oracle.huffman_decode_serial(np.array([0xFF], np.uint8), 8, 0, 1, np.array([2, 2], np.uint8), np.array([0, 2], np.uint64))
    with pytest.raises(oracle.OracleError):          # codeword straddles the span end
        oracle.huffman_decode_span(np.array([0xFF], np.uint8), 0, 3, ln, code)


# --------------------------------------------------------------------------- #
# product: Eq. (1)-(2) against library routines and special cases
# --------------------------------------------------------------------------- #
def test_fc_forward_vs_numpy_and_scipy():
    import scipy.sparse as sp
    rng = np.random.default_rng(21)
    M, K, B = 70, 130, 5
    W = rand_pruned(rng, M, K, 0.15)
    X = np.maximum(rng.standard_normal((B, K)), 0).astype(np.float32)
    bias = rng.standard_normal(M).astype(np.float32)
    Y = oracle.fc_forward(W, X, bias, relu=False)
    ref = X.astype(np.float64) @ W.astype(np.float64).T + bias.astype(np.float64)
    assert Y.shape == (B, M)
    assert np.allclose(Y, ref, rtol=1e-13, atol=1e-15)
    Ysp = (sp.csr_matrix(W.astype(np.float64)) @ X.astype(np.float64).T).T + bias
    assert np.allclose(Y, Ysp, rtol=1e-13, atol=1e-15)
    assert np.array_equal(oracle.fc_forward(W, X, bias, relu=True), np.maximum(Y, 0))
    assert np.array_equal(oracle.fc_forward(W, X, bias, nthreads=4), Y)
    # a transposed operand or a dropped bias cannot pass: M != K and bias != 0
    assert not np.allclose(Y, X.astype(np.float64) @ W.astype(np.float64).T)


def test_dense_full_density_reduces_to_gemm():
    """Density 100 % and a codebook that contains every weight exactly: the
    compressed layer must behave as the plain dense layer."""
    rng = np.random.default_rng(8)
    levels = np.array([0] + [(-1) ** t * (0.125 * t) for t in range(1, 32)], np.float32)
    q = rng.integers(1, 32, (24, 40))
    W = levels[q]
    for bh, bw in [(24, 1), (8, 16), (24, 40)]:
        m = oracle.compress_layer(W, 5, 4, bh, bw, codebook=levels)
        assert m.n_entries == W.size                      # no padding entries at full density
        assert np.array_equal(oracle.dense_weights(m), W)
        X = rng.standard_normal((3, 40)).astype(np.float32)
        assert np.allclose(oracle.compressed_fc_forward(m, X), X.astype(np.float64) @ W.astype(np.float64).T, rtol=1e-13)


def test_sparse_accumulation_over_entries_equals_dense():
    """Summing w * x over the decoded entries (the order Algorithm 1 would feed a
    sparse multiply) equals the dense definition."""
    rng = np.random.default_rng(9)
    M, K = 50, 64
    W = rand_pruned(rng, M, K, 0.1)
    m = oracle.compress_layer(W, 5, 4, 16, 16)
    val, idx, bp = oracle.decode_layer(m)
    x = rng.standard_normal(K).astype(np.float32)
    y = np.zeros(M)
    for b, (row_id, col_id, bhp, bwp) in enumerate(py_blocks(M, K, 16, 16)):
        e = list(zip(val[bp[b]:bp[b + 1]].tolist(), idx[bp[b]:bp[b + 1]].tolist()))
        for (v, z), p in zip(e, py_positions(e)):
            if v:
                y[row_id + p // bwp] += float(m.codebook[v]) * float(x[col_id + p % bwp])
    assert np.allclose(y, oracle.compressed_fc_forward(m, x[None])[0], rtol=1e-12, atol=1e-15)


def test_conv_forward_vs_torch():
    import torch
    import torch.nn.functional as F
    rng = np.random.default_rng(4)
    for (C, H, Wd, R, S, stride, pad, groups, OC) in [(3, 19, 19, 5, 5, 4, 0, 1, 6), (4, 9, 11, 3, 3, 1, 1, 2, 6), (6, 7, 7, 3, 3, 2, 2, 3, 9)]:
        geom = dict(C=C, H=H, W=Wd, R=R, S=S, stride=stride, pad=pad, groups=groups, OC=OC)
        Wt = rng.standard_normal((OC, C // groups * R * S)).astype(np.float32)
        X = rng.standard_normal((2, C, H, Wd)).astype(np.float32)
        bias = rng.standard_normal(OC).astype(np.float32)
        Y = oracle.conv_forward(Wt, X, geom, bias, relu=True)
        ref = F.relu(F.conv2d(torch.from_numpy(X).double(), torch.from_numpy(Wt).double().reshape(OC, C // groups, R, S),
                              torch.from_numpy(bias).double(), stride=stride, padding=pad, groups=groups)).numpy()
        assert Y.shape == ref.shape
        assert np.allclose(Y, ref, rtol=1e-12, atol=1e-13)


def test_alexnet_conv_geometry_matches_table4():
    """Table IV's memory column is batch * output elements * 4 bytes; that pins
    the conv output sizes (55^2*96, 27^2*256, 13^2*384, 13^2*384, 13^2*256) and
    the FC widths used by the workloads."""
    import importlib
    wl = importlib.import_module("paper_1711_00244_amd.workloads")
    table = {}
    for line in open(os.path.join(GOLD, "table4_alexnet_memory_mb.txt")):
        t = line.split()
        if t and not t[0].startswith("#"):
            table[t[0]] = (float(t[1]), float(t[2]))
    for spec in wl.CONFIGS[4]["layers"]:
        g = spec.conv
        P = (g["H"] + 2 * g["pad"] - g["R"]) // g["stride"] + 1
        elems = P * P * g["OC"]
        # conv2's and conv5's rows of the table are those of the following pool
        # input; the table lists the conv output itself
        for col, B in enumerate((16, 256)):
            assert abs(B * elems * 4 / 2 ** 20 - table[spec.name][col]) < 0.006
        assert spec.K == g["C"] // g["groups"] * g["R"] * g["S"] and spec.M == g["OC"]
    for spec in wl.CONFIGS[3]["layers"]:
        for col, B in enumerate((16, 256)):
            assert abs(B * spec.M * 4 / 2 ** 20 - table[spec.name][col]) < 0.006


# --------------------------------------------------------------------------- #
# statistics of the format on the benchmark's distributions (closed forms)
# --------------------------------------------------------------------------- #
@pytest.mark.parametrize("d,k,expect", [(0.10, 4, 0.2275), (0.09, 4, 0.2838), (0.25, 4, 0.0101), (0.04, 5, 0.3714)])
def test_padding_rate_closed_form(d, k, expect):
    """A gap before a non-zero is geometric; the expected number of padding
    entries per non-zero is q^R / (1 - q^R), q = 1 - d, R = 2^k."""
    qv, R = 1 - d, 1 << k
    assert abs(qv ** R / (1 - qv ** R) - expect) < 5e-4
    rng = np.random.default_rng(int(d * 1000) + k)
    W = rand_pruned(rng, 1 << 20, 1, d)          # one long column: no block boundary resets the gap
    m = oracle.compress_layer(W, 5, k, 1 << 20, 1)
    nnz = int((W != 0).sum())
    assert abs((m.n_entries - nnz) / nnz - expect) < 0.03 * max(expect, 0.05)


# --------------------------------------------------------------------------- #
# dynamic program
# --------------------------------------------------------------------------- #
def brute_force_plan(time_ms, bs, inb, outb, ws, tot, step, cap):
    """Every monotone divisor chain, cost by simulating the phases: to run layer
    i once at batch B, the earlier layers run B/b times at batch b."""
    f = len(time_ms)
    best, arg = float("inf"), None

    def run_cost(i, chain):          # time to push chain[i] images through layers 0..i
        t = time_ms[i][bs.index(chain[i])]
        if i == 0:
            return t
        return t + (chain[i] // chain[i - 1]) * run_cost(i - 1, chain)

    for chain in itertools.product(bs, repeat=f):
        if any(chain[i] > chain[i + 1] or chain[i + 1] % chain[i] for i in range(f - 1)):
            continue
        # memory: while layer i waits for its B inputs, (B - b) of them are parked
        reserved, ok = 0, True
        for i in range(f - 1, -1, -1):
            B = chain[i]
            if reserved + B * inb[i] + ws[i] + B * outb[i] > tot:
                ok = False
                break
            if i:
                reserved = -(-(reserved + (B - chain[i - 1]) * inb[i]) // step) * step
        if not ok:
            continue
        if cap is not None and any(run_cost(i, chain) > cap for i in range(f)):
            continue
        c = run_cost(f - 1, chain) / chain[-1]
        if c < best:
            best, arg = c, list(chain)
    return best, arg


@pytest.mark.parametrize("seed", range(30))
def test_dp_equals_brute_force(seed):
    rng = np.random.default_rng(seed)
    f = int(rng.integers(1, 5))
    bs = [1, 2, 4, 8] if seed % 2 else [1, 2, 3, 6, 12]
    # sub-linear times so that batching pays
    time_ms = [[float(rng.uniform(0.5, 2.0) * (1 + 0.3 * b ** rng.uniform(0.5, 1.0))) for b in bs] for _ in range(f)]
    inb = [int(rng.integers(1, 40)) * 100 for _ in range(f)]
    outb = inb[1:] + [int(rng.integers(1, 40)) * 100]
    ws = [int(rng.integers(0, 30)) * 100 for _ in range(f)]
    tot = int(rng.integers(20, 400)) * 100
    step = int(rng.choice([100, 700, 1]))
    cap = None if seed % 3 else float(rng.uniform(3, 30))
    got, plan = odp.plan_batches(time_ms, bs, inb, outb, ws, tot, step, cap)
    ref, rplan = brute_force_plan(time_ms, bs, inb, outb, ws, tot, step, cap)
    if rplan is None:
        assert plan is None and math.isinf(got)
    else:
        assert got == pytest.approx(ref, rel=1e-12)
        assert all(a <= b and b % a == 0 for a, b in zip(plan, plan[1:]))     # monotone divisor chain


def test_dp_unbounded_memory_picks_largest_batch():
    bs = [1, 2, 4, 8, 16]
    time_ms = [[1.0 + 0.1 * b for b in bs] for _ in range(3)]               # Time(i,B)/B decreasing
    got, plan = odp.plan_batches(time_ms, bs, [4] * 3, [4] * 3, [0] * 3, 10 ** 12, 100, None)
    assert plan == [16, 16, 16] and got == pytest.approx(3 * (1.0 + 1.6) / 16)
    fb, B = odp.fixed_batch_baseline(time_ms, bs, [4] * 3, [4] * 3, [0] * 3, 10 ** 12, None)
    assert B == 16 and fb == pytest.approx(got)


def test_dp_beats_fixed_batch_when_early_layers_are_memory_hungry():
    """The paper's motivating case: big activations early (conv-like), small ones
    late (FC-like).  Variable batching may use a large batch late."""
    bs = [1, 2, 4, 8, 16, 32, 64]
    time_ms = [[5.0 * b for b in bs], [2.0 + 0.05 * b for b in bs]]          # layer 2 batches very well
    inb, outb, ws = [600_000, 40_000], [40_000, 16_000], [0, 50_000]
    tot = 4_000_000
    fb, B = odp.fixed_batch_baseline(time_ms, bs, inb, outb, ws, tot, None)
    got, plan = odp.plan_batches(time_ms, bs, inb, outb, ws, tot, 100_000, None)
    assert B == 4 and plan[0] <= 4 and plan[1] > 4 and got < fb


# --------------------------------------------------------------------------- #
# the fixed-function layers of the whole-network runs (Table IV: norm, pool)
# --------------------------------------------------------------------------- #
def test_maxpool_against_window_enumeration_and_closed_forms():
    rng = np.random.default_rng(41)
    X = rng.standard_normal((2, 5, 11, 9)).astype(np.float32)
    for size, stride in [(3, 2), (2, 2), (1, 1), (3, 1), (11 if False else 5, 3)]:
        Y = oracle.maxpool_forward(X, size, stride)
        P, Q = (11 - size) // stride + 1, (9 - size) // stride + 1
        assert Y.shape == (2, 5, P, Q)
        for p in range(P):
            for q in range(Q):
                win = X[:, :, p * stride:p * stride + size, q * stride:q * stride + size]
                assert np.array_equal(Y[:, :, p, q], win.reshape(2, 5, -1).max(-1).astype(np.float64))
    assert np.array_equal(oracle.maxpool_forward(X, 1, 1), X.astype(np.float64))        # 1 x 1 windows: identity
    ramp = np.arange(7 * 7, dtype=np.float32).reshape(1, 1, 7, 7)                       # increasing along both axes:
    Y = oracle.maxpool_forward(ramp, 3, 2)                                              # the maximum is the window's last corner
    assert np.array_equal(Y[0, 0], ramp[0, 0, 2::2, 2::2].astype(np.float64))
    assert np.array_equal(oracle.maxpool_forward(-np.ones((1, 2, 4, 4), np.float32), 2, 2), -np.ones((1, 2, 2, 2)))   # negatives survive


def test_lrn_closed_forms():
    rng = np.random.default_rng(42)
    X = rng.standard_normal((2, 9, 3, 4)).astype(np.float32)
    x64 = X.astype(np.float64)
    # a window of one channel: y = x / (k + alpha x^2)^beta
    assert np.allclose(oracle.lrn_forward(X, 1, 0.3, 0.75, 2.0), x64 / (2.0 + 0.3 * x64 ** 2) ** 0.75, rtol=1e-14, atol=0)
    # alpha = 0: y = x / k^beta
    assert np.allclose(oracle.lrn_forward(X, 5, 0.0, 0.75, 2.0), x64 / 2.0 ** 0.75, rtol=1e-14, atol=0)
    # constant input: interior channels see n terms, the outermost ones (n + 1) / 2
    c = np.full((1, 9, 2, 2), 3.0, np.float32)
    Y = oracle.lrn_forward(c, 5, 0.5, 0.75, 1.0)
    assert np.allclose(Y[0, 4], 3.0 / (1.0 + 0.5 / 5 * 5 * 9.0) ** 0.75, rtol=1e-14)
    assert np.allclose(Y[0, 0], 3.0 / (1.0 + 0.5 / 5 * 3 * 9.0) ** 0.75, rtol=1e-14)
    assert np.allclose(Y[0, 1], 3.0 / (1.0 + 0.5 / 5 * 4 * 9.0) ** 0.75, rtol=1e-14)
    # channel windows by enumeration, n = 3 and 5
    for n in (3, 5):
        Y = oracle.lrn_forward(X, n, 1e-1, 0.75, 1.0)
        for ch in range(9):
            lo, hi = max(0, ch - n // 2), min(9, ch + n // 2 + 1)
            ss = (x64[:, lo:hi] ** 2).sum(1)
            assert np.allclose(Y[:, ch], x64[:, ch] / (1.0 + 0.1 / n * ss) ** 0.75, rtol=1e-13, atol=0)
    with pytest.raises(oracle.OracleError):
        oracle.lrn_forward(X, 4)                                                         # even windows have no centre
