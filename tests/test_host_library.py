"""CPU-only tests of the library's host side: the C ABI loads and exports what the
header declares, the compressor's output is decoded by the ORACLE's bit-serial
decoder into the oracle's own entries, every table field is re-derived from that
serial walk, error paths, serialisation, and the batch planner against the
oracle's dynamic program.  No kernels run here."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import oracle
from oracle import dp as odp
import paper_1711_00244_amd as cl
from paper_1711_00244_amd import binding, workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def rand_pruned(rng, M, K, d, sigma=0.02):
    W = (rng.standard_normal((M, K)) * sigma).astype(np.float32)
    W[W == 0] = 1e-3
    W *= rng.random((M, K)) < d
    W[W == 0] = 0.0
    return W


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "compressed_layer.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(cl_[a-z_]+)\s*\(", hdr))
    assert declared == set(binding.EXPORTS)
    lib = C.CDLL(binding.library_path())
    for name in declared:
        assert hasattr(lib, name), name


def cross_decode(layer):
    """Decode the library's records with the oracle's bit-serial tree walk and
    re-derive every table field from the walk.  -> (val, idx, block_ptr)."""
    hv = layer.host_view()
    meta, records = hv["chunk_meta"], hv["records"]
    vlen, vcode = hv["val_len"], hv["val_code"].astype(np.uint64)
    ilen, icode = hv["idx_len"], hv["idx_code"].astype(np.uint64)
    bp = hv["block_ptr"].astype(np.int64)
    d = hv["desc"]
    nbw = -(-d["K"] // d["block_w"])
    vals, idxs = [], []
    n_seen, carry, cur_blk = 0, 0, -1
    assert int(meta[-1]["rec_off"]) == records.size and int(meta[-1]["sym_off"]) == hv["n_entries"]
    for c in range(hv["n_chunks"]):
        m = meta[c]
        r0, r1 = int(m["rec_off"]), int(meta[c + 1]["rec_off"])
        assert 1 <= r1 - r0 <= binding.RECORDS_PER_CHUNK
        blk = int(m["blk"])
        if blk != cur_blk:                       # a new block starts: its first chunk, carry back to 0
            assert int(m["sym_off"]) == bp[blk]
            cur_blk, carry = blk, 0
        assert int(m["sym_off"]) == n_seen and int(m["pos0"]) == carry
        panel = blk // nbw
        assert hv["panel_chunk"][panel] <= c < hv["panel_chunk"][panel + 1]
        for r in range(r0, r1):
            w = int(records[r])
            n = w & 15
            assert 1 <= n <= binding.MAX_RECORD_ENTRIES
            fwd = np.frombuffer(w.to_bytes(8, "little"), np.uint8)
            # the relative-index span is read from bit 63 downwards: reverse the 64 bits
            rw = int(format(w, "064b")[::-1], 2)
            rev = np.frombuffer(rw.to_bytes(8, "little"), np.uint8)
            v, vend = oracle.huffman_decode_serial(fwd, 64, 4, n, vlen, vcode)
            z, zend = oracle.huffman_decode_serial(rev, 64, 0, n, ilen, icode)
            assert vend + zend <= 64
            assert (w >> vend) & ((1 << (64 - vend - zend)) - 1) == 0      # zero bits between the spans
            vals.append(v)
            idxs.append(z)
            n_seen += n
            carry += int(z.astype(np.int64).sum()) + n
        assert n_seen <= bp[blk + 1]
        if c + 1 == hv["n_chunks"] or int(meta[c + 1]["blk"]) != blk:
            assert n_seen == bp[blk + 1]
    cat = lambda xs: np.concatenate(xs) if xs else np.zeros(0, np.uint8)
    return cat(vals), cat(idxs), bp


CASES = [(64, 48, 64, 1, 0.1, 5, 4), (64, 48, 16, 16, 0.3, 5, 4), (100, 70, 32, 24, 0.09, 5, 4), (200, 333, 128, 128, 0.09, 5, 4),
         (33, 129, 128, 128, 0.84, 8, 8), (50, 50, 7, 50, 0.02, 3, 2), (1, 1, 1, 1, 1.0, 1, 1), (40, 1, 40, 1, 0.5, 8, 1),
         (96, 363, 96, 363, 0.84, 8, 8), (300, 200, 128, 128, 0.04, 5, 5), (128, 256, 128, 128, 0.0, 5, 4), (128, 256, 128, 128, 1.0, 5, 4)]


@pytest.mark.parametrize("M,K,bh,bw,d,r,k", CASES)
def test_oracle_decodes_library_streams(M, K, bh, bw, d, r, k):
    rng = np.random.default_rng(M * 7 + K + r)
    W = rand_pruned(rng, M, K, d)
    L = cl.compress_layer(W, r, k, bh, bw)
    m = oracle.compress_layer(W, r, k, bh, bw, keep=True)
    hv = L.host_view()
    assert np.array_equal(hv["codebook"], m.codebook)                    # same linear codebook, bit for bit
    val, idx, bp = cross_decode(L)
    assert np.array_equal(val, m.extra["val"]) and np.array_equal(idx, m.extra["idx"])
    assert np.array_equal(bp, m.extra["block_ptr"])
    st = L.stats()
    assert st["nnz"] == int((W != 0).sum()) and st["entries"] == val.size and st["padding"] == int((val == 0).sum())
    # the oracle's unrestricted Huffman is a lower bound on the length-limited size
    vbits, cbits = m.stream_bits
    assert st["val_bits_unlimited"] == vbits and st["idx_bits_unlimited"] == cbits
    assert st["val_bits"] >= vbits and st["idx_bits"] >= cbits
    if val.size > 1000:
        assert st["val_bits"] <= 1.01 * vbits + 64 and st["idx_bits"] <= 1.01 * cbits + 64
    assert max(st["val_max_len"], st["idx_max_len"]) <= binding.MAX_CODE_LEN
    # the derived table of entries that are not padding before each chunk, and the fullest block,
    # from the oracle's own entries
    before = np.concatenate([[0], np.cumsum(m.extra["val"] != 0)])
    assert np.array_equal(hv["chunk_nz"], before[hv["chunk_meta"]["sym_off"]])
    per_block = before[m.extra["block_ptr"][1:]] - before[m.extra["block_ptr"][:-1]]
    assert hv["max_block_nnz"] == (int(per_block.max()) if per_block.size else 0)
    # and the most blocks that eight consecutive chunks of a block row (counted from its first) touch
    widest, pc, blk = 0, hv["panel_chunk"], hv["chunk_meta"]["blk"]
    for p in range(len(pc) - 1):
        for c in range(int(pc[p]), int(pc[p + 1]), 8):
            widest = max(widest, int(blk[min(c + 8, int(pc[p + 1])) - 1]) - int(blk[c]) + 1)
    assert hv["max_group_blocks"] == widest
    # the order of the large-batch sparse path - per block the surviving weights of columns 0-63,
    # then those of columns 64-127, each half row by row: where each chunk's first weight of each
    # half goes and where each group of eight rows starts, from the oracle's entries
    if bh <= 128 and bw <= 128:
        bhh, bww = min(bh, M), min(bw, K)
        nbw_ = -(-K // bww)
        want_gp = np.zeros((len(bp) - 1, 2, 17), np.uint32)
        want_ch = np.zeros((hv["n_chunks"], 2), np.uint32)
        sym_off, blk_of = hv["chunk_meta"]["sym_off"], hv["chunk_meta"]["blk"]
        start = 0
        for b in range(len(bp) - 1):
            bwp = min(bww, K - (b % nbw_) * bww)
            v_b, z_b = m.extra["val"][bp[b]:bp[b + 1]], m.extra["idx"][bp[b]:bp[b + 1]].astype(np.int64)
            pos = np.cumsum(z_b + 1) - 1
            live = v_b != 0
            half = (pos % bwp >= 64).astype(np.int64)
            group = pos // bwp // 8
            n0 = int((live & (half == 0)).sum())
            for h in range(2):
                sel = live & (half == h)
                counts = np.bincount(group[sel], minlength=16)[:16]
                want_gp[b, h, :] = start + h * n0 + np.concatenate([[0], np.cumsum(counts)])
                before = np.concatenate([[0], np.cumsum(sel)])
                for c in np.nonzero(blk_of[:hv["n_chunks"]] == b)[0]:
                    want_ch[c, h] = start + h * n0 + before[sym_off[c] - bp[b]]
            start += int(live.sum())
        assert np.array_equal(hv["group_ptr"], want_gp)
        assert np.array_equal(hv["chunk_half"], want_ch)
    else:
        assert hv["group_ptr"] is None and hv["chunk_half"] is None
    # rebuilt dense matrix from the library's entries equals the oracle's
    Wd = oracle.reconstruct(val, idx, bp, hv["codebook"], M, K, min(bh, M), min(bw, K), k)
    assert np.array_equal(Wd, oracle.dense_weights(m))
    L.free()


def test_supplied_codebook_and_code_length_limit():
    rng = np.random.default_rng(2)
    W = rand_pruned(rng, 256, 512, 0.3)
    cb = np.concatenate([[0], np.sort(rng.standard_normal(255)) * 0.02]).astype(np.float32)
    for lim in (8, 9, 12):
        L = cl.compress_layer(W, 8, 4, 128, 128, codebook=cb, max_code_len=lim)
        st = L.stats()
        assert max(st["val_max_len"], st["idx_max_len"]) <= lim
        val, idx, bp = cross_decode(L)
        q = oracle.quantize(W, 8, cb)
        v2, i2, b2 = oracle.build_entries(q, 128, 128, 4)
        assert np.array_equal(val, v2) and np.array_equal(idx, i2)
    # the limit costs little once it is a few bits above log2(alphabet)
    a = cl.compress_layer(W, 8, 4, 128, 128, codebook=cb, max_code_len=8).stats()
    b = cl.compress_layer(W, 8, 4, 128, 128, codebook=cb, max_code_len=12).stats()
    assert b["val_bits"] <= a["val_bits"] and b["val_bits"] <= 1.002 * b["val_bits_unlimited"]


def test_compress_rejects_bad_arguments():
    W = np.ones((4, 4), np.float32)
    for kw in [dict(weight_bits=0), dict(weight_bits=9), dict(index_bits=0), dict(index_bits=9), dict(block_h=0),
               dict(block_w=-1), dict(max_code_len=13), dict(max_code_len=3)]:
        args = dict(weight_bits=5, index_bits=4, block_h=4, block_w=4, max_code_len=0)
        args.update(kw)
        with pytest.raises(cl.CLError) as e:
            cl.compress_layer(W, **args)
        assert e.value.code == binding.CL_EINVAL
    bad = W.copy()
    bad[1, 2] = np.inf
    with pytest.raises(cl.CLError):
        cl.compress_layer(bad, 5, 4, 4, 4)
    with pytest.raises(cl.CLError):        # codebook[0] must be the reserved zero
        cl.compress_layer(W, 2, 4, 4, 4, codebook=np.array([1, 2, 3, 4], np.float32))
    lib = binding.lib()
    out = C.c_void_p()
    d = binding.LayerDesc(4, 4, 5, 4, 4, 4, 4096, 0)
    assert lib.cl_compress_layer(None, None, None, C.byref(out)) == binding.CL_EINVAL
    assert lib.cl_compress_layer(C.byref(d), None, None, C.byref(out)) == binding.CL_EINVAL
    d.chunk_bits = 2048
    assert lib.cl_compress_layer(C.byref(d), W.ctypes.data_as(C.c_void_p), None, C.byref(out)) == binding.CL_EINVAL
    big = binding.LayerDesc(1 << 16, 1 << 16, 5, 4, 128, 128, 4096, 0)     # M*K overflow, rejected before W is read
    assert lib.cl_compress_layer(C.byref(big), W.ctypes.data_as(C.c_void_p), None, C.byref(out)) == binding.CL_EINVAL
    assert b"M*K" in lib.cl_last_error()


def test_device_entry_points_need_an_uploaded_layer():
    """Without an upload (and here without a GPU) the device calls refuse; they
    never fall back to the CPU."""
    L = cl.compress_layer(np.eye(8, dtype=np.float32), 5, 4, 8, 8)
    lib = binding.lib()
    n = C.c_size_t(0)
    assert lib.cl_fc_workspace_bytes(L.handle, 0, 0, C.byref(n)) == binding.CL_EINVAL
    assert lib.cl_fc_workspace_bytes(L.handle, 1, 7, C.byref(n)) == binding.CL_EINVAL
    rc = lib.cl_compressed_fc_forward(L.handle, None, None, None, 1, 0, 0, None, 0, None)
    assert rc in (binding.CL_EINVAL, binding.CL_EHIP)
    rc = lib.cl_decode_layer(L.handle, None, None, None, None, None)
    assert rc in (binding.CL_EINVAL, binding.CL_EHIP)


def test_serialize_round_trip_and_corruption():
    rng = np.random.default_rng(12)
    W = rand_pruned(rng, 130, 300, 0.1)
    L = cl.compress_layer(W, 5, 4, 64, 128)
    img = L.serialize()
    L2 = cl.layer_deserialize(img)
    a, b = L.host_view(), L2.host_view()
    for key in a:
        if isinstance(a[key], np.ndarray):
            assert np.array_equal(a[key], b[key]), key
        else:
            assert a[key] == b[key], key
    assert L.stats() == L2.stats()
    # truncated, extended, and bit-flipped images are refused
    for bad in (img[:-1], img + b"\0", img[:40]):
        with pytest.raises(cl.CLError) as e:
            cl.layer_deserialize(bad)
        assert e.value.code == binding.CL_ECORRUPT
    rng = np.random.default_rng(0)
    for _ in range(40):
        pos = int(rng.integers(0, len(img)))
        flipped = bytearray(img)
        flipped[pos] ^= 1 << int(rng.integers(0, 8))
        with pytest.raises(cl.CLError) as e:
            cl.layer_deserialize(bytes(flipped))
        assert e.value.code == binding.CL_ECORRUPT


def test_validation_catches_inconsistent_tables_even_with_a_good_checksum():
    """Re-seal a tampered image with a fresh checksum: the structural validation
    (full host decode) must still refuse it."""
    rng = np.random.default_rng(13)
    W = rand_pruned(rng, 130, 300, 0.1)
    L = cl.compress_layer(W, 5, 4, 64, 128)
    img = bytearray(L.serialize())
    hv = L.host_view()
    hdr = len(img) - (hv["codebook"].nbytes + hv["val_len"].nbytes + hv["idx_len"].nbytes + hv["block_ptr"].nbytes +
                      hv["panel_chunk"].nbytes + hv["chunk_meta"].nbytes + hv["records"].nbytes)

    def reseal(buf):
        h = 1469598103934665603
        for byte in bytes(buf[hdr:]):
            h = ((h ^ byte) * 1099511628211) & (2 ** 64 - 1)
        buf[hdr - 8:hdr] = h.to_bytes(8, "little")
        return bytes(buf)

    assert cl.layer_deserialize(reseal(bytearray(img))).stats() == L.stats()
    off_bp = hdr + hv["codebook"].nbytes + hv["val_len"].nbytes + hv["idx_len"].nbytes
    off_meta = off_bp + hv["block_ptr"].nbytes + hv["panel_chunk"].nbytes
    off_rec = off_meta + hv["chunk_meta"].nbytes
    tampered = []
    t = bytearray(img); t[off_bp + 4] ^= 1; tampered.append(t)                 # block_ptr[1]
    t = bytearray(img); t[off_meta + 16] ^= 1; tampered.append(t)              # sym_off of chunk 1
    t = bytearray(img); t[off_meta + 16 + 4] ^= 1; tampered.append(t)          # rec_off of chunk 1
    t = bytearray(img); t[off_meta + 16 + 8] ^= 1; tampered.append(t)          # blk of chunk 1
    t = bytearray(img); t[off_meta + 16 + 12] ^= 1; tampered.append(t)         # pos0 of chunk 1
    t = bytearray(img); t[off_rec] ^= 1; tampered.append(t)                    # entry count of record 0
    t = bytearray(img); t[hdr + hv["codebook"].nbytes + 5] = 1; tampered.append(t)   # a code length (breaks Kraft)
    for t in tampered:
        with pytest.raises(cl.CLError) as e:
            cl.layer_deserialize(reseal(t))
        assert e.value.code == binding.CL_ECORRUPT
    assert off_rec < len(img)


def test_format_statistics_on_benchmark_shapes():
    """Scaled-down AlexNet fc6 (same density / bit widths): padding rate and bits
    per non-zero land where the closed forms say."""
    spec, W = wl.layer_weights(2, 0, scale=0.25)
    L = cl.compress_layer(W, spec.r, spec.k, 128, 128)
    st = L.stats()
    q, R = 1 - spec.density, 1 << spec.k
    assert abs(st["padding"] / st["nnz"] - q ** R / (1 - q ** R)) < 0.02
    bits_per_nnz = st["model_bytes"] * 8 / st["nnz"]
    assert 9.0 < bits_per_nnz < 12.0
    # tables are a small fraction of the payload
    assert st["table_bytes"] < 0.05 * st["payload_bytes"]
    # records are well filled: count field (4 bits) + padding stay under a fifth of the payload
    assert (st["val_bits"] + st["idx_bits"]) / (st["n_records"] * 64) > 0.80
    # almost all chunks are full wavefronts
    assert st["n_records"] / st["n_chunks"] > 55


@pytest.mark.parametrize("seed", range(25))
def test_planner_matches_oracle_dp(seed):
    rng = np.random.default_rng(100 + seed)
    f = int(rng.integers(1, 5))
    bs = [1, 2, 4, 8, 16] if seed % 2 else [1, 2, 3, 6, 12, 24]
    time_ms = [[float(rng.uniform(0.5, 2.0) * (1 + 0.3 * b ** rng.uniform(0.4, 1.0))) for b in bs] for _ in range(f)]
    inb = [int(rng.integers(1, 40)) * 100 for _ in range(f)]
    outb = inb[1:] + [int(rng.integers(1, 40)) * 100]
    ws = [int(rng.integers(0, 30)) * 100 for _ in range(f)]
    tot = int(rng.integers(20, 600)) * 100
    step = int(rng.choice([100, 700, 1]))
    cap = None if seed % 3 else float(rng.uniform(3, 40))
    ref, rplan = odp.plan_batches(time_ms, bs, inb, outb, ws, tot, step, cap)
    got, plan = cl.plan_batches(time_ms, bs, inb, outb, ws, tot, step, cap)
    if rplan is None:
        assert plan is None
    else:
        assert got == pytest.approx(ref, rel=1e-12)
        # the returned plan is itself feasible and costs what was reported
        cost, A = 0.0, 0
        for i in range(f):
            cost = time_ms[i][bs.index(plan[i])] + (0 if i == 0 else (plan[i] // plan[i - 1]) * cost)
        assert cost / plan[-1] == pytest.approx(got, rel=1e-12)
        for i in range(f - 1, -1, -1):
            assert A + plan[i] * inb[i] + ws[i] + plan[i] * outb[i] <= tot
            if i:
                assert plan[i] % plan[i - 1] == 0
                A = -(-(A + (plan[i] - plan[i - 1]) * inb[i]) // step) * step


def test_scheduler_charges_a_dispatch_what_the_recurrence_says():
    """The scheduler's cost of a dispatch with per-layer batch sizes is the Sec. V-C
    recurrence for exactly those sizes (earlier layers repeated until the later
    layer's batch is full): equal to the oracle's optimum when the sizes are the
    plan's, and to a hand count on a small case."""
    from paper_1711_00244_amd import scheduler
    rng = np.random.default_rng(3)
    bs = [1, 2, 4, 8, 16]
    for _ in range(10):
        f = int(rng.integers(1, 5))
        time_ms = np.sort(rng.random((f, len(bs))) + 0.1, axis=1)
        inb, outb, ws = [int(x) for x in rng.integers(100, 5000, f)], [int(x) for x in rng.integers(100, 5000, f)], [0] * f
        tot = int(rng.integers(20000, 200000))
        want, plan = odp.plan_batches(time_ms.tolist(), bs, inb, outb, ws, tot, 1024)
        if plan is None:
            continue
        p = scheduler.Plan(list(plan), want, bs, time_ms, ws, tot)
        assert p.dispatch_ms(plan) / plan[-1] == pytest.approx(want, rel=1e-12)
    t = np.array([[1.0, 1.5, 2.0], [10.0, 11.0, 12.0], [100.0, 101.0, 102.0]])
    p = scheduler.Plan([1, 2, 4], 0.0, [1, 2, 4], t, [0, 0, 0], 0)
    assert p.dispatch_ms([1, 2, 4]) == 102.0 + 2 * (11.0 + 2 * 1.0)
    assert p.dispatch_ms([4, 4, 4]) == 2.0 + 12.0 + 102.0
    assert p.bpl_for(2) == [1, 2, 2] and p.bpl_for(4) == [1, 2, 4] and p.bpl_for(1) == [1, 1, 1]


def test_planner_rejects_bad_arguments():
    with pytest.raises(cl.CLError):
        cl.plan_batches([[1.0, 2.0]], [2, 1], [1], [1], [0], 100, 1)
    with pytest.raises(cl.CLError):
        cl.plan_batches([[1.0, float("nan")]], [1, 2], [1], [1], [0], 100, 1)
    assert cl.plan_batches([[1.0, 2.0]], [1, 2], [1000], [1000], [0], 100, 1) == (float("inf"), None)


def test_conv_block_h_divides_a_groups_filters():
    """The binding's choice of block height for grouped convolutions: the largest
    divisor of the filters per group that fits the requested height."""
    assert cl.conv_block_h(96, 1) == 128            # no groups: as asked
    assert cl.conv_block_h(256, 2) == 128           # AlexNet conv2 / conv5: 128 filters per group
    assert cl.conv_block_h(384, 2) == 96            # AlexNet conv4: 192 per group
    assert cl.conv_block_h(384, 2, 64) == 64
    assert cl.conv_block_h(14, 2) == 7
    for oc, g, bh in [(384, 2, 128), (60, 3, 16), (26, 2, 128)]:
        h = cl.conv_block_h(oc, g, bh)
        assert (oc // g) % h == 0 and h <= bh


def test_bench_refuses_more_than_one_gpu():
    """Every box of this build has one GPU: the benchmark says so and exits without touching
    a device when asked for more."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in (r.stdout + r.stderr)
