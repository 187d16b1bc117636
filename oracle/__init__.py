"""CPU oracle: thin ctypes binding over ``oracle.c`` plus the layer-level steps.

TEST INFRASTRUCTURE ONLY.  Imported by ``tests/``, by the smoke check and by the
CPU-baseline leg of the benchmark; the product package never imports it and it
never imports the product package.

The C file holds the arithmetic, one function per passage of the paper; this
module strings those functions together in the order Algorithm 2 states them.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass, field

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

GCC_CMD = ["gcc", "-O2", "-std=c99", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC",
           _SRC, "-o", _LIB, "-lm"]


def build(force: bool = False) -> str:
    """Compile oracle.c with gcc (a second's work).  Returns the library path."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        subprocess.run(GCC_CMD, check=True)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        i64, i32, p = C.c_int64, C.c_int, C.c_void_p
        _lib.orc_linear_codebook.argtypes = [p, i64, i32, p]
        _lib.orc_quantize.argtypes = [p, i64, i32, p, p]
        _lib.orc_num_blocks.argtypes = [i32] * 4
        _lib.orc_num_blocks.restype = i64
        _lib.orc_build_entries.argtypes = [p, i32, i32, i32, i32, i32, i32, p, p, p]
        _lib.orc_build_entries.restype = i64
        _lib.orc_huffman_code.argtypes = [p, i32, p, p]
        _lib.orc_huffman_encode.argtypes = [p, i64, i32, p, p, p, i64]
        _lib.orc_huffman_encode.restype = i64
        _lib.orc_huffman_decode_serial.argtypes = [p, i64, i64, i64, i32, p, p, p, p]
        _lib.orc_huffman_decode_serial.restype = i64
        _lib.orc_huffman_decode_span.argtypes = [p, i64, i64, i32, p, p, p, i64]
        _lib.orc_huffman_decode_span.restype = i64
        _lib.orc_reconstruct.argtypes = [p, p, p, p, i32, i32, i32, i32, i32, i32, p, p]
        _lib.orc_fc_forward.argtypes = [p, p, p, i32, i32, i32, i32, i32, p]
        _lib.orc_conv_forward.argtypes = [p, p, p] + [i32] * 12 + [p]
        _lib.orc_maxpool_forward.argtypes = [p] + [i32] * 6 + [p]
        _lib.orc_lrn_forward.argtypes = [p] + [i32] * 5 + [C.c_double] * 3 + [p]
    return _lib


class OracleError(RuntimeError):
    pass


def _ptr(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _chk(rc, what):
    if rc < 0:
        raise OracleError(f"{what}: error {rc}")
    return rc


def _c(a, dtype):
    return np.ascontiguousarray(a, dtype=dtype)


# --------------------------------------------------------------------------- #
# one-to-one wrappers
# --------------------------------------------------------------------------- #
def linear_codebook(W, r: int) -> np.ndarray:
    W = _c(W, np.float32)
    cb = np.zeros(1 << r, np.float32)
    _chk(lib().orc_linear_codebook(_ptr(W), W.size, r, _ptr(cb)), "linear_codebook")
    return cb


def quantize(W, r: int, codebook) -> np.ndarray:
    W = _c(W, np.float32)
    cb = _c(codebook, np.float32)
    if cb.size != (1 << r):
        raise OracleError("codebook must have 2^r entries")
    q = np.zeros(W.shape, np.uint8)
    _chk(lib().orc_quantize(_ptr(W), W.size, r, _ptr(cb), _ptr(q)), "quantize")
    return q


def num_blocks(M, K, bh, bw) -> int:
    return int(_chk(lib().orc_num_blocks(M, K, bh, bw), "num_blocks"))


def build_entries(q, bh: int, bw: int, k: int, colmajor: bool = False):
    """q: M x K uint8 index matrix -> (val, idx, block_ptr)."""
    q = _c(q, np.uint8)
    M, K = q.shape
    n = _chk(lib().orc_build_entries(_ptr(q), M, K, bh, bw, k, int(colmajor), None, None, None), "build_entries")
    val = np.zeros(n, np.uint8)
    idx = np.zeros(n, np.uint8)
    bp = np.zeros(num_blocks(M, K, bh, bw) + 1, np.int64)
    n2 = lib().orc_build_entries(_ptr(q), M, K, bh, bw, k, int(colmajor), _ptr(val), _ptr(idx), _ptr(bp))
    assert n2 == n
    return val, idx, bp


def huffman_code(counts):
    counts = _c(counts, np.int64)
    ln = np.zeros(counts.size, np.uint8)
    code = np.zeros(counts.size, np.uint64)
    _chk(lib().orc_huffman_code(_ptr(counts), counts.size, _ptr(ln), _ptr(code)), "huffman_code")
    return ln, code


def huffman_encode(sym, ln, code):
    """-> (bytes as uint8 array padded to a whole byte, total bits)."""
    sym = _c(sym, np.uint8)
    ln = _c(ln, np.uint8)
    code = _c(code, np.uint64)
    nbits = _chk(lib().orc_huffman_encode(_ptr(sym), sym.size, ln.size, _ptr(ln), _ptr(code), None, 0), "encode")
    buf = np.zeros((nbits + 7) // 8 + 1, np.uint8)
    end = lib().orc_huffman_encode(_ptr(sym), sym.size, ln.size, _ptr(ln), _ptr(code), _ptr(buf), 0)
    assert end == nbits
    return buf, int(nbits)


def huffman_decode_serial(buf, total_bits, start_bit, n, ln, code, want_bitpos=False):
    buf = _c(buf, np.uint8)
    ln = _c(ln, np.uint8)
    code = _c(code, np.uint64)
    if total_bits > buf.size * 8:
        raise OracleError("total_bits exceeds buffer")
    out = np.zeros(n, np.uint8)
    bitpos = np.zeros(n, np.int64) if want_bitpos else None
    end = _chk(lib().orc_huffman_decode_serial(_ptr(buf), total_bits, start_bit, n, ln.size, _ptr(ln), _ptr(code),
                                               _ptr(out), _ptr(bitpos)), "decode_serial")
    return (out, int(end), bitpos) if want_bitpos else (out, int(end))


def huffman_decode_span(buf, start_bit, end_bit, ln, code):
    buf = _c(buf, np.uint8)
    ln = _c(ln, np.uint8)
    code = _c(code, np.uint64)
    if end_bit > buf.size * 8:
        raise OracleError("end_bit exceeds buffer")
    cap = max(int(end_bit - start_bit), 1)
    out = np.zeros(cap, np.uint8)
    n = _chk(lib().orc_huffman_decode_span(_ptr(buf), start_bit, end_bit, ln.size, _ptr(ln), _ptr(code),
                                           _ptr(out), cap), "decode_span")
    return out[:n].copy()


def reconstruct(val, idx, block_ptr, codebook, M, K, bh, bw, k, colmajor=False, want_q=False):
    val = _c(val, np.uint8)
    idx = _c(idx, np.uint8)
    bp = _c(block_ptr, np.int64)
    cb = _c(codebook, np.float32)
    if bp.size != num_blocks(M, K, bh, bw) + 1 or val.size != idx.size or (bp.size and bp[-1] != val.size):
        raise OracleError("inconsistent entry arrays")
    Wd = np.zeros((M, K), np.float32)
    qd = np.zeros((M, K), np.uint8) if want_q else None
    _chk(lib().orc_reconstruct(_ptr(val), _ptr(idx), _ptr(bp), _ptr(cb), M, K, bh, bw, k, int(colmajor),
                               _ptr(Wd), _ptr(qd)), "reconstruct")
    return (Wd, qd) if want_q else Wd


def fc_forward(W, X, bias=None, relu=False, nthreads=1) -> np.ndarray:
    """W: M x K fp32, X: B x K fp32 -> Y: B x M fp64 (Eq. 1-2)."""
    W = _c(W, np.float32)
    X = _c(X, np.float32)
    M, K = W.shape
    B = X.shape[0]
    assert X.shape[1] == K
    b = None if bias is None else _c(bias, np.float32)
    Y = np.zeros((B, M), np.float64)
    _chk(lib().orc_fc_forward(_ptr(W), _ptr(X), _ptr(b), M, K, B, int(relu), nthreads, _ptr(Y)), "fc_forward")
    return Y


def conv_forward(W, X, geom, bias=None, relu=False, nthreads=1) -> np.ndarray:
    """W: OC x (C/groups*R*S) fp32, X: B x C x H x W fp32 -> B x OC x P x Q fp64.
    geom: dict(C,H,W,R,S,stride,pad,groups,OC)."""
    W = _c(W, np.float32)
    X = _c(X, np.float32)
    g = geom
    B = X.shape[0]
    assert X.shape[1:] == (g["C"], g["H"], g["W"])
    assert W.shape == (g["OC"], g["C"] // g["groups"] * g["R"] * g["S"])
    P = (g["H"] + 2 * g["pad"] - g["R"]) // g["stride"] + 1
    Q = (g["W"] + 2 * g["pad"] - g["S"]) // g["stride"] + 1
    b = None if bias is None else _c(bias, np.float32)
    Y = np.zeros((B, g["OC"], P, Q), np.float64)
    _chk(lib().orc_conv_forward(_ptr(W), _ptr(X), _ptr(b), B, g["C"], g["H"], g["W"], g["OC"], g["R"], g["S"],
                                g["stride"], g["pad"], g["groups"], int(relu), nthreads, _ptr(Y)), "conv_forward")
    return Y


def maxpool_forward(X, size: int, stride: int) -> np.ndarray:
    """X: B x C x H x W fp32 -> B x C x P x Q fp64, P = (H - size) // stride + 1
    (the pooling layers of the AlexNet runs, Table IV)."""
    X = _c(X, np.float32)
    B, Cc, H, W = X.shape
    P, Q = (H - size) // stride + 1, (W - size) // stride + 1
    Y = np.zeros((B, Cc, P, Q), np.float64)
    _chk(lib().orc_maxpool_forward(_ptr(X), B, Cc, H, W, size, stride, _ptr(Y)), "maxpool_forward")
    return Y


def lrn_forward(X, n: int = 5, alpha: float = 1e-4, beta: float = 0.75, k: float = 1.0) -> np.ndarray:
    """Across-channel local response normalisation (the norm layers of Table IV):
    y[c] = x[c] / (k + alpha / n * sum of x[c']^2 over the n channels around c)^beta."""
    X = _c(X, np.float32)
    B, Cc, H, W = X.shape
    Y = np.zeros(X.shape, np.float64)
    _chk(lib().orc_lrn_forward(_ptr(X), B, Cc, H, W, n, float(alpha), float(beta), float(k), _ptr(Y)),
         "lrn_forward")
    return Y


# --------------------------------------------------------------------------- #
# the compressed model of Sec. III-B / IV-A and the steps of Algorithm 2
# --------------------------------------------------------------------------- #
@dataclass
class OracleModel:
    """What the paper's inference algorithms take as input: the two Huffman bit
    streams, the row_ptr array of <val address, col_ind address> pairs (one per
    block, plus the end), the codebook, and the parameters that say how to read
    them."""
    M: int
    K: int
    r: int
    k: int
    bh: int
    bw: int
    colmajor: bool
    codebook: np.ndarray
    val_stream: np.ndarray
    col_stream: np.ndarray
    row_ptr: np.ndarray            # (nblocks + 1, 2) int64 bit addresses
    val_len: np.ndarray
    val_code: np.ndarray
    col_len: np.ndarray
    col_code: np.ndarray
    n_entries: int
    extra: dict = field(default_factory=dict)

    @property
    def stream_bits(self):
        return int(self.row_ptr[-1, 0]), int(self.row_ptr[-1, 1])


def compress_layer(W, r, k, bh, bw, codebook=None, colmajor=False, keep=False) -> OracleModel:
    """Sec. III-B pipeline on an already pruned matrix (pruned = exact zeros):
    quantise -> relative-indexed entries per block -> Huffman code each array."""
    W = _c(W, np.float32)
    M, K = W.shape
    cb = linear_codebook(W, r) if codebook is None else _c(codebook, np.float32)
    q = quantize(W, r, cb)
    val, idx, bp = build_entries(q, bh, bw, k, colmajor)
    vlen, vcode = huffman_code(np.bincount(val, minlength=1 << r))
    clen, ccode = huffman_code(np.bincount(idx, minlength=1 << k))
    vbuf, vbits = huffman_encode(val, vlen, vcode)
    cbuf, cbits = huffman_encode(idx, clen, ccode)
    # row_ptr: bit address at which each block starts in either stream
    vcum = np.concatenate([[0], np.cumsum(vlen[val].astype(np.int64))])
    ccum = np.concatenate([[0], np.cumsum(clen[idx].astype(np.int64))])
    row_ptr = np.stack([vcum[bp], ccum[bp]], axis=1)
    assert row_ptr[-1, 0] == vbits and row_ptr[-1, 1] == cbits
    m = OracleModel(M, K, r, k, bh, bw, colmajor, cb, vbuf, cbuf, row_ptr, vlen, vcode, clen, ccode, int(val.size))
    if keep:
        m.extra = {"q": q, "val": val, "idx": idx, "block_ptr": bp}
    return m


def decode_layer(m: OracleModel):
    """Algorithm 2 steps 3-6 for every block: take the block's spans from
    row_ptr and Huffman-decode them bit by bit.  -> (val, idx, block_ptr)."""
    vals, idxs, bp = [], [], [0]
    nblocks = m.row_ptr.shape[0] - 1
    for i in range(nblocks):
        v = huffman_decode_span(m.val_stream, int(m.row_ptr[i, 0]), int(m.row_ptr[i + 1, 0]), m.val_len, m.val_code)
        c = huffman_decode_span(m.col_stream, int(m.row_ptr[i, 1]), int(m.row_ptr[i + 1, 1]), m.col_len, m.col_code)
        if v.size != c.size:
            raise OracleError(f"block {i}: val and col_ind spans decode to different lengths")
        vals.append(v)
        idxs.append(c)
        bp.append(bp[-1] + v.size)
    cat = lambda xs: np.concatenate(xs) if xs else np.zeros(0, np.uint8)
    return cat(vals), cat(idxs), np.asarray(bp, np.int64)


def decode_layer_whole(m: OracleModel):
    """Same result as decode_layer, walking each stream once from bit 0 (what the
    benchmark's CPU baseline times; the block spans are contiguous)."""
    vbits, cbits = m.stream_bits
    val, ve = huffman_decode_serial(m.val_stream, vbits, 0, m.n_entries, m.val_len, m.val_code)
    idx, ce = huffman_decode_serial(m.col_stream, cbits, 0, m.n_entries, m.col_len, m.col_code)
    if ve != vbits or ce != cbits:
        raise OracleError("streams do not end where row_ptr says")
    return val, idx


def dense_weights(m: OracleModel, val=None, idx=None, block_ptr=None) -> np.ndarray:
    """Algorithm 2 steps 7-9 for every block -> the M x K matrix the layer multiplies by."""
    if val is None:
        val, idx, block_ptr = decode_layer(m)
    return reconstruct(val, idx, block_ptr, m.codebook, m.M, m.K, m.bh, m.bw, m.k, m.colmajor)


def compressed_fc_forward(m: OracleModel, X, bias=None, relu=False, nthreads=1) -> np.ndarray:
    """Decode, rebuild the dense matrix, multiply (Eq. 1-2)."""
    return fc_forward(dense_weights(m), X, bias, relu, nthreads)
