"""ctypes binding over libcompressed_layer.so: argument marshalling only.

Every step of the path (decode, prefix sums, codebook lookup, multiply) runs in
the library's HIP kernels.  Tensors are torch CUDA tensors used as raw device
memory; the stream is torch's current stream.  There is no fallback: if the
library is missing or was not built, importing a symbol from it raises.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

from . import build as _build

CL_OK, CL_EINVAL, CL_ENOMEM, CL_ECORRUPT, CL_EUNSUPPORTED, CL_EHIP = 0, -1, -2, -3, -4, -5
PATH_AUTO, PATH_SPARSE, PATH_MFMA_F32, PATH_MFMA_BF16, PATH_SPARSE_WIDE = 0, 1, 2, 3, 4
CHUNK_BITS, RECORD_BITS, RECORDS_PER_CHUNK, MAX_RECORD_ENTRIES, MAX_CODE_LEN = 4096, 64, 64, 15, 12
STATIC_SCRATCH_BYTES = 16 << 20        # CL_STATIC_SCRATCH_BYTES

EXPORTS = [
    "cl_last_error", "cl_compress_layer", "cl_layer_upload", "cl_layer_free", "cl_layer_stats",
    "cl_layer_host_view", "cl_layer_serialize", "cl_layer_deserialize", "cl_decode_layer",
    "cl_fc_workspace_bytes", "cl_fc_resolved_path", "cl_compressed_fc_forward", "cl_compressed_fc_forward_static", "cl_fc_stack_workspace_bytes",
    "cl_compressed_fc_stack_forward", "cl_layer_group_create", "cl_layer_group_free", "cl_fc_group_workspace_bytes",
    "cl_compressed_fc_group_forward", "cl_conv_workspace_bytes", "cl_conv_workspace_bytes_min",
    "cl_compressed_conv_forward", "cl_plan_batches", "cl_maxpool_forward", "cl_lrn_forward",
    "cl_set_kernel_timing", "cl_last_kernel_ms",
]


class LayerDesc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("M", "K", "weight_bits", "index_bits", "block_h", "block_w", "chunk_bits", "max_code_len")]


class Stats(C.Structure):
    _fields_ = [(n, C.c_int64) for n in ("nnz", "padding", "entries", "n_blocks", "n_chunks", "val_bits", "idx_bits",
                                         "val_bits_unlimited", "idx_bits_unlimited", "n_records", "payload_bytes", "table_bytes",
                                         "model_bytes", "lut_bytes")] + [("val_max_len", C.c_int32), ("idx_max_len", C.c_int32)]


class ChunkMeta(C.Structure):
    _fields_ = [("sym_off", C.c_uint32), ("rec_off", C.c_uint32), ("blk", C.c_uint32), ("pos0", C.c_uint32)]


class HostView(C.Structure):
    _fields_ = [("desc", LayerDesc), ("codebook", C.POINTER(C.c_float)), ("val_len", C.POINTER(C.c_uint8)),
                ("val_code", C.POINTER(C.c_uint32)), ("idx_len", C.POINTER(C.c_uint8)), ("idx_code", C.POINTER(C.c_uint32)),
                ("block_ptr", C.POINTER(C.c_uint32)), ("panel_chunk", C.POINTER(C.c_uint32)),
                ("chunk_meta", C.POINTER(ChunkMeta)), ("records", C.POINTER(C.c_uint64)),
                ("n_blocks", C.c_int64), ("n_chunks", C.c_int64), ("n_records", C.c_int64), ("n_entries", C.c_int64),
                ("n_panels", C.c_int32), ("chunk_nz", C.POINTER(C.c_uint32)), ("max_block_nnz", C.c_int64),
                ("max_group_blocks", C.c_int32), ("chunk_half", C.POINTER(C.c_uint32)), ("group_ptr", C.POINTER(C.c_uint32))]


class ConvDesc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("C", "H", "W", "R", "S", "stride", "pad", "groups", "out_channels")]


class CLError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"[{code}] {msg}")
        self.code = code


_lib = None


def library_path() -> str:
    return _build.LIB


def lib():
    """Load the built library; build it only if no built library is there."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_build.LIB):
        _build.build_library()
    # PyTorch brings a HIP runtime of its own, and device memory comes from PyTorch: its
    # runtime has to be the one in the process before this library resolves its HIP
    # symbols (loaded the other way round, PyTorch afterwards finds no GPU)
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    L = C.CDLL(_build.LIB)
    p, i32, i64, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t
    L.cl_last_error.restype = C.c_char_p
    L.cl_compress_layer.argtypes = [C.POINTER(LayerDesc), p, p, C.POINTER(p)]
    L.cl_layer_upload.argtypes = [p]
    L.cl_layer_free.argtypes = [p]
    L.cl_layer_stats.argtypes = [p, C.POINTER(Stats)]
    L.cl_layer_host_view.argtypes = [p, C.POINTER(HostView)]
    L.cl_layer_serialize.argtypes = [p, p, C.POINTER(sz)]
    L.cl_layer_deserialize.argtypes = [p, sz, C.POINTER(p)]
    L.cl_decode_layer.argtypes = [p, p, p, p, p, p]
    L.cl_fc_workspace_bytes.argtypes = [p, i32, i32, C.POINTER(sz)]
    L.cl_fc_resolved_path.argtypes = [p, i32, i32, C.POINTER(i32)]
    L.cl_compressed_fc_forward_static.argtypes = [p, p, p, p, i32, i32, i32, p]
    L.cl_compressed_fc_forward.argtypes = [p, p, p, p, i32, i32, i32, p, sz, p]
    L.cl_fc_stack_workspace_bytes.argtypes = [p, i32, i32, i32, C.POINTER(sz)]
    L.cl_compressed_fc_stack_forward.argtypes = [p, i32, p, p, p, i32, i32, i32, i32, p, sz, p]
    L.cl_layer_group_create.argtypes = [p, i32, C.POINTER(p)]
    L.cl_fc_group_workspace_bytes.argtypes = [p, i32, C.POINTER(sz)]
    L.cl_compressed_fc_group_forward.argtypes = [p, p, sz, p, sz, p, i32, i32, p, sz, p]
    L.cl_conv_workspace_bytes.argtypes = [p, C.POINTER(ConvDesc), i32, i32, C.POINTER(sz)]
    L.cl_conv_workspace_bytes_min.argtypes = [p, C.POINTER(ConvDesc), i32, i32, C.POINTER(sz)]
    L.cl_compressed_conv_forward.argtypes = [p, C.POINTER(ConvDesc), p, p, p, i32, i32, i32, p, sz, p]
    L.cl_plan_batches.argtypes = [i32, p, i32, p, p, p, p, i64, i64, C.c_double, p, C.POINTER(C.c_double)]
    L.cl_maxpool_forward.argtypes = [p, p] + [i32] * 6 + [p]
    L.cl_lrn_forward.argtypes = [p, p] + [i32] * 5 + [C.c_float] * 3 + [p]
    L.cl_set_kernel_timing.argtypes = [i32]
    L.cl_last_kernel_ms.argtypes = [C.POINTER(C.c_float), C.POINTER(i32)]
    for name in EXPORTS:
        if name not in ("cl_last_error", "cl_layer_group_free"):
            getattr(L, name).restype = i32
    L.cl_layer_group_free.restype = None
    L.cl_layer_group_free.argtypes = [C.c_void_p]
    _lib = L
    return L


def _check(rc):
    if rc != CL_OK:
        raise CLError(rc, lib().cl_last_error().decode())


def _np_ptr(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _dev_ptr(t):
    """Raw device address of a torch CUDA tensor (or None)."""
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("expected a contiguous CUDA tensor")
    return C.c_void_p(t.data_ptr())


def _stream():
    import torch
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _want(t, shape, what):
    """A tensor handed to the library as a raw pointer must be what the kernels
    assume: fp32, contiguous, on the GPU, of exactly this shape."""
    import torch
    if t is None:
        return
    if t.dtype != torch.float32 or tuple(t.shape) != tuple(shape) or not t.is_cuda or not t.is_contiguous():
        raise ValueError(f"{what} must be a contiguous float32 CUDA tensor of shape {tuple(shape)}, "
                         f"got {t.dtype} {tuple(t.shape)}")


class Layer:
    """Owns a cl_layer handle."""

    def __init__(self, handle):
        self._h = C.c_void_p(handle)
        v = HostView()
        _check(lib().cl_layer_host_view(self._h, C.byref(v)))
        self.M, self.K = v.desc.M, v.desc.K
        self._ws_cache = {}

    @property
    def handle(self):
        if not self._h:
            raise ValueError("layer was freed")
        return self._h

    def free(self):
        if self._h:
            lib().cl_layer_free(self._h)
            self._h = C.c_void_p(None)

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass

    # -- mirrors of the C entry points ------------------------------------- #
    def upload(self):
        _check(lib().cl_layer_upload(self.handle))
        return self

    def stats(self) -> dict:
        s = Stats()
        _check(lib().cl_layer_stats(self.handle, C.byref(s)))
        return {n: getattr(s, n) for n, _ in Stats._fields_}

    def host_view(self) -> dict:
        """numpy copies of the host sections."""
        v = HostView()
        _check(lib().cl_layer_host_view(self.handle, C.byref(v)))
        d = v.desc
        nval, nidx = 1 << d.weight_bits, 1 << d.index_bits

        def arr(ptr, n, dt):
            if n == 0:
                return np.zeros(0, dt)
            return np.ctypeslib.as_array(ptr, shape=(n,)).astype(dt, copy=True)

        nc = int(v.n_chunks)
        meta = np.zeros(nc + 1, dtype=[("sym_off", "<u4"), ("rec_off", "<u4"), ("blk", "<u4"), ("pos0", "<u4")])
        C.memmove(meta.ctypes.data, v.chunk_meta, meta.nbytes)
        return dict(desc={n: getattr(d, n) for n, _ in LayerDesc._fields_},
                    codebook=arr(v.codebook, nval, np.float32), val_len=arr(v.val_len, nval, np.uint8),
                    val_code=arr(v.val_code, nval, np.uint32), idx_len=arr(v.idx_len, nidx, np.uint8),
                    idx_code=arr(v.idx_code, nidx, np.uint32), block_ptr=arr(v.block_ptr, int(v.n_blocks) + 1, np.uint32),
                    panel_chunk=arr(v.panel_chunk, int(v.n_panels) + 1, np.uint32), chunk_meta=meta,
                    records=arr(v.records, int(v.n_records), np.uint64),
                    chunk_nz=arr(v.chunk_nz, nc + 1, np.uint32), max_block_nnz=int(v.max_block_nnz),
                    max_group_blocks=int(v.max_group_blocks),
                    chunk_half=None if not v.group_ptr else
                    arr(v.chunk_half, 2 * nc, np.uint32).reshape(nc, 2) if nc else np.zeros((0, 2), np.uint32),
                    group_ptr=arr(v.group_ptr, int(v.n_blocks) * 34, np.uint32).reshape(int(v.n_blocks), 2, 17) if v.group_ptr else None,
                    n_blocks=int(v.n_blocks), n_chunks=nc, n_records=int(v.n_records), n_entries=int(v.n_entries),
                    n_panels=int(v.n_panels))

    def serialize(self) -> bytes:
        n = C.c_size_t(0)
        _check(lib().cl_layer_serialize(self.handle, None, C.byref(n)))
        buf = C.create_string_buffer(n.value)
        _check(lib().cl_layer_serialize(self.handle, buf, C.byref(n)))
        return buf.raw[:n.value]


def conv_block_h(out_channels: int, groups: int, block_h: int = 128) -> int:
    """Block height for a convolution layer: with filter groups the library wants
    block_h to divide the filters of a group, so the largest such divisor up to
    block_h (AlexNet conv4, 192 filters per group: 96)."""
    per_group = out_channels // groups
    if groups == 1 or per_group % block_h == 0:
        return block_h
    return max(d for d in range(1, min(block_h, per_group) + 1) if per_group % d == 0)


def compress_layer(W, weight_bits, index_bits, block_h, block_w, codebook=None, max_code_len=0, upload=False) -> Layer:
    W = np.ascontiguousarray(W, np.float32)
    if W.ndim != 2:
        raise ValueError("W must be M x K")
    d = LayerDesc(W.shape[0], W.shape[1], weight_bits, index_bits, block_h, block_w, CHUNK_BITS, max_code_len)
    cb = None if codebook is None else np.ascontiguousarray(codebook, np.float32)
    if cb is not None and cb.size != (1 << weight_bits):
        raise ValueError("codebook must have 2^weight_bits entries")
    out = C.c_void_p()
    _check(lib().cl_compress_layer(C.byref(d), _np_ptr(W), _np_ptr(cb), C.byref(out)))
    layer = Layer(out.value)
    if upload:
        layer.upload()
    return layer


def layer_deserialize(data: bytes) -> Layer:
    out = C.c_void_p()
    _check(lib().cl_layer_deserialize(data, len(data), C.byref(out)))
    return Layer(out.value)


def decode_layer(layer: Layer, want_dense=True):
    """-> (val_sym, idx_sym, block_ptr, dense or None) as torch CUDA tensors."""
    import torch
    st = layer.stats()
    hv = Stats  # noqa: F841 (kept for symmetry with the C names)
    v = HostView()
    _check(lib().cl_layer_host_view(layer.handle, C.byref(v)))
    dev = torch.device("cuda")
    val = torch.empty(st["entries"], dtype=torch.uint8, device=dev)
    idx = torch.empty(st["entries"], dtype=torch.uint8, device=dev)
    bp = torch.empty(st["n_blocks"] + 1, dtype=torch.int32, device=dev)
    dense = torch.empty((v.desc.M, v.desc.K), dtype=torch.float32, device=dev) if want_dense else None
    _check(lib().cl_decode_layer(layer.handle, _dev_ptr(val), _dev_ptr(idx), _dev_ptr(bp), _dev_ptr(dense), _stream()))
    return val, idx, bp, dense


def fc_workspace_bytes(layer: Layer, batch: int, path: int = PATH_AUTO) -> int:
    key = (batch, path)
    if key not in layer._ws_cache:
        n = C.c_size_t(0)
        _check(lib().cl_fc_workspace_bytes(layer.handle, batch, path, C.byref(n)))
        layer._ws_cache[key] = n.value
    return layer._ws_cache[key]


def fc_resolved_path(layer: Layer, batch: int, path: int = PATH_AUTO) -> int:
    """The path cl_compressed_fc_forward takes for (layer, batch, path)."""
    out = C.c_int32(0)
    _check(lib().cl_fc_resolved_path(layer.handle, batch, path, C.byref(out)))
    return out.value


def compressed_fc_forward(layer: Layer, X, bias=None, relu=False, path=PATH_AUTO, out=None, workspace=None):
    """X: (B, K) fp32 CUDA tensor -> Y: (B, M) fp32 CUDA tensor."""
    import torch
    M, K = layer.M, layer.K
    if X.dtype != torch.float32 or X.dim() != 2 or X.shape[1] != K:
        raise ValueError(f"X must be (B, {K}) float32")
    B = X.shape[0]
    _want(X, (B, K), "X")
    _want(bias, (M,), "bias")
    _want(out, (B, M), "out")
    Y = out if out is not None else torch.empty((B, M), dtype=torch.float32, device=X.device)
    need = fc_workspace_bytes(layer, B, path)
    if workspace is None and need:
        workspace = torch.empty(need, dtype=torch.uint8, device=X.device)
    wbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().cl_compressed_fc_forward(layer.handle, _dev_ptr(X), _dev_ptr(bias), _dev_ptr(Y), B, int(relu), path,
                                          _dev_ptr(workspace), C.c_size_t(wbytes), _stream()))
    return Y


def compressed_fc_forward_static(layer: Layer, X, out, bias=None, relu=False, path=PATH_AUTO):
    """cl_compressed_fc_forward_static: scratch in the library's static device array; the
    caller brings the output, nothing is allocated here or in the library."""
    B = X.shape[0] if X.dim() == 2 else -1
    _want(X, (B, layer.K), "X")
    _want(bias, (layer.M,), "bias")
    if out is None:
        raise ValueError("the non-allocating call needs the caller's output tensor")
    _want(out, (B, layer.M), "out")
    _check(lib().cl_compressed_fc_forward_static(layer.handle, _dev_ptr(X), _dev_ptr(bias), _dev_ptr(out), B, int(relu), path,
                                                 _stream()))
    return out


def _handles(layers):
    return (C.c_void_p * len(layers))(*[l.handle for l in layers])


def fc_stack_workspace_bytes(layers, batch: int, path: int = PATH_AUTO) -> int:
    n = C.c_size_t(0)
    _check(lib().cl_fc_stack_workspace_bytes(_handles(layers), len(layers), batch, path, C.byref(n)))
    return n.value


def compressed_fc_stack_forward(layers, X, biases=None, relu_hidden=True, relu_last=False, path=PATH_AUTO, out=None,
                                workspace=None):
    """A stack of FC layers in one call: X (B, K_0) fp32 CUDA tensor -> (B, M_last)."""
    import torch
    layers = list(layers)
    if X.dtype != torch.float32 or X.dim() != 2 or X.shape[1] != layers[0].K:
        raise ValueError(f"X must be (B, {layers[0].K}) float32")
    B = X.shape[0]
    _want(X, (B, layers[0].K), "X")
    _want(out, (B, layers[-1].M), "out")
    if biases is not None:
        if len(biases) != len(layers):
            raise ValueError("one bias (or None) per layer")
        for b, l in zip(biases, layers):
            _want(b, (l.M,), "bias")
    Y = out if out is not None else torch.empty((B, layers[-1].M), dtype=torch.float32, device=X.device)
    if workspace is None:
        workspace = torch.empty(max(256, fc_stack_workspace_bytes(layers, B, path)), dtype=torch.uint8, device=X.device)
    bias_ptrs = None
    if biases is not None:
        bias_ptrs = (C.c_void_p * len(layers))(*[None if b is None else _dev_ptr(b).value for b in biases])
    _check(lib().cl_compressed_fc_stack_forward(_handles(layers), len(layers), _dev_ptr(X), bias_ptrs, _dev_ptr(Y), B,
                                                int(relu_hidden), int(relu_last), path, _dev_ptr(workspace),
                                                C.c_size_t(workspace.numel() * workspace.element_size()), _stream()))
    return Y


class LayerGroup:
    """Several uploaded layers of one shape, run in one grid (cl_layer_group_*)."""

    def __init__(self, layers):
        self.layers = list(layers)                       # kept alive: the group holds pointers to them
        h = C.c_void_p()
        _check(lib().cl_layer_group_create(_handles(self.layers), len(self.layers), C.byref(h)))
        self.handle = h

    def free(self):
        if self.handle:
            lib().cl_layer_group_free(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass

    def workspace_bytes(self, batch: int) -> int:
        n = C.c_size_t(0)
        _check(lib().cl_fc_group_workspace_bytes(self.handle, batch, C.byref(n)))
        return n.value

    def forward(self, X, bias=None, relu=False, out=None, workspace=None):
        """X: (n, B, K) - one input per layer - or (B, K) shared by all; bias (n, M), (M,) or
        None -> (n, B, M) fp32 CUDA tensor."""
        import torch
        n, L0 = len(self.layers), self.layers[0]
        if X.dtype != torch.float32 or X.dim() not in (2, 3) or X.shape[-1] != L0.K or (X.dim() == 3 and X.shape[0] != n):
            raise ValueError(f"X must be ({n}, B, {L0.K}) or (B, {L0.K}) float32")
        B = X.shape[-2]
        _want(X, tuple(X.shape), "X")
        x_stride = B * L0.K if X.dim() == 3 else 0
        bias_stride = 0
        if bias is not None:
            if bias.dim() == 2:
                _want(bias, (n, L0.M), "bias")
                bias_stride = L0.M
            else:
                _want(bias, (L0.M,), "bias")
        _want(out, (n, B, L0.M), "out")
        Y = out if out is not None else torch.empty((n, B, L0.M), dtype=torch.float32, device=X.device)
        if workspace is None:
            workspace = torch.empty(max(256, self.workspace_bytes(B)), dtype=torch.uint8, device=X.device)
        _check(lib().cl_compressed_fc_group_forward(self.handle, _dev_ptr(X), C.c_size_t(x_stride), _dev_ptr(bias) if bias is not None else None,
                                                    C.c_size_t(bias_stride), _dev_ptr(Y), B, int(relu), _dev_ptr(workspace),
                                                    C.c_size_t(workspace.numel() * workspace.element_size()), _stream()))
        return Y


def conv_workspace_bytes(layer: Layer, conv: dict, batch: int, path: int = PATH_AUTO, compact: bool = False) -> int:
    """Scratch for the fast form of the call, or (compact) the least it works with."""
    cd = ConvDesc(conv["C"], conv["H"], conv["W"], conv["R"], conv["S"], conv["stride"], conv["pad"], conv["groups"], conv["OC"])
    n = C.c_size_t(0)
    fn = lib().cl_conv_workspace_bytes_min if compact else lib().cl_conv_workspace_bytes
    _check(fn(layer.handle, C.byref(cd), batch, path, C.byref(n)))
    return n.value


def compressed_conv_forward(layer: Layer, conv: dict, X, bias=None, relu=False, path=PATH_AUTO, out=None, workspace=None):
    """X: (B, C, H, W) fp32 CUDA tensor -> (B, OC, P, Q)."""
    import torch
    cd = ConvDesc(conv["C"], conv["H"], conv["W"], conv["R"], conv["S"], conv["stride"], conv["pad"], conv["groups"], conv["OC"])
    if X.dim() != 4:
        raise ValueError("X must be (B, C, H, W)")
    B = X.shape[0]
    P = (conv["H"] + 2 * conv["pad"] - conv["R"]) // conv["stride"] + 1
    Q = (conv["W"] + 2 * conv["pad"] - conv["S"]) // conv["stride"] + 1
    _want(X, (B, conv["C"], conv["H"], conv["W"]), "X")
    _want(bias, (conv["OC"],), "bias")
    _want(out, (B, conv["OC"], P, Q), "out")
    Y = out if out is not None else torch.empty((B, conv["OC"], P, Q), dtype=torch.float32, device=X.device)
    need = conv_workspace_bytes(layer, conv, B, path)
    if workspace is None and need:
        workspace = torch.empty(need, dtype=torch.uint8, device=X.device)
    wbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().cl_compressed_conv_forward(layer.handle, C.byref(cd), _dev_ptr(X), _dev_ptr(bias), _dev_ptr(Y), B,
                                            int(relu), path, _dev_ptr(workspace), C.c_size_t(wbytes), _stream()))
    return Y


def maxpool_forward(X, size: int, stride: int, out=None):
    """X: (B, C, H, W) fp32 CUDA tensor -> (B, C, P, Q)."""
    import torch
    if X.dtype != torch.float32 or X.dim() != 4 or not X.is_contiguous():
        raise ValueError("X must be a contiguous (B, C, H, W) float32 tensor")
    B, Cc, H, W = X.shape
    P, Q = (H - size) // stride + 1, (W - size) // stride + 1
    _want(out, (B, Cc, max(P, 0), max(Q, 0)), "out")
    if out is not None and out.data_ptr() == X.data_ptr():
        raise ValueError("pooling is not in place")
    Y = out if out is not None else torch.empty((B, Cc, max(P, 0), max(Q, 0)), dtype=torch.float32, device=X.device)
    _check(lib().cl_maxpool_forward(_dev_ptr(X), _dev_ptr(Y), B, Cc, H, W, size, stride, _stream()))
    return Y


def lrn_forward(X, n: int = 5, alpha: float = 1e-4, beta: float = 0.75, k: float = 1.0, out=None):
    """X: (B, C, H, W) fp32 CUDA tensor -> same shape."""
    import torch
    if X.dtype != torch.float32 or X.dim() != 4 or not X.is_contiguous():
        raise ValueError("X must be a contiguous (B, C, H, W) float32 tensor")
    B, Cc, H, W = X.shape
    _want(out, (B, Cc, H, W), "out")
    if out is not None and out.data_ptr() == X.data_ptr():
        raise ValueError("normalisation is not in place: neighbouring channels are read by other workgroups")
    Y = out if out is not None else torch.empty_like(X)
    _check(lib().cl_lrn_forward(_dev_ptr(X), _dev_ptr(Y), B, Cc, H, W, n, float(alpha), float(beta), float(k), _stream()))
    return Y


def plan_batches(time_ms, batch_set, in_bytes_per_image, out_bytes_per_image, ws_bytes, tot_bytes, mem_step_bytes,
                 latency_cap_ms=None):
    """-> (ms_per_image, [batch per layer]) or (inf, None) when nothing is feasible."""
    t = np.ascontiguousarray(time_ms, np.float64)
    f, nb = t.shape
    bs = np.ascontiguousarray(batch_set, np.int32)
    inb = np.ascontiguousarray(in_bytes_per_image, np.int64)
    outb = np.ascontiguousarray(out_bytes_per_image, np.int64)
    ws = np.ascontiguousarray(ws_bytes, np.int64)
    assert bs.size == nb and inb.size == f and outb.size == f and ws.size == f
    plan = np.zeros(f, np.int32)
    ms = C.c_double(0)
    rc = lib().cl_plan_batches(f, _np_ptr(bs), nb, _np_ptr(t), _np_ptr(inb), _np_ptr(outb), _np_ptr(ws), int(tot_bytes),
                               int(mem_step_bytes), float(latency_cap_ms or 0.0), _np_ptr(plan), C.byref(ms))
    if rc == CL_EUNSUPPORTED:
        return float("inf"), None
    _check(rc)
    return ms.value, plan.tolist()


def set_kernel_timing(enable: bool):
    _check(lib().cl_set_kernel_timing(int(enable)))


def last_kernel_ms():
    """-> (milliseconds, launches) of the main kernel(s) of the last forward call."""
    ms, n = C.c_float(0), C.c_int32(0)
    _check(lib().cl_last_kernel_ms(C.byref(ms), C.byref(n)))
    return ms.value, n.value
