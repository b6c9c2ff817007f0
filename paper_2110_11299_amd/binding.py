"""Thin ctypes binding of libdsa_hip.so: argument marshalling only.

Every function takes torch CUDA tensors (PyTorch owns device memory and streams), passes
their device pointers and the current stream through the C ABI declared in include/dsa.h
and returns the output tensors.  There is no fallback: without the built library, or on a
failed status, these raise.
"""
from __future__ import annotations

import ctypes
from pathlib import Path

_LIB_PATH = Path(__file__).resolve().parent / "libdsa_hip.so"
_lib = None

DSA_OK = 0
DSA_F32, DSA_BF16 = 0, 1

EXPORTS = [
    "dsa_keep_from_ratio", "dsa_workspace_bytes", "dsa_predict_mask", "dsa_sddmm", "dsa_sparse_softmax",
    "dsa_spmm", "dsa_masked_attention", "dsa_attention_fwd", "dsa_attention_fwd_noalloc",
    "dsa_noalloc_max_mask_bytes", "dsa_approx_rowmax", "dsa_mfma_i8_sustained", "dsa_gather_roof",
    "dsa_threshold_workspace_bytes", "dsa_predict_mask_threshold", "dsa_masked_attention_csr",
    "dsa_project_quantize", "dsa_project_workspace_bytes",
    "dsa_project_quantize_bits", "dsa_project_quantize_ternary", "dsa_predict_workspace_bytes_bits", "dsa_predict_mask_bits",
    "dsa_workspace_bytes_bits", "dsa_attention_fwd_bits",
    "dsa_status_string", "dsa_version",
]


class DsaShape(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("H", ctypes.c_int32), ("L", ctypes.c_int32), ("d", ctypes.c_int32),
                ("k", ctypes.c_int32), ("keep", ctypes.c_int32), ("vec", ctypes.c_int32),
                ("dtype", ctypes.c_int32), ("scale", ctypes.c_float)]


class DsaError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


def lib():
    """The loaded C-ABI library.  Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not _LIB_PATH.exists():
            raise RuntimeError(f"{_LIB_PATH} is missing: build it first (python -m paper_2110_11299_amd.build "
                               "or __graft_entry__.build()); there is no fallback path")
        # PyTorch ships its own HIP runtime under the same soname as the system one.  Import it
        # first, so that this library binds to the runtime that owns torch's streams and memory
        # instead of pulling a second runtime into the process.
        import torch  # noqa: F401
        L = ctypes.CDLL(str(_LIB_PATH))
        vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
        shp = ctypes.POINTER(DsaShape)
        L.dsa_keep_from_ratio.restype = i32
        L.dsa_keep_from_ratio.argtypes = [i32, ctypes.c_double]
        L.dsa_workspace_bytes.restype = sz
        L.dsa_workspace_bytes.argtypes = [shp]
        L.dsa_predict_mask.restype = i32
        L.dsa_predict_mask.argtypes = [shp, vp, vp, vp, vp, sz, vp]
        L.dsa_sddmm.restype = i32
        L.dsa_sddmm.argtypes = [shp, vp, vp, vp, vp, vp]
        L.dsa_sparse_softmax.restype = i32
        L.dsa_sparse_softmax.argtypes = [shp, vp, vp, vp]
        L.dsa_spmm.restype = i32
        L.dsa_spmm.argtypes = [shp, vp, vp, vp, vp, vp]
        L.dsa_masked_attention.restype = i32
        L.dsa_masked_attention.argtypes = [shp, vp, vp, vp, vp, vp, vp]
        L.dsa_attention_fwd.restype = i32
        L.dsa_attention_fwd.argtypes = [shp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.dsa_attention_fwd_noalloc.restype = i32
        L.dsa_attention_fwd_noalloc.argtypes = [shp, vp, vp, vp, vp, vp, vp, vp]
        L.dsa_noalloc_max_mask_bytes.restype = sz
        L.dsa_noalloc_max_mask_bytes.argtypes = []
        L.dsa_approx_rowmax.restype = i32
        L.dsa_approx_rowmax.argtypes = [shp, vp, vp, vp, vp]
        L.dsa_project_workspace_bytes.restype = sz
        L.dsa_project_workspace_bytes.argtypes = [shp]
        L.dsa_project_quantize.restype = i32
        L.dsa_project_quantize.argtypes = [shp, vp, vp, vp, vp, vp, sz, vp]
        L.dsa_project_quantize_bits.restype = i32
        L.dsa_project_quantize_bits.argtypes = [shp, i32, vp, vp, vp, vp, vp, sz, vp]
        L.dsa_project_quantize_ternary.restype = i32
        L.dsa_project_quantize_ternary.argtypes = [shp, i32, vp, vp, vp, vp, vp, sz, vp]
        L.dsa_predict_workspace_bytes_bits.restype = sz
        L.dsa_predict_workspace_bytes_bits.argtypes = [shp, i32]
        L.dsa_predict_mask_bits.restype = i32
        L.dsa_predict_mask_bits.argtypes = [shp, i32, vp, vp, vp, vp, sz, vp]
        L.dsa_workspace_bytes_bits.restype = sz
        L.dsa_workspace_bytes_bits.argtypes = [shp, i32]
        L.dsa_attention_fwd_bits.restype = i32
        L.dsa_attention_fwd_bits.argtypes = [shp, i32, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.dsa_mfma_i8_sustained.restype = i32
        L.dsa_mfma_i8_sustained.argtypes = [i32, i32, vp, vp]
        L.dsa_threshold_workspace_bytes.restype = sz
        L.dsa_threshold_workspace_bytes.argtypes = [shp]
        L.dsa_predict_mask_threshold.restype = i32
        L.dsa_predict_mask_threshold.argtypes = [shp, vp, vp, i32, vp, vp, ctypes.c_int64, vp, sz, vp]
        L.dsa_masked_attention_csr.restype = i32
        L.dsa_masked_attention_csr.argtypes = [shp, vp, vp, vp, vp, vp, vp, vp]
        L.dsa_gather_roof.restype = i32
        L.dsa_gather_roof.argtypes = [shp, vp, vp, vp, vp, vp]
        L.dsa_status_string.restype = ctypes.c_char_p
        L.dsa_status_string.argtypes = [i32]
        L.dsa_version.restype = ctypes.c_char_p
        L.dsa_version.argtypes = []
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().dsa_status_string(status).decode()


def version() -> str:
    return lib().dsa_version().decode()


def keep_from_ratio(L: int, ratio: float) -> int:
    return int(lib().dsa_keep_from_ratio(L, ratio))


def make_shape(B, H, L, d, k, keep, vec, dtype, scale) -> DsaShape:
    return DsaShape(B, H, L, d, k, keep, vec, dtype, scale)


def workspace_bytes(shape: DsaShape) -> int:
    return int(lib().dsa_workspace_bytes(ctypes.byref(shape)))


def project_workspace_bytes(shape: DsaShape) -> int:
    return int(lib().dsa_project_workspace_bytes(ctypes.byref(shape)))


def predict_workspace_bytes_bits(shape: DsaShape, bits: int) -> int:
    return int(lib().dsa_predict_workspace_bytes_bits(ctypes.byref(shape), bits))


def _check(status: int, where: str):
    if status != DSA_OK:
        raise DsaError(status, where)


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    import torch
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dev(t, dtype, shape):
    import torch
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.is_contiguous() and t.dtype == dtype
            and tuple(t.shape) == tuple(shape)):
        raise ValueError(f"expected a contiguous CUDA tensor {dtype} {tuple(shape)}, got "
                         f"{getattr(t, 'dtype', type(t))} {tuple(getattr(t, 'shape', ()))}")
    return t


def _qkv_dtype(shape: DsaShape):
    import torch
    return torch.float32 if shape.dtype == DSA_F32 else torch.bfloat16


def _dims(s: DsaShape):
    return (s.B, s.H, s.L, s.d), (s.B, s.H, s.L, s.k), (s.B, s.H, s.L // s.vec, s.keep), (s.B, s.H, s.L, s.keep)


def alloc_workspace(shape: DsaShape, device="cuda"):
    import torch
    n = workspace_bytes(shape)
    return torch.empty(max(n, 16), dtype=torch.uint8, device=device)


def dsa_predict_mask(shape, Qt, Kt, idx=None, ws=None):
    import torch
    _, tk, ti, _ = _dims(shape)
    _dev(Qt, torch.int8, tk); _dev(Kt, torch.int8, tk)
    idx = torch.empty(ti, dtype=torch.int32, device=Qt.device) if idx is None else _dev(idx, torch.int32, ti)
    ws = alloc_workspace(shape, Qt.device) if ws is None else ws
    _check(lib().dsa_predict_mask(ctypes.byref(shape), _ptr(Qt), _ptr(Kt), _ptr(idx), _ptr(ws),
                                  ws.numel(), _stream()), "dsa_predict_mask")
    return idx


def dsa_sddmm(shape, Q, K, idx, S=None):
    import torch
    tq, _, ti, ts = _dims(shape)
    dt = _qkv_dtype(shape)
    _dev(Q, dt, tq); _dev(K, dt, tq); _dev(idx, torch.int32, ti)
    S = torch.empty(ts, dtype=torch.float32, device=Q.device) if S is None else _dev(S, torch.float32, ts)
    _check(lib().dsa_sddmm(ctypes.byref(shape), _ptr(Q), _ptr(K), _ptr(idx), _ptr(S), _stream()), "dsa_sddmm")
    return S


def dsa_sparse_softmax(shape, S, P=None):
    import torch
    _, _, _, ts = _dims(shape)
    _dev(S, torch.float32, ts)
    P = torch.empty_like(S) if P is None else _dev(P, torch.float32, ts)
    _check(lib().dsa_sparse_softmax(ctypes.byref(shape), _ptr(S), _ptr(P), _stream()), "dsa_sparse_softmax")
    return P


def dsa_spmm(shape, P, idx, V, O=None):
    import torch
    tq, _, ti, ts = _dims(shape)
    _dev(P, torch.float32, ts); _dev(idx, torch.int32, ti); _dev(V, _qkv_dtype(shape), tq)
    O = torch.empty(tq, dtype=torch.float32, device=V.device) if O is None else _dev(O, torch.float32, tq)
    _check(lib().dsa_spmm(ctypes.byref(shape), _ptr(P), _ptr(idx), _ptr(V), _ptr(O), _stream()), "dsa_spmm")
    return O


def dsa_masked_attention(shape, Q, K, V, idx, O=None):
    import torch
    tq, _, ti, _ = _dims(shape)
    dt = _qkv_dtype(shape)
    _dev(Q, dt, tq); _dev(K, dt, tq); _dev(V, dt, tq); _dev(idx, torch.int32, ti)
    O = torch.empty(tq, dtype=torch.float32, device=Q.device) if O is None else _dev(O, torch.float32, tq)
    _check(lib().dsa_masked_attention(ctypes.byref(shape), _ptr(Q), _ptr(K), _ptr(V), _ptr(idx), _ptr(O),
                                      _stream()), "dsa_masked_attention")
    return O


def dsa_attention_fwd(shape, Q, K, V, Qt, Kt, O=None, idx_out=None, ws=None, want_idx=True):
    """Returns (O, idx); idx is None when want_idx is False and no idx_out was given."""
    import torch
    tq, tk, ti, _ = _dims(shape)
    dt = _qkv_dtype(shape)
    _dev(Q, dt, tq); _dev(K, dt, tq); _dev(V, dt, tq); _dev(Qt, torch.int8, tk); _dev(Kt, torch.int8, tk)
    O = torch.empty(tq, dtype=torch.float32, device=Q.device) if O is None else _dev(O, torch.float32, tq)
    if idx_out is None and want_idx:
        idx_out = torch.empty(ti, dtype=torch.int32, device=Q.device)
    elif idx_out is not None:
        _dev(idx_out, torch.int32, ti)
    ws = alloc_workspace(shape, Q.device) if ws is None else ws
    _check(lib().dsa_attention_fwd(ctypes.byref(shape), _ptr(Q), _ptr(K), _ptr(V), _ptr(Qt), _ptr(Kt),
                                   _ptr(O), _ptr(idx_out), _ptr(ws), ws.numel(), _stream()),
           "dsa_attention_fwd")
    return O, idx_out


def noalloc_max_mask_bytes() -> int:
    return int(lib().dsa_noalloc_max_mask_bytes())


def dsa_attention_fwd_noalloc(shape, Q, K, V, Qt, Kt, O):
    """Whole path with the mask in the library's fixed device array; O must be given (the call
    itself allocates nothing)."""
    import torch
    tq, tk, _, _ = _dims(shape)
    dt = _qkv_dtype(shape)
    _dev(Q, dt, tq); _dev(K, dt, tq); _dev(V, dt, tq); _dev(Qt, torch.int8, tk); _dev(Kt, torch.int8, tk)
    _dev(O, torch.float32, tq)
    _check(lib().dsa_attention_fwd_noalloc(ctypes.byref(shape), _ptr(Q), _ptr(K), _ptr(V), _ptr(Qt), _ptr(Kt),
                                           _ptr(O), _stream()), "dsa_attention_fwd_noalloc")
    return O


def dsa_approx_rowmax(shape, Qt, Kt, rowmax=None):
    import torch
    _, tk, _, _ = _dims(shape)
    _dev(Qt, torch.int8, tk); _dev(Kt, torch.int8, tk)
    tr = (shape.B, shape.H, shape.L)
    rowmax = torch.empty(tr, dtype=torch.int32, device=Qt.device) if rowmax is None else _dev(rowmax, torch.int32, tr)
    _check(lib().dsa_approx_rowmax(ctypes.byref(shape), _ptr(Qt), _ptr(Kt), _ptr(rowmax), _stream()),
           "dsa_approx_rowmax")
    return rowmax


def dsa_mfma_i8_sustained(blocks: int, iters: int, sink=None):
    """Launches the pure int8 MFMA stream; returns the number of int8 operations it performs."""
    import torch
    if sink is None:
        sink = torch.empty(blocks * 256, dtype=torch.int32, device="cuda")
    _dev(sink, torch.int32, (blocks * 256,))
    _check(lib().dsa_mfma_i8_sustained(blocks, iters, _ptr(sink), _stream()), "dsa_mfma_i8_sustained")
    return 4 * blocks * 4 * iters * 65536


def threshold_workspace_bytes(shape: DsaShape) -> int:
    return int(lib().dsa_threshold_workspace_bytes(ctypes.byref(shape)))


def dsa_predict_mask_threshold(shape, Qt, Kt, theta, col_capacity, row_ptr=None, col=None, ws=None):
    """Threshold mask in CSR form.  Returns (row_ptr int32 [units + 1], col int32 [col_capacity]); the entries of
    col beyond row_ptr[-1] are not written, and nothing beyond col_capacity is."""
    import torch
    _, tk, _, _ = _dims(shape)
    _dev(Qt, torch.int8, tk); _dev(Kt, torch.int8, tk)
    units = shape.B * shape.H * (shape.L // shape.vec)
    row_ptr = torch.empty(units + 1, dtype=torch.int32, device=Qt.device) if row_ptr is None \
        else _dev(row_ptr, torch.int32, (units + 1,))
    col = torch.empty(max(col_capacity, 4), dtype=torch.int32, device=Qt.device) if col is None else col
    if ws is None:
        ws = torch.empty(max(threshold_workspace_bytes(shape), 16), dtype=torch.uint8, device=Qt.device)
    _check(lib().dsa_predict_mask_threshold(ctypes.byref(shape), _ptr(Qt), _ptr(Kt), int(theta), _ptr(row_ptr), _ptr(col),
                                            int(col_capacity), _ptr(ws), ws.numel(), _stream()),
           "dsa_predict_mask_threshold")
    return row_ptr, col


def dsa_masked_attention_csr(shape, Q, K, V, row_ptr, col, O=None):
    import torch
    tq, _, _, _ = _dims(shape)
    dt = _qkv_dtype(shape)
    _dev(Q, dt, tq); _dev(K, dt, tq); _dev(V, dt, tq)
    _dev(row_ptr, torch.int32, (shape.B * shape.H * (shape.L // shape.vec) + 1,))
    O = torch.empty(tq, dtype=torch.float32, device=Q.device) if O is None else _dev(O, torch.float32, tq)
    _check(lib().dsa_masked_attention_csr(ctypes.byref(shape), _ptr(Q), _ptr(K), _ptr(V), _ptr(row_ptr), _ptr(col),
                                          _ptr(O), _stream()), "dsa_masked_attention_csr")
    return O


def dsa_gather_roof(shape, K, V, idx, sink=None):
    """Launches the gather-only twin of the fine-grained attention kernel; returns the gathered bytes."""
    import torch
    tq, _, ti, _ = _dims(shape)
    dt = _qkv_dtype(shape)
    _dev(K, dt, tq); _dev(V, dt, tq); _dev(idx, torch.int32, ti)
    n = shape.B * shape.H * shape.L * 64
    sink = torch.empty(n, dtype=torch.int32, device=K.device) if sink is None else _dev(sink, torch.int32, (n,))
    _check(lib().dsa_gather_roof(ctypes.byref(shape), _ptr(K), _ptr(V), _ptr(idx), _ptr(sink), _stream()),
           "dsa_gather_roof")
    return 2 * shape.B * shape.H * shape.L * shape.keep * shape.d * K.element_size()


def dsa_project_quantize(shape, X, R, Xt=None, ws=None, want_amax=True):
    """Returns (Xt int8 [B,H,L,k], amax float tensor of one element or None)."""
    import torch
    tq, tk, _, _ = _dims(shape)
    _dev(X, _qkv_dtype(shape), tq); _dev(R, torch.float32, (shape.d, shape.k))
    Xt = torch.empty(tk, dtype=torch.int8, device=X.device) if Xt is None else _dev(Xt, torch.int8, tk)
    need = project_workspace_bytes(shape)
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device=X.device) if ws is None else ws
    amax = torch.empty(1, dtype=torch.float32, device=X.device) if want_amax else None
    _check(lib().dsa_project_quantize(ctypes.byref(shape), _ptr(X), _ptr(R), _ptr(Xt), _ptr(amax), _ptr(ws),
                                      ws.numel(), _stream()), "dsa_project_quantize")
    return Xt, amax


def _packed_dims(shape: DsaShape, bits: int):
    return (shape.B, shape.H, shape.L, shape.k * bits // 8)


def dsa_project_quantize_bits(shape, bits, X, R, Xt=None, ws=None, want_amax=True):
    """Returns (packed codes uint8 [B,H,L,k*bits/8], amax float tensor of one element or None)."""
    import torch
    tq, _, _, _ = _dims(shape)
    tp = _packed_dims(shape, bits)
    _dev(X, _qkv_dtype(shape), tq); _dev(R, torch.float32, (shape.d, shape.k))
    Xt = torch.empty(tp, dtype=torch.uint8, device=X.device) if Xt is None else _dev(Xt, torch.uint8, tp)
    need = project_workspace_bytes(shape)
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device=X.device) if ws is None else ws
    amax = torch.empty(1, dtype=torch.float32, device=X.device) if want_amax else None
    _check(lib().dsa_project_quantize_bits(ctypes.byref(shape), bits, _ptr(X), _ptr(R), _ptr(Xt), _ptr(amax),
                                           _ptr(ws), ws.numel(), _stream()), "dsa_project_quantize_bits")
    return Xt, amax


def dsa_project_quantize_ternary(shape, bits, X, P3, Xt=None, ws=None, want_amax=True):
    """Projection with a ternary matrix P3 (int8 [d,k] in {-1,0,1}).  Returns (packed codes uint8, amax or None)."""
    import torch
    tq, _, _, _ = _dims(shape)
    tp = _packed_dims(shape, bits)
    _dev(X, _qkv_dtype(shape), tq); _dev(P3, torch.int8, (shape.d, shape.k))
    Xt = torch.empty(tp, dtype=torch.uint8, device=X.device) if Xt is None else _dev(Xt, torch.uint8, tp)
    need = project_workspace_bytes(shape)
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device=X.device) if ws is None else ws
    amax = torch.empty(1, dtype=torch.float32, device=X.device) if want_amax else None
    _check(lib().dsa_project_quantize_ternary(ctypes.byref(shape), bits, _ptr(X), _ptr(P3), _ptr(Xt), _ptr(amax),
                                              _ptr(ws), ws.numel(), _stream()), "dsa_project_quantize_ternary")
    return Xt, amax


def dsa_predict_mask_bits(shape, bits, Qt, Kt, idx=None, ws=None):
    """Mask from packed low-precision codes (uint8 [B,H,L,k*bits/8])."""
    import torch
    _, _, ti, _ = _dims(shape)
    tp = _packed_dims(shape, bits)
    _dev(Qt, torch.uint8, tp); _dev(Kt, torch.uint8, tp)
    idx = torch.empty(ti, dtype=torch.int32, device=Qt.device) if idx is None else _dev(idx, torch.int32, ti)
    if ws is None:
        ws = torch.empty(max(predict_workspace_bytes_bits(shape, bits), 16), dtype=torch.uint8, device=Qt.device)
    _check(lib().dsa_predict_mask_bits(ctypes.byref(shape), bits, _ptr(Qt), _ptr(Kt), _ptr(idx), _ptr(ws),
                                       ws.numel(), _stream()), "dsa_predict_mask_bits")
    return idx


def workspace_bytes_bits(shape: DsaShape, bits: int) -> int:
    return int(lib().dsa_workspace_bytes_bits(ctypes.byref(shape), bits))


def dsa_attention_fwd_bits(shape, bits, Q, K, V, Qt, Kt, O=None, idx_out=None, ws=None, want_idx=True):
    """Whole path from packed low-precision codes.  Returns (O, idx or None)."""
    import torch
    tq, _, ti, _ = _dims(shape)
    tp = _packed_dims(shape, bits)
    dt = _qkv_dtype(shape)
    _dev(Q, dt, tq); _dev(K, dt, tq); _dev(V, dt, tq); _dev(Qt, torch.uint8, tp); _dev(Kt, torch.uint8, tp)
    O = torch.empty(tq, dtype=torch.float32, device=Q.device) if O is None else _dev(O, torch.float32, tq)
    if idx_out is None and want_idx:
        idx_out = torch.empty(ti, dtype=torch.int32, device=Q.device)
    elif idx_out is not None:
        _dev(idx_out, torch.int32, ti)
    if ws is None:
        ws = torch.empty(max(workspace_bytes_bits(shape, bits), 16), dtype=torch.uint8, device=Q.device)
    _check(lib().dsa_attention_fwd_bits(ctypes.byref(shape), bits, _ptr(Q), _ptr(K), _ptr(V), _ptr(Qt), _ptr(Kt),
                                        _ptr(O), _ptr(idx_out), _ptr(ws), ws.numel(), _stream()),
           "dsa_attention_fwd_bits")
    return O, idx_out
