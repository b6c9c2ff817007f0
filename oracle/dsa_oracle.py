"""ctypes front end of the CPU oracle (`dsa_oracle.c`).

TEST INFRASTRUCTURE, NOT A PRODUCT PATH: only tests, the smoke check and the
benchmark's cpu_baseline leg may import this.  It imports nothing from the HIP
package.  Arrays in, arrays out; all arithmetic lives in the C file.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from pathlib import Path

import numpy as np

_HERE = Path(__file__).resolve().parent
_SRC = _HERE / "dsa_oracle.c"
_LIB = _HERE / "libdsa_oracle.so"
_lib = None

CFLAGS = ["-O3", "-march=native", "-fopenmp", "-std=c11", "-fPIC", "-shared", "-Wall", "-Wextra"]
# DSA_ORACLE_SANITIZE=1 builds a second library with AddressSanitizer and UndefinedBehaviorSanitizer and
# loads that one (the process then needs libasan preloaded: see the sanitizer command in the design doc).
if os.environ.get("DSA_ORACLE_SANITIZE") == "1":
    CFLAGS = ["-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
              "-fopenmp", "-std=c11", "-fPIC", "-shared", "-Wall", "-Wextra"]
    _LIB = _HERE / "libdsa_oracle_san.so"


def build(force: bool = False) -> Path:
    """Compile the oracle with gcc.  Rebuilds when the source is newer than the library."""
    if force or not _LIB.exists() or _LIB.stat().st_mtime < _SRC.stat().st_mtime:
        tmp = _LIB.with_suffix(f".tmp{os.getpid()}.so")
        subprocess.run(["gcc", *CFLAGS, str(_SRC), "-o", str(tmp), "-lm"], check=True)
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(str(_LIB))
        i32, i64, f64, vp = ctypes.c_int32, ctypes.c_int64, ctypes.c_double, ctypes.c_void_p
        lib.dsao_num_threads.restype = i32
        lib.dsao_num_threads.argtypes = []
        lib.dsao_keep_from_ratio.restype = i32
        lib.dsao_keep_from_ratio.argtypes = [i32, f64]
        lib.dsao_approx_scores.restype = i32
        lib.dsao_approx_scores.argtypes = [vp, vp, i32, i32, i32, i32, vp, i64, vp]
        lib.dsao_predict_mask.restype = i32
        lib.dsao_predict_mask.argtypes = [vp, vp, i32, i32, i32, i32, i32, vp, i64, vp]
        lib.dsao_sddmm.restype = i32
        lib.dsao_sddmm.argtypes = [vp, vp, vp, i32, i32, i32, i32, i32, f64, vp, i64, vp]
        lib.dsao_sparse_softmax.restype = i32
        lib.dsao_sparse_softmax.argtypes = [vp, i64, i32, vp]
        lib.dsao_spmm.restype = i32
        lib.dsao_spmm.argtypes = [vp, vp, vp, i32, i32, i32, i32, i32, vp, i64, vp]
        lib.dsao_masked_attention.restype = i32
        lib.dsao_masked_attention.argtypes = [vp, vp, vp, vp, i32, i32, i32, i32, i32, f64,
                                              vp, i64, vp, vp, vp]
        lib.dsao_project_quantize.restype = i32
        lib.dsao_project_quantize.argtypes = [vp, vp, i64, i32, i32, vp, vp]
        lib.dsao_project_quantize_bits.restype = i32
        lib.dsao_project_quantize_bits.argtypes = [vp, vp, i64, i32, i32, i32, vp, vp]
        lib.dsao_predict_mask_threshold.restype = i32
        lib.dsao_predict_mask_threshold.argtypes = [vp, vp, i32, i32, i32, i32, i64, vp, vp]
        lib.dsao_masked_attention_csr.restype = i32
        lib.dsao_masked_attention_csr.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, i32, f64, vp, i64, vp]
        lib.dsao_project_quantize_ternary.restype = i32
        lib.dsao_project_quantize_ternary.argtypes = [vp, vp, i64, i32, i32, i32, vp, vp]
        lib.dsao_pack_codes.restype = i32
        lib.dsao_pack_codes.argtypes = [vp, i64, i32, vp]
        lib.dsao_unpack_codes.restype = i32
        lib.dsao_unpack_codes.argtypes = [vp, i64, i32, vp]
        _lib = lib
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _arr(a, dtype, ndim=None):
    a = np.ascontiguousarray(a, dtype=dtype)
    if ndim is not None and a.ndim != ndim:
        raise ValueError(f"expected {ndim} dims, got shape {a.shape}")
    return a


def _sel(sel):
    if sel is None:
        return None, 0
    s = _arr(sel, np.int64, 1)
    return s, s.size


def num_threads() -> int:
    return int(_load().dsao_num_threads())


def keep_from_ratio(L: int, ratio: float) -> int:
    return int(_load().dsao_keep_from_ratio(L, ratio))


def _flat_heads(x, dtype):
    """[B,H,L,c] or [N,L,c] -> contiguous [N,L,c]."""
    x = np.ascontiguousarray(x, dtype=dtype)
    if x.ndim == 4:
        x = x.reshape(x.shape[0] * x.shape[1], x.shape[2], x.shape[3])
    if x.ndim != 3:
        raise ValueError(f"expected [B,H,L,c] or [N,L,c], got {x.shape}")
    return x


def approx_scores(Qt, Kt, vec=1, units=None) -> np.ndarray:
    """Steps 1-2.  int64 [n_units, L]."""
    Qt, Kt = _flat_heads(Qt, np.int8), _flat_heads(Kt, np.int8)
    N, L, k = Qt.shape
    assert Kt.shape == Qt.shape
    u, nu = _sel(units)
    if u is None:
        nu = N * (L // vec)
    out = np.empty((nu, L), dtype=np.int64)
    rc = _load().dsao_approx_scores(_p(Qt), _p(Kt), N, L, k, vec, _p(u), nu, _p(out))
    if rc:
        raise ValueError("dsao_approx_scores: bad arguments")
    return out


def predict_mask(Qt, Kt, keep, vec=1, units=None) -> np.ndarray:
    """Steps 1-3.  int32 [n_units, keep] (all units of all heads, flattened, if units is None)."""
    Qt, Kt = _flat_heads(Qt, np.int8), _flat_heads(Kt, np.int8)
    N, L, k = Qt.shape
    assert Kt.shape == Qt.shape
    u, nu = _sel(units)
    if u is None:
        nu = N * (L // vec)
    out = np.empty((nu, keep), dtype=np.int32)
    rc = _load().dsao_predict_mask(_p(Qt), _p(Kt), N, L, k, vec, keep, _p(u), nu, _p(out))
    if rc:
        raise ValueError("dsao_predict_mask: bad arguments")
    return out


def _idx_full(idx, N, L, vec):
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    keep = idx.shape[-1]
    idx = idx.reshape(-1, keep)
    if idx.shape[0] != N * (L // vec):
        raise ValueError("idx must cover every unit of every head")
    if idx.size and (idx.min() < 0 or idx.max() >= L):
        raise ValueError("idx out of range")
    return idx, keep


def sddmm(Q, K, idx, scale, vec=1, rows=None) -> np.ndarray:
    """Step 4.  float64 [n_rows, keep]."""
    Q, K = _flat_heads(Q, np.float32), _flat_heads(K, np.float32)
    N, L, d = Q.shape
    idx, keep = _idx_full(idx, N, L, vec)
    r, nr = _sel(rows)
    if r is None:
        nr = N * L
    S = np.empty((nr, keep), dtype=np.float64)
    rc = _load().dsao_sddmm(_p(Q), _p(K), _p(idx), N, L, d, vec, keep, float(scale), _p(r), nr, _p(S))
    if rc:
        raise ValueError("dsao_sddmm: bad arguments")
    return S


def sparse_softmax(S) -> np.ndarray:
    """Step 5.  float64, same shape as S ([..., keep])."""
    S = np.ascontiguousarray(S, dtype=np.float64)
    keep = S.shape[-1]
    P = np.empty_like(S)
    rc = _load().dsao_sparse_softmax(_p(S), S.size // keep, keep, _p(P))
    if rc:
        raise ValueError("dsao_sparse_softmax: bad arguments")
    return P


def spmm(P, idx, V, vec=1, rows=None) -> np.ndarray:
    """Step 6.  float64 [n_rows, d]."""
    V = _flat_heads(V, np.float32)
    N, L, d = V.shape
    idx, keep = _idx_full(idx, N, L, vec)
    r, nr = _sel(rows)
    if r is None:
        nr = N * L
    P = np.ascontiguousarray(P, dtype=np.float64).reshape(nr, keep)
    O = np.empty((nr, d), dtype=np.float64)
    rc = _load().dsao_spmm(_p(P), _p(idx), _p(V), N, L, d, vec, keep, _p(r), nr, _p(O))
    if rc:
        raise ValueError("dsao_spmm: bad arguments")
    return O


def masked_attention(Q, K, V, idx, scale, vec=1, rows=None, return_sp=False):
    """Steps 4-6 given idx.  float64 O [n_rows, d] (and S, P [n_rows, keep])."""
    Q, K, V = (_flat_heads(x, np.float32) for x in (Q, K, V))
    N, L, d = Q.shape
    idx, keep = _idx_full(idx, N, L, vec)
    r, nr = _sel(rows)
    if r is None:
        nr = N * L
    O = np.empty((nr, d), dtype=np.float64)
    S = np.empty((nr, keep), dtype=np.float64) if return_sp else None
    P = np.empty((nr, keep), dtype=np.float64) if return_sp else None
    rc = _load().dsao_masked_attention(_p(Q), _p(K), _p(V), _p(idx), N, L, d, vec, keep,
                                       float(scale), _p(r), nr, _p(O), _p(S), _p(P))
    if rc:
        raise ValueError("dsao_masked_attention: bad arguments")
    return (O, S, P) if return_sp else O


def attention_fwd(Q, K, V, Qt, Kt, keep, scale, vec=1):
    """Whole path, all rows.  Returns (O float64 [N*L, d], idx int32 [N*L/vec, keep])."""
    idx = predict_mask(Qt, Kt, keep, vec)
    return masked_attention(Q, K, V, idx, scale, vec), idx


def predict_mask_threshold(Qt, Kt, theta, vec=1):
    """Step 3' (threshold mask).  Returns (row_ptr int64 [n_units + 1], col int32 [nnz]): unit u keeps the keys
    col[row_ptr[u]:row_ptr[u+1]], ascending: every key with score >= theta, or its single best key if none."""
    Qt, Kt = _flat_heads(Qt, np.int8), _flat_heads(Kt, np.int8)
    N, L, k = Qt.shape
    assert Kt.shape == Qt.shape
    row_ptr = np.zeros(N * (L // vec) + 1, dtype=np.int64)
    if _load().dsao_predict_mask_threshold(_p(Qt), _p(Kt), N, L, k, vec, int(theta), _p(row_ptr), None):
        raise ValueError("dsao_predict_mask_threshold: bad arguments")
    col = np.empty(int(row_ptr[-1]), dtype=np.int32)
    if _load().dsao_predict_mask_threshold(_p(Qt), _p(Kt), N, L, k, vec, int(theta), _p(row_ptr), _p(col)):
        raise ValueError("dsao_predict_mask_threshold: bad arguments")
    return row_ptr, col


def masked_attention_csr(Q, K, V, row_ptr, col, scale, vec=1, rows=None):
    """Steps 4-6 for a CSR mask.  float64 O [n_rows, d]."""
    Q, K, V = (_flat_heads(x, np.float32) for x in (Q, K, V))
    N, L, d = Q.shape
    row_ptr = _arr(row_ptr, np.int64, 1)
    col = _arr(col, np.int32, 1)
    assert row_ptr.size == N * (L // vec) + 1 and row_ptr[-1] == col.size
    r, nr = _sel(rows)
    if r is None:
        nr = N * L
    O = np.empty((nr, d), dtype=np.float64)
    if _load().dsao_masked_attention_csr(_p(Q), _p(K), _p(V), _p(row_ptr), _p(col), N, L, d, vec, float(scale),
                                         _p(r), nr, _p(O)):
        raise ValueError("dsao_masked_attention_csr: bad arguments")
    return O


def project_quantize(X, R, bits=8):
    """Step 0.  X [..., d] float32 (bf16 inputs widened exactly), R [d, k] float32.
    Returns (int8 [..., k] with |code| <= 2^(bits-1) - 1, amax float32)."""
    X = np.ascontiguousarray(X, dtype=np.float32)
    R = np.ascontiguousarray(R, dtype=np.float32)
    d, k = R.shape
    if X.shape[-1] != d:
        raise ValueError("X and R do not match")
    rows = X.size // d
    out = np.empty(X.shape[:-1] + (k,), dtype=np.int8)
    amax = np.zeros(1, dtype=np.float32)
    rc = _load().dsao_project_quantize_bits(_p(X), _p(R), rows, d, k, int(bits), _p(out), _p(amax))
    if rc:
        raise ValueError("dsao_project_quantize_bits: bad arguments")
    return out, np.float32(amax[0])


def project_quantize_ternary(X, P3, bits=8):
    """Step 0 with a ternary projection (equation 5).  X [..., d] float32, P3 [d, k] int8 in {-1, 0, 1}.
    Returns (codes int8 [..., k], amax)."""
    X = np.ascontiguousarray(X, dtype=np.float32)
    P3 = _arr(P3, np.int8, 2)
    d, k = P3.shape
    assert X.shape[-1] == d
    rows = X.size // d
    Xt = np.empty(X.shape[:-1] + (k,), dtype=np.int8)
    amax = np.zeros(1, dtype=np.float32)
    rc = _load().dsao_project_quantize_ternary(_p(X), _p(P3), rows, d, k, bits, _p(Xt), _p(amax))
    if rc:
        raise ValueError("dsao_project_quantize_ternary: bad arguments" if rc == 1 else "P3 has entries outside {-1, 0, 1}")
    return Xt, float(amax[0])


def pack_codes(codes, bits):
    """int8 codes [..., k] -> uint8 [..., k*bits/8] (8/bits codes per byte, low field first)."""
    codes = np.ascontiguousarray(codes, dtype=np.int8)
    per = 8 // bits
    out = np.empty(codes.shape[:-1] + (codes.shape[-1] // per,), dtype=np.uint8)
    rc = _load().dsao_pack_codes(_p(codes), codes.size, int(bits), _p(out))
    if rc:
        raise ValueError("dsao_pack_codes: bad arguments" if rc == 1 else "dsao_pack_codes: code out of range")
    return out


def unpack_codes(packed, bits):
    """Inverse of pack_codes."""
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    per = 8 // bits
    out = np.empty(packed.shape[:-1] + (packed.shape[-1] * per,), dtype=np.int8)
    rc = _load().dsao_unpack_codes(_p(packed), out.size, int(bits), _p(out))
    if rc:
        raise ValueError("dsao_unpack_codes: bad arguments")
    return out
