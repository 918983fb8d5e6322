"""ctypes front end of the CPU oracle (``autosage_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by the
benchmark's CPU-baseline leg.  The GPU library and its Python binding never
import this package, and this package never imports them.

All functions take host NumPy arrays and return float64 / integer NumPy arrays.
bf16 operands are passed as ``uint16`` bit patterns, IEEE fp16 operands as ``numpy.float16`` arrays (widened
to float32, which holds every fp16 value exactly, before the C code sees them).
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "autosage_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None

F32, BF16 = 0, 1


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (OpenMP over rows) into oracle/liboracle.so."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c99", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        lib.oracle_graph_signature.restype = ctypes.c_uint64
        lib.oracle_num_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _dense(a):
    a = np.ascontiguousarray(a)
    if a.dtype == np.float32:
        return a, F32
    if a.dtype == np.uint16:
        return a, BF16
    if a.dtype == np.float16:
        return np.ascontiguousarray(a.astype(np.float32)), F32
    raise TypeError("dense operands must be float32, float16 or uint16 (bf16 bits), got %s" % a.dtype)


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def spmm(rowptr, colind, val, B) -> np.ndarray:
    """C = A B in float64; A is (rowptr, colind, val), B is [n_cols, F]."""
    lib = _load()
    rowptr, colind = _i32(rowptr), _i32(colind)
    val = np.ascontiguousarray(val, dtype=np.float32)
    B, dt = _dense(B)
    n_rows, F = rowptr.shape[0] - 1, B.shape[1]
    C = np.zeros((n_rows, F), dtype=np.float64)
    rc = lib.oracle_spmm(ctypes.c_int64(n_rows), _p(rowptr), _p(colind), _p(val), _p(B),
                         ctypes.c_int64(F), ctypes.c_int32(F), ctypes.c_int(dt), _p(C), ctypes.c_int64(F))
    assert rc == 0
    return C


def sddmm(rowptr, colind, X, Y) -> np.ndarray:
    """out[p] = <X[i,:], Y[colind[p],:]> in CSR order, float64."""
    lib = _load()
    rowptr, colind = _i32(rowptr), _i32(colind)
    X, dt = _dense(X)
    Y, dt2 = _dense(Y)
    assert dt == dt2 and X.shape[1] == Y.shape[1]
    n_rows, F = rowptr.shape[0] - 1, X.shape[1]
    out = np.zeros(int(rowptr[-1]), dtype=np.float64)
    rc = lib.oracle_sddmm(ctypes.c_int64(n_rows), _p(rowptr), _p(colind), _p(X), ctypes.c_int64(F),
                          _p(Y), ctypes.c_int64(F), ctypes.c_int32(F), ctypes.c_int(dt), _p(out))
    assert rc == 0
    return out


def row_softmax(rowptr, s) -> np.ndarray:
    """Row-softmax over the stored entries; s is [nnz] or [nnz, H]; returns the same shape, float64."""
    lib = _load()
    rowptr = _i32(rowptr)
    s = np.ascontiguousarray(s, dtype=np.float64)
    H = 1 if s.ndim == 1 else s.shape[1]
    out = np.zeros_like(s)
    rc = lib.oracle_row_softmax(ctypes.c_int64(rowptr.shape[0] - 1), _p(rowptr), _p(s), ctypes.c_int32(H), _p(out))
    assert rc == 0
    return out


def csr_attention(rowptr, colind, Q, K, V, scale, return_scores: bool = False):
    """O = softmax_row(scale * SDDMM(Q, K)) V on the pattern; Q is [n_rows, H, d], K and V are [n_cols, H, d]."""
    lib = _load()
    rowptr, colind = _i32(rowptr), _i32(colind)
    Q, dt = _dense(Q)
    K, dt2 = _dense(K)
    V, dt3 = _dense(V)
    assert dt == dt2 == dt3 and Q.ndim == 3 and K.shape == V.shape and K.shape[1:] == Q.shape[1:]
    N, H, d = Q.shape
    assert colind.size == 0 or int(colind.max()) < K.shape[0]
    assert rowptr.shape[0] == N + 1
    nnz = int(rowptr[-1])
    O = np.zeros((N, H, d), dtype=np.float64)
    S = np.zeros((nnz, H), dtype=np.float64) if return_scores else None
    P = np.zeros((nnz, H), dtype=np.float64) if return_scores else None
    rc = lib.oracle_csr_attention(ctypes.c_int64(N), _p(rowptr), _p(colind), _p(Q), _p(K), _p(V),
                                  ctypes.c_int32(H), ctypes.c_int32(d), ctypes.c_double(scale), ctypes.c_int(dt),
                                  _p(S) if return_scores else None, _p(P) if return_scores else None, _p(O))
    assert rc == 0
    return (O, S, P) if return_scores else O


def hub_partition(rowptr, hub_t: int, hub_chunk: int):
    """Returns (hub_rows, chunk_ptr, light_rows) as int32 arrays."""
    lib = _load()
    rowptr = _i32(rowptr)
    n = rowptr.shape[0] - 1
    hub_rows = np.zeros(max(n, 1), dtype=np.int32)
    light_rows = np.zeros(max(n, 1), dtype=np.int32)
    chunk_ptr = np.zeros(n + 1, dtype=np.int32)
    nh, nl = ctypes.c_int32(0), ctypes.c_int32(0)
    rc = lib.oracle_hub_partition(ctypes.c_int64(n), _p(rowptr), ctypes.c_int32(hub_t), ctypes.c_int32(hub_chunk),
                                  ctypes.byref(nh), _p(hub_rows), _p(chunk_ptr), ctypes.byref(nl), _p(light_rows))
    if rc != 0:
        raise ValueError("hub_t and hub_chunk must be >= 1")
    return hub_rows[:nh.value].copy(), chunk_ptr[:nh.value + 1].copy(), light_rows[:nl.value].copy()


def degree_histogram(rowptr):
    """Returns (hist int64[33], max_deg)."""
    lib = _load()
    rowptr = _i32(rowptr)
    hist = np.zeros(33, dtype=np.int64)
    mx = ctypes.c_int64(0)
    lib.oracle_degree_histogram(ctypes.c_int64(rowptr.shape[0] - 1), _p(rowptr), _p(hist), ctypes.byref(mx))
    return hist, int(mx.value)


def graph_signature(rowptr, n_cols: int) -> int:
    lib = _load()
    rowptr = _i32(rowptr)
    return int(lib.oracle_graph_signature(ctypes.c_int64(rowptr.shape[0] - 1), ctypes.c_int64(n_cols), _p(rowptr)))


def decide(t_cand, t_baseline: float, alpha: float) -> int:
    """Index of the accepted candidate, or -1 when the guardrail keeps the baseline."""
    lib = _load()
    t = np.ascontiguousarray(t_cand, dtype=np.float64)
    return int(lib.oracle_decide(ctypes.c_int32(t.shape[0]), _p(t), ctypes.c_double(t_baseline), ctypes.c_double(alpha)))


def csr_transpose(rowptr, colind, val, n_cols: int):
    """A^T as CSR: returns (t_rowptr, t_colind, t_val, perm); stable (source rows ascending inside a row of A^T)."""
    lib = _load()
    rowptr, colind = _i32(rowptr), _i32(colind)
    val = np.ascontiguousarray(val, dtype=np.float32)
    n_rows, nnz = rowptr.shape[0] - 1, int(rowptr[-1])
    t_rowptr = np.zeros(n_cols + 1, dtype=np.int32)
    t_colind = np.zeros(max(nnz, 1), dtype=np.int32)
    t_val = np.zeros(max(nnz, 1), dtype=np.float32)
    perm = np.zeros(max(nnz, 1), dtype=np.int32)
    rc = lib.oracle_csr_transpose(ctypes.c_int64(n_rows), ctypes.c_int64(n_cols), _p(rowptr), _p(colind), _p(val),
                                  _p(t_rowptr), _p(t_colind), _p(t_val), _p(perm))
    assert rc == 0
    return t_rowptr, t_colind[:nnz], t_val[:nnz], perm[:nnz]


def row_softmax_backward(rowptr, P, dP) -> np.ndarray:
    """dS = P * (dP - rowsum(P * dP)) over the stored entries of each row (and head); float64."""
    lib = _load()
    rowptr = _i32(rowptr)
    P = np.ascontiguousarray(P, dtype=np.float64)
    dP = np.ascontiguousarray(dP, dtype=np.float64)
    assert P.shape == dP.shape
    H = 1 if P.ndim == 1 else P.shape[1]
    dS = np.zeros_like(P)
    rc = lib.oracle_row_softmax_backward(ctypes.c_int64(rowptr.shape[0] - 1), _p(rowptr), _p(P), _p(dP), ctypes.c_int32(H),
                                         _p(dS))
    assert rc == 0
    return dS


def csr_attention_backward(rowptr, colind, Q, K, V, dO, scale):
    """(dQ, dK, dV) of csr_attention for the upstream gradient dO [N, H, d]; float64 arrays [N, H, d]."""
    lib = _load()
    rowptr, colind = _i32(rowptr), _i32(colind)
    Q, dt = _dense(Q)
    K, dt2 = _dense(K)
    V, dt3 = _dense(V)
    assert dt == dt2 == dt3 and Q.ndim == 3 and Q.shape == K.shape == V.shape
    N, H, d = Q.shape
    dO = np.ascontiguousarray(dO, dtype=np.float64)
    assert dO.shape == (N, H, d) and rowptr.shape[0] == N + 1
    assert colind.size == 0 or int(colind.max()) < N
    dQ, dK, dV = (np.zeros((N, H, d), dtype=np.float64) for _ in range(3))
    rc = lib.oracle_csr_attention_backward(ctypes.c_int64(N), _p(rowptr), _p(colind), _p(Q), _p(K), _p(V), _p(dO),
                                           ctypes.c_int32(H), ctypes.c_int32(d), ctypes.c_double(scale), ctypes.c_int(dt),
                                           _p(dQ), _p(dK), _p(dV))
    assert rc == 0
    return dQ, dK, dV
