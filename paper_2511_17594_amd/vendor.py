"""The vendor's sparse library (hipSPARSE generic API) on the same device buffers, for the reported baseline.

Reached through ctypes from the shared library that ships with ROCm; nothing of the product path goes
through this module.  Dense operands are row-major fp32 as everywhere else, CSR indices int32, and the
scalars are alpha = 1, beta = 0 so that the results are the same quantities the library computes:

    SpMM   C[n_rows, F] = A * B            (hipsparseSpMM, every CSR algorithm the library offers)
    SDDMM  out[p] = <X[i, :], Y[j, :]>     (hipsparseSDDMM on the pattern of A: the values of the CSR
                                            descriptor are the output, Y enters transposed)

`spmm_times` / `sddmm_time` return milliseconds per call (median of HIP-event timings, preprocessing
outside the timed region) and leave the result in the caller's output tensor so that it can be compared.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

HIPSPARSE_INDEX_32I = 2
HIPSPARSE_INDEX_BASE_ZERO = 0
HIPSPARSE_ORDER_ROW = 2
HIPSPARSE_OPERATION_NON_TRANSPOSE = 0
HIPSPARSE_OPERATION_TRANSPOSE = 1
HIP_R_32F = 0
SPMM_ALGS = {"default": 0, "csr_alg1": 4, "csr_alg2": 6, "csr_alg3": 12}
SDDMM_ALG_DEFAULT = 0


class VendorError(RuntimeError):
    pass


def _load():
    for cand in (os.environ.get("HIPSPARSE_LIB"), "/opt/rocm/lib/libhipsparse.so", "libhipsparse.so", "libhipsparse.so.1"):
        if not cand:
            continue
        try:
            return ctypes.CDLL(cand)
        except OSError:
            continue
    raise VendorError("libhipsparse.so not found")


def _chk(status, what):
    if status != 0:
        raise VendorError("%s failed with hipsparseStatus_t %d" % (what, status))


def _p(t):
    return ctypes.c_void_p(t.data_ptr())


class Session:
    """One hipSPARSE handle bound to torch's current stream."""

    def __init__(self, torch):
        self.torch = torch
        self.lib = _load()
        self.handle = ctypes.c_void_p()
        _chk(self.lib.hipsparseCreate(ctypes.byref(self.handle)), "hipsparseCreate")
        self.stream = torch.cuda.current_stream()
        _chk(self.lib.hipsparseSetStream(self.handle, ctypes.c_void_p(self.stream.cuda_stream)), "hipsparseSetStream")
        self.one = ctypes.c_float(1.0)
        self.zero = ctypes.c_float(0.0)

    def close(self):
        if self.handle:
            self.lib.hipsparseDestroy(self.handle)
            self.handle = ctypes.c_void_p()

    def _csr(self, n_rows, n_cols, nnz, rowptr, colind, val):
        d = ctypes.c_void_p()
        _chk(self.lib.hipsparseCreateCsr(ctypes.byref(d), ctypes.c_int64(n_rows), ctypes.c_int64(n_cols), ctypes.c_int64(nnz),
                                         _p(rowptr), _p(colind), _p(val), HIPSPARSE_INDEX_32I, HIPSPARSE_INDEX_32I,
                                         HIPSPARSE_INDEX_BASE_ZERO, HIP_R_32F), "hipsparseCreateCsr")
        return d

    def _dense(self, t):
        rows, cols = t.shape
        d = ctypes.c_void_p()
        _chk(self.lib.hipsparseCreateDnMat(ctypes.byref(d), ctypes.c_int64(rows), ctypes.c_int64(cols), ctypes.c_int64(t.stride(0)),
                                           _p(t), HIP_R_32F, HIPSPARSE_ORDER_ROW), "hipsparseCreateDnMat")
        return d

    def _timed(self, fn, iters):
        torch = self.torch
        fn()
        torch.cuda.synchronize()
        ts = []
        for _ in range(iters):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(self.stream)
            fn()
            e1.record(self.stream)
            e1.synchronize()
            ts.append(e0.elapsed_time(e1))
        return float(np.median(ts))

    def spmm_times(self, n_rows, n_cols, rowptr, colind, val, B, C, iters=5, algs=None):
        """{algorithm name: ms per call} for C = A * B; algorithms the library refuses are left out.
        C holds the result of the last algorithm that ran."""
        torch, lib = self.torch, self.lib
        nnz = int(colind.numel())
        a, b, c = self._csr(n_rows, n_cols, nnz, rowptr, colind, val), self._dense(B), self._dense(C)
        out = {}
        try:
            for name, alg in (algs or SPMM_ALGS).items():
                args = (self.handle, HIPSPARSE_OPERATION_NON_TRANSPOSE, HIPSPARSE_OPERATION_NON_TRANSPOSE, ctypes.byref(self.one),
                        a, b, ctypes.byref(self.zero), c, HIP_R_32F, alg)
                size = ctypes.c_size_t(0)
                if lib.hipsparseSpMM_bufferSize(*args, ctypes.byref(size)) != 0:
                    continue
                buf = torch.empty(max(int(size.value), 16), dtype=torch.uint8, device=B.device)
                if lib.hipsparseSpMM_preprocess(*args, _p(buf)) != 0:
                    continue
                if lib.hipsparseSpMM(*args, _p(buf)) != 0:
                    continue
                out[name] = self._timed(lambda: lib.hipsparseSpMM(*args, _p(buf)), iters)
                del buf
        finally:
            lib.hipsparseDestroySpMat(a)
            lib.hipsparseDestroyDnMat(b)
            lib.hipsparseDestroyDnMat(c)
        return out

    def sddmm_time(self, n_rows, n_cols, rowptr, colind, X, Y, out, iters=5):
        """ms per call for out[p] = <X[i, :], Y[colind[p], :]> (None when the library refuses the shapes).
        `out` must hold finite values on entry: the library forms beta * out with beta = 0."""
        torch, lib = self.torch, self.lib
        nnz = int(colind.numel())
        c, x, y = self._csr(n_rows, n_cols, nnz, rowptr, colind, out), self._dense(X), self._dense(Y)
        try:
            args = (self.handle, HIPSPARSE_OPERATION_NON_TRANSPOSE, HIPSPARSE_OPERATION_TRANSPOSE, ctypes.byref(self.one),
                    x, y, ctypes.byref(self.zero), c, HIP_R_32F, SDDMM_ALG_DEFAULT)
            size = ctypes.c_size_t(0)
            if lib.hipsparseSDDMM_bufferSize(*args, ctypes.byref(size)) != 0:
                return None
            buf = torch.empty(max(int(size.value), 16), dtype=torch.uint8, device=X.device)
            if lib.hipsparseSDDMM_preprocess(*args, _p(buf)) != 0:
                return None
            if lib.hipsparseSDDMM(*args, _p(buf)) != 0:
                return None
            return self._timed(lambda: lib.hipsparseSDDMM(*args, _p(buf)), iters)
        finally:
            lib.hipsparseDestroySpMat(c)
            lib.hipsparseDestroyDnMat(x)
            lib.hipsparseDestroyDnMat(y)
