"""Helpers shared by the GPU parity tests (no arithmetic of the method lives here)."""
import numpy as np


def dev(a, torch, dtype=None):
    """Host NumPy array -> torch tensor on cuda:0 (bf16 bit patterns travel as int16)."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).cuda()
    t = torch.from_numpy(a)
    return t.cuda() if dtype is None else t.to(dtype).cuda()


def dtype_code(ab, a):
    """Library dtype of a host dense operand: uint16 = bf16 bit patterns, float16 = IEEE fp16, else fp32."""
    return ab.BF16 if a.dtype == np.uint16 else ab.F16 if a.dtype == np.float16 else ab.F32


CANCEL_FLOOR = 0.1   # a row whose result cancels below 10 % of the magnitude of its terms is scaled by that floor


def rel_l1_rows(got, ref, ref_abs=None, eps=1e-30):
    """Per-row L1-scaled error: ||got_i - ref_i||_1 / max(||ref_i||_1, 0.1 * ||abs_i||_1, eps); shape [rows].

    ref_abs is the same oracle result computed on the absolute values of the inputs (the sum of the
    magnitudes of the terms of every output).  fp32 summation cannot do better than a few units of
    2^-24 relative to that magnitude, so rows that cancel almost completely are scaled by a tenth of
    it instead of by their (tiny) result.  Without ref_abs the plain row scaling is used."""
    got = np.asarray(got, dtype=np.float64).reshape(ref.shape[0], -1)
    ref2 = np.asarray(ref, dtype=np.float64).reshape(ref.shape[0], -1)
    num = np.abs(got - ref2).sum(axis=1)
    den = np.abs(ref2).sum(axis=1)
    if ref_abs is not None:
        den = np.maximum(den, CANCEL_FLOOR * np.abs(np.asarray(ref_abs, dtype=np.float64).reshape(ref.shape[0], -1)).sum(axis=1))
    return num / np.maximum(den, eps)


def _segment_sums(x, rowptr):
    rp = np.asarray(rowptr, dtype=np.int64)
    out = np.zeros(rp.shape[0] - 1, dtype=np.float64)
    nz = rp[1:] > rp[:-1]
    if x.shape[0]:
        out[nz] = np.add.reduceat(x, rp[:-1][nz])
    return out


def rel_l1_segments(got, ref, rowptr, ref_abs=None, eps=1e-30):
    """Same metric where "row i" is the slice rowptr[i]:rowptr[i+1] of a per-nonzero array
    (trailing dimensions, e.g. heads, are folded into the slice)."""
    got = np.asarray(got, dtype=np.float64).reshape(ref.shape[0], -1)
    ref2 = np.asarray(ref, dtype=np.float64).reshape(ref.shape[0], -1)
    n = _segment_sums(np.abs(got - ref2).sum(axis=1), rowptr)
    d = _segment_sums(np.abs(ref2).sum(axis=1), rowptr)
    if ref_abs is not None:
        ra = np.abs(np.asarray(ref_abs, dtype=np.float64).reshape(ref.shape[0], -1)).sum(axis=1)
        d = np.maximum(d, CANCEL_FLOOR * _segment_sums(ra, rowptr))
    return n / np.maximum(d, eps)
