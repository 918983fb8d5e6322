"""Helpers shared by the GPU parity tests (no arithmetic of the method lives here)."""
import numpy as np


def dev(a, torch, dtype=None):
    """Host NumPy array -> torch tensor on cuda:0 (bf16 bit patterns travel as int16)."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).cuda()
    t = torch.from_numpy(a)
    return t.cuda() if dtype is None else t.to(dtype).cuda()


def rel_l1_rows(got, ref, eps=1e-30):
    """Per-row L1-scaled error: ||got_i - ref_i||_1 / max(||ref_i||_1, eps); shape [rows]."""
    got = np.asarray(got, dtype=np.float64).reshape(ref.shape[0], -1)
    ref2 = np.asarray(ref, dtype=np.float64).reshape(ref.shape[0], -1)
    num = np.abs(got - ref2).sum(axis=1)
    den = np.abs(ref2).sum(axis=1)
    return num / np.maximum(den, eps)


def rel_l1_segments(got, ref, rowptr, eps=1e-30):
    """Same metric where "row i" is the slice rowptr[i]:rowptr[i+1] of a per-nonzero array
    (trailing dimensions, e.g. heads, are folded into the slice)."""
    got = np.asarray(got, dtype=np.float64).reshape(ref.shape[0], -1)
    ref2 = np.asarray(ref, dtype=np.float64).reshape(ref.shape[0], -1)
    rp = np.asarray(rowptr, dtype=np.int64)
    num = np.concatenate([[0.0], np.cumsum(np.abs(got - ref2).sum(axis=1))])
    den = np.concatenate([[0.0], np.cumsum(np.abs(ref2).sum(axis=1))])
    n = num[rp[1:]] - num[rp[:-1]]
    d = den[rp[1:]] - den[rp[:-1]]
    return n / np.maximum(d, eps)
