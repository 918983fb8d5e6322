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


# The per-row L1-scaled error is ||got_i - ref_i||_1 / ||ref_i||_1.  An fp32 evaluation carries an error of a
# few 2^-24 of the *magnitude of the terms* M_i (the same oracle run on absolute values), whatever the result
# is, so a row whose result cancelled cannot be held to 1e-5 of that result.  The denominator therefore has a
# floor, at one of two levels:
#   - FLOOR_FEW * M_i for a row that can cancel by chance or by structure: its norm is taken over fewer than
#     FEW_OUTPUTS outputs (a degree-1 SDDMM row is one dot product, an F = 1 SpMM row one sum), or every output is
#     a sum of fewer than FEW_TERMS products (two entries of one column with opposite values cancel in every
#     feature at once), or the caller does not say how many terms an output has.  The bound on such a row never
#     drops below 1e-5 * 1e-2 * M_i = 1.7 * 2^-24 * M_i, less than two roundings of the terms;
#   - FLOOR_MANY * M_i for every other row.  Long sums of random signs cancel only statistically (a hub row of
#     65536 terms still has ||ref|| = 4.5e-3 * M), so this level is inactive on every row of the five
#     configurations: rows of 64 entries or more -- hub rows included -- are held to the plain 1e-5.
FEW_OUTPUTS = 8
FEW_TERMS = 64
FLOOR_FEW = 1e-2
FLOOR_MANY = 1e-3


# The row-softmax backward is a structural difference, dS = P * (dP - sum_q P_q dP_q): a row dominated by one
# entry cancels to rounding level by construction, whatever its length.  Its comparisons therefore scale every row
# by at least BACKWARD_FLOOR of the magnitude of its terms (bound 1e-6 * M, about 17 units of 2^-24).
BACKWARD_FLOOR = 0.1


def _floors(outputs, terms, floors):
    few, many = (FLOOR_FEW, FLOOR_MANY) if floors is None else floors
    is_few = np.asarray(outputs) < FEW_OUTPUTS
    is_few = is_few | (True if terms is None else (np.asarray(terms) < FEW_TERMS))
    return np.where(is_few, few, many)


def _finish(num, den, mag, outputs, terms, eps, stats, floors=None):
    if mag is None:
        floored = np.zeros(num.shape, dtype=bool)
        den_f = den
    else:
        floor = _floors(outputs, terms, floors) * mag
        floored = floor > den
        den_f = np.maximum(den, floor)
    err = num / np.maximum(den_f, eps)
    if stats is not None:
        plain = num / np.maximum(den, eps)
        keep = ~floored
        stats["rows"] = int(num.size)
        stats["floored_rows"] = int(floored.sum())
        stats["max_plain_unfloored"] = float(plain[keep].max()) if keep.any() else 0.0
        stats["max_floored"] = float(err[floored].max()) if floored.any() else 0.0
        stats["max"] = float(err.max()) if err.size else 0.0
    return err


def rel_l1_rows(got, ref, ref_abs=None, terms=None, eps=1e-30, stats=None, floors=None):
    """Per-row L1-scaled error ||got_i - ref_i||_1 / max(||ref_i||_1, floor_i * ||abs_i||_1, eps); shape [rows].

    ref_abs is the same oracle result computed on the absolute values of the inputs (the magnitude of the
    terms of every output); floor_i is described above.  Without ref_abs the plain row scaling is used.
    terms = products summed into one output of row i (SpMM: the row's degree; an array or a scalar); None = unknown.
    stats (a dict) receives the number of floored rows and the maxima over floored and unfloored rows.
    floors = (few, many) overrides the two floor levels (the row-softmax backward passes BACKWARD_FLOOR twice)."""
    got = np.asarray(got, dtype=np.float64).reshape(ref.shape[0], -1)
    ref2 = np.asarray(ref, dtype=np.float64).reshape(ref.shape[0], -1)
    num = np.abs(got - ref2).sum(axis=1)
    den = np.abs(ref2).sum(axis=1)
    mag = None
    if ref_abs is not None:
        mag = np.abs(np.asarray(ref_abs, dtype=np.float64).reshape(ref.shape[0], -1)).sum(axis=1)
    return _finish(num, den, mag, np.full(num.shape, ref2.shape[1]), terms, eps, stats, floors)


def _segment_sums(x, rowptr):
    rp = np.asarray(rowptr, dtype=np.int64)
    out = np.zeros(rp.shape[0] - 1, dtype=np.float64)
    nz = rp[1:] > rp[:-1]
    if x.shape[0]:
        out[nz] = np.add.reduceat(x, rp[:-1][nz])
    return out


def rel_l1_segments(got, ref, rowptr, ref_abs=None, terms=None, eps=1e-30, stats=None, floors=None):
    """Same metric where "row i" is the slice rowptr[i]:rowptr[i+1] of a per-nonzero array
    (trailing dimensions, e.g. heads, are folded into the slice); terms = products per output (SDDMM: F)."""
    got = np.asarray(got, dtype=np.float64).reshape(ref.shape[0], -1)
    ref2 = np.asarray(ref, dtype=np.float64).reshape(ref.shape[0], -1)
    n = _segment_sums(np.abs(got - ref2).sum(axis=1), rowptr)
    d = _segment_sums(np.abs(ref2).sum(axis=1), rowptr)
    mag = None
    if ref_abs is not None:
        mag = _segment_sums(np.abs(np.asarray(ref_abs, dtype=np.float64).reshape(ref.shape[0], -1)).sum(axis=1), rowptr)
    rp = np.asarray(rowptr, dtype=np.int64)
    return _finish(n, d, mag, (rp[1:] - rp[:-1]) * ref2.shape[1], terms, eps, stats, floors)


def stats_line(tag, stats):
    """One printable line of what a parity comparison measured (shown with pytest -s / in the run's log)."""
    return ("%s: %d rows, plain per-row error max %.2e on the %d rows above their floor, %d floored rows (max %.2e)"
            % (tag, stats["rows"], stats["max_plain_unfloored"], stats["rows"] - stats["floored_rows"],
               stats["floored_rows"], stats["max_floored"]))
