"""Seeded synthetic inputs shaped like the paper's workloads.

This module only draws random numbers and arranges them into CSR arrays and
dense operands.  It holds none of the method's arithmetic (no SpMM, SDDMM,
softmax, hub partition or selector logic), so both the HIP path and the CPU
checker may be fed from it without sharing any computation.

Every generator is a pure function of its arguments (NumPy PCG64 seeded with
``[seed, config_id]``), runs on the host, and returns int32 CSR arrays whose
rows are sorted and duplicate free.

Workload families (the paper's Experimental Setup and Synthetic stressors
sections name them; the real datasets are not available, so configs 3 and 4 are
stand-ins that only take the published shape: rows, nonzeros, degree character):

  1  tiny Erdos-Renyi graph                      (family of the ER stressor)
  2  power-law out-degree skew stressor with hub rows
  3  dense-community graph, symmetric, val = 1/deg(i)   (Reddit-shaped)
  4  large sparse power-law graph, symmetric + self loops (Products-shaped)
  5  multi-head attention operands on the pattern of config 2
"""
from __future__ import annotations

import dataclasses
from typing import Optional

import numpy as np

__all__ = [
    "CSR", "rng_for", "float_to_bf16_bits", "bf16_bits_to_float",
    "distinct_columns", "csr_from_degrees", "powerlaw_degrees",
    "config1_tiny", "config2_powerlaw", "config3_community", "config4_large",
    "config5_attention", "hub_split_graph", "er_graph", "dense_operand",
    "row_slice",
]


@dataclasses.dataclass
class CSR:
    """A host-side CSR triple (rowptr, colind, val) for an n_rows x n_cols matrix."""
    n_rows: int
    n_cols: int
    rowptr: np.ndarray   # int32 [n_rows + 1]
    colind: np.ndarray   # int32 [nnz]
    val: np.ndarray      # float32 [nnz]

    @property
    def nnz(self) -> int:
        return int(self.rowptr[-1])

    @property
    def degrees(self) -> np.ndarray:
        return np.diff(self.rowptr.astype(np.int64))


def rng_for(seed: int, config_id: int, stream: int = 0) -> np.random.Generator:
    return np.random.default_rng([int(seed), int(config_id), int(stream)])


# --------------------------------------------------------------------------- #
# bf16 storage helpers (bit patterns only; round-to-nearest-even)
# --------------------------------------------------------------------------- #
def float_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 array -> uint16 array holding the bf16 bit patterns (RNE, NaN kept)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    rounded = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
    out = rounded.astype(np.uint16)
    nan = np.isnan(x)
    if nan.any():
        out[nan] = 0x7FC0
    return out


def bf16_bits_to_float(b: np.ndarray) -> np.ndarray:
    """uint16 bf16 bit patterns -> the fp32 values they denote (exact)."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << 16).view(np.float32)


# --------------------------------------------------------------------------- #
# pattern builders
# --------------------------------------------------------------------------- #
def distinct_columns(rng: np.random.Generator, deg: np.ndarray, n_cols: int,
                     big_row: int = 2048):
    """For every row i draw deg[i] distinct column ids uniformly from [0, n_cols).

    Returns (rowptr int32, colind int32) with sorted rows.  Rows with at least
    ``big_row`` entries are drawn one by one without replacement; the rest are
    drawn in bulk with replacement, deduplicated, and topped up until every row
    has exactly its requested degree.
    """
    deg = np.asarray(deg, dtype=np.int64)
    if (deg > n_cols).any():
        raise ValueError("degree exceeds number of columns")
    n_rows = deg.shape[0]
    rowptr64 = np.zeros(n_rows + 1, dtype=np.int64)
    np.cumsum(deg, out=rowptr64[1:])
    nnz = int(rowptr64[-1])
    if nnz >= 2**31:
        raise ValueError("nnz does not fit int32")
    # rows that fill a good part of the column range are also drawn without replacement (the top-up
    # of a nearly full row converges slowly)
    big = np.flatnonzero(deg >= min(big_row, max(1, n_cols // 4)))
    small_deg = deg.copy()
    small_deg[big] = 0

    # bulk part: keys = row * n_cols + col, kept distinct
    keys = np.empty(0, dtype=np.int64)
    need = small_deg.copy()
    rows_all = np.arange(n_rows, dtype=np.int64)
    for _ in range(64):
        tot = int(need.sum())
        if tot == 0:
            break
        r = np.repeat(rows_all, need)
        c = rng.integers(0, n_cols, size=tot, dtype=np.int64)
        keys = np.concatenate([keys, r * n_cols + c])
        keys.sort(kind="stable")
        if keys.size:
            keep = np.empty(keys.size, dtype=bool)
            keep[0] = True
            np.not_equal(keys[1:], keys[:-1], out=keep[1:])
            keys = keys[keep]
        have = np.bincount(keys // n_cols, minlength=n_rows).astype(np.int64)
        need = small_deg - have
    else:  # pragma: no cover
        raise RuntimeError("top-up did not converge")

    colind = np.empty(nnz, dtype=np.int32)
    small_rows = keys // n_cols
    small_cols = (keys - small_rows * n_cols).astype(np.int32)
    # scatter the bulk part to its CSR positions (keys are sorted by row, col)
    small_ptr = np.zeros(n_rows + 1, dtype=np.int64)
    np.cumsum(small_deg, out=small_ptr[1:])
    pos_in_row = np.arange(keys.size, dtype=np.int64) - small_ptr[small_rows]
    colind[rowptr64[small_rows] + pos_in_row] = small_cols
    for i in big:
        d = int(deg[i])
        cols = rng.choice(n_cols, size=d, replace=False)
        cols.sort()
        colind[rowptr64[i]:rowptr64[i] + d] = cols.astype(np.int32)
    return rowptr64.astype(np.int32), colind


def csr_from_degrees(rng, deg, n_cols, val_low=-1.0, val_high=1.0) -> CSR:
    rowptr, colind = distinct_columns(rng, deg, n_cols)
    val = rng.uniform(val_low, val_high, size=colind.shape[0]).astype(np.float32)
    return CSR(len(deg), n_cols, rowptr, colind, val)


def powerlaw_degrees(rng, n: int, gamma: float, mean: float, dmax: Optional[int],
                     dmin: int = 1) -> np.ndarray:
    """d_i = clip(round(x_m * u_i^(-1/(gamma-1))), dmin, dmax); x_m bisected for the mean."""
    u = rng.random(n)
    u = np.maximum(u, 1e-300)
    base = u ** (-1.0 / (gamma - 1.0))

    def degs(xm):
        d = np.rint(xm * base)
        hi = float(dmax) if dmax is not None else float(n)
        return np.clip(d, dmin, hi).astype(np.int64)

    lo, hi = 1e-3, float(mean) * 4
    for _ in range(80):
        mid = 0.5 * (lo + hi)
        if degs(mid).mean() < mean:
            lo = mid
        else:
            hi = mid
    return degs(hi)


def _symmetrise(src: np.ndarray, dst: np.ndarray, n: int, self_loops: bool):
    """Union of (src,dst) and (dst,src) (+ diagonal), deduplicated, as int32 CSR pattern."""
    parts = [src * n + dst, dst * n + src]
    if self_loops:
        diag = np.arange(n, dtype=np.int64)
        parts.append(diag * n + diag)
    keys = np.concatenate(parts)
    del parts
    keys.sort()
    keep = np.empty(keys.size, dtype=bool)
    keep[0] = True
    np.not_equal(keys[1:], keys[:-1], out=keep[1:])
    keys = keys[keep]
    del keep
    rows = keys // n
    colind = (keys - rows * n).astype(np.int32)
    del keys
    deg = np.bincount(rows, minlength=n).astype(np.int64)
    del rows
    rowptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(deg, out=rowptr[1:])
    if rowptr[-1] >= 2**31:
        raise ValueError("nnz does not fit int32")
    return rowptr.astype(np.int32), colind


def dense_operand(rng, n: int, F: int, std: float = 1.0) -> np.ndarray:
    out = rng.standard_normal(size=(n, F), dtype=np.float32)
    if std != 1.0:
        out *= np.float32(std)
    return out


# --------------------------------------------------------------------------- #
# the five configurations
# --------------------------------------------------------------------------- #
def er_graph(n: int, p: float, seed: int = 0, config_id: int = 1) -> CSR:
    """Erdos-Renyi: deg_i ~ Binomial(n, p), distinct uniform columns, val ~ U[-1,1)."""
    rng = rng_for(seed, config_id)
    deg = rng.binomial(n, p, size=n).astype(np.int64)
    return csr_from_degrees(rng, deg, n)


def config1_tiny(n: int = 4096, mean_deg: float = 16.0, F: int = 32, seed: int = 0):
    """Config 1: ER graph with about 16 nonzeros per row; B, X, Y ~ N(0,1) of width F."""
    A = er_graph(n, mean_deg / n, seed, 1)
    rng = rng_for(seed, 1, 1)
    B = dense_operand(rng, n, F)
    X = dense_operand(rng, n, F)
    Y = dense_operand(rng, n, F)
    return A, B, X, Y


def config2_powerlaw(n: int = 262144, mean_deg: float = 32.0, gamma: float = 2.1,
                     dmax: int = 65536, seed: int = 0) -> CSR:
    """Config 2: Pareto out-degrees (pdf ~ d^-gamma) with mean 32, clipped at dmax; uniform columns."""
    rng = rng_for(seed, 2)
    deg = powerlaw_degrees(rng, n, gamma, mean_deg, min(dmax, n))
    return csr_from_degrees(rng, deg, n)


def config3_community(n: int = 232965, mean_deg: float = 492.0, sigma: float = 1.0,
                      p_intra: float = 0.7, comm_size: float = 5000.0,
                      oversample: float = 1.125, seed: int = 0) -> CSR:
    """Config 3: lognormal target degrees, planted contiguous communities, symmetric, val=1/deg(i).

    Every node draws about half its target degree as half-edges; each half-edge
    stays inside the node's community with probability p_intra, else goes to a
    uniform node.  The edge set is symmetrised and deduplicated.  ``oversample``
    compensates the duplicates that symmetrising removes so that the final
    number of nonzeros lands near n * mean_deg.
    """
    rng = rng_for(seed, 3)
    mu = np.log(mean_deg) - 0.5 * sigma * sigma
    tgt = np.exp(rng.normal(mu, sigma, size=n))
    tgt = np.clip(tgt, 1.0, n / 4.0)
    half = np.maximum(np.rint(0.5 * oversample * tgt), 1).astype(np.int64)
    # communities: contiguous id blocks with lognormal sizes
    sizes = []
    tot = 0
    while tot < n:
        s = int(max(64, np.rint(np.exp(rng.normal(np.log(comm_size), 0.5)))))
        s = min(s, n - tot)
        sizes.append(s)
        tot += s
    sizes = np.asarray(sizes, dtype=np.int64)
    starts = np.zeros(sizes.size, dtype=np.int64)
    np.cumsum(sizes[:-1], out=starts[1:])
    comm_of = np.repeat(np.arange(sizes.size, dtype=np.int64), sizes)
    # targets are drawn with probability proportional to the target degree
    # (inside the community, or over the whole graph), so that the realised
    # degree of a node follows its lognormal target
    cum = np.zeros(n + 1, dtype=np.float64)
    np.cumsum(tgt, out=cum[1:])
    src = np.repeat(np.arange(n, dtype=np.int64), half)
    m = src.size
    u = rng.random(m)
    intra = rng.random(m) < p_intra
    c = comm_of[src]
    lo = np.where(intra, cum[starts[c]], 0.0)
    hi = np.where(intra, cum[starts[c] + sizes[c]], cum[n])
    del intra, c
    dst = np.searchsorted(cum, lo + u * (hi - lo), side="right").astype(np.int64) - 1
    del u, lo, hi
    np.maximum(dst, 0, out=dst)
    np.minimum(dst, n - 1, out=dst)
    rowptr, colind = _symmetrise(src, dst, n, self_loops=False)
    del src, dst
    deg = np.diff(rowptr.astype(np.int64))
    inv = (1.0 / np.maximum(deg, 1)).astype(np.float32)
    val = np.repeat(inv, deg)
    return CSR(n, n, rowptr, colind, val)


def config4_large(n: int = 2449029, mean_half: float = 25.45, gamma: float = 2.3,
                  seed: int = 0) -> CSR:
    """Config 4: unclipped power-law half-edge degrees, uniform targets, symmetric, self loops, val~U[0,1)."""
    rng = rng_for(seed, 4)
    half = powerlaw_degrees(rng, n, gamma, mean_half, dmax=n // 4)
    src = np.repeat(np.arange(n, dtype=np.int64), half)
    dst = rng.integers(0, n, size=src.size, dtype=np.int64)
    rowptr, colind = _symmetrise(src, dst, n, self_loops=True)
    del src, dst
    val = rng.random(colind.shape[0], dtype=np.float32)
    return CSR(n, n, rowptr, colind, val)


def config5_attention(n: int, H: int = 8, d: int = 64, seed: int = 0,
                      qk_std: Optional[float] = None):
    """Config 5 operands: Q, K, V [n, H, d] drawn N(0, sigma^2) and stored as bf16 bit patterns.

    The config text gives N(0, 1/sqrt(d)); it is read as variance 1/sqrt(d),
    i.e. sigma = d^(-1/4).  ``qk_std`` overrides sigma for Q and K (parity tests
    also use 1.0 so that the softmax is far from flat).
    """
    rng = rng_for(seed, 5)
    sigma = float(d) ** -0.25
    sq = sigma if qk_std is None else float(qk_std)
    Q = float_to_bf16_bits(dense_operand(rng, n, H * d, sq)).reshape(n, H, d)
    K = float_to_bf16_bits(dense_operand(rng, n, H * d, sq)).reshape(n, H, d)
    V = float_to_bf16_bits(dense_operand(rng, n, H * d, sigma)).reshape(n, H, d)
    return Q, K, V


def hub_split_graph(n: int = 20000, n_hub: int = 32, hub_deg: int = 5000,
                    other_deg: int = 64, seed: int = 0) -> CSR:
    """Shape of the paper's CTA-per-hub table: a few rows of degree hub_deg, the rest other_deg.

    The paper does not say how many hub rows it used; n_hub is a parameter here.
    Hub rows are placed at evenly spaced row ids.
    """
    rng = rng_for(seed, 6)
    deg = np.full(n, other_deg, dtype=np.int64)
    if n_hub > 0:
        hubs = (np.arange(n_hub, dtype=np.int64) * n) // n_hub
        deg[hubs] = hub_deg
    return csr_from_degrees(rng, deg, n)


def largest_input(nnz: int, n_rows: int = 1050000, n_cols: int = 1 << 20, hub_row: int = 7,
                  hub_deg: int = 300000, seed: int = 0) -> CSR:
    """A matrix with exactly `nnz` stored entries, for the size limit of the library (about 17 GB of host
    memory at 2^31 - 2^20 entries).  Row i holds 2040 + i % 8 entries, row 5 none, row `hub_row` hub_deg, and
    the last row whatever is left, so the last nonzero of the last (long) row sits at position nnz - 1.
    Columns are uniform and unsorted, duplicates may occur (both are legal inputs); values U[-1, 1).
    """
    rng = rng_for(seed, 8)
    deg = 2040 + (np.arange(n_rows, dtype=np.int64) % 8)
    deg[5] = 0
    deg[hub_row] = hub_deg
    deg[-1] = 0
    rest = int(nnz) - int(deg.sum())
    if rest < 0:
        raise ValueError("nnz too small for %d rows" % n_rows)
    deg[-1] = rest
    rowptr = np.zeros(n_rows + 1, dtype=np.int64)
    np.cumsum(deg, out=rowptr[1:])
    colind = np.empty(nnz, dtype=np.int32)
    val = np.empty(nnz, dtype=np.float32)
    step = 1 << 26
    for lo in range(0, nnz, step):                       # in pieces: bounded temporaries
        hi = min(nnz, lo + step)
        colind[lo:hi] = rng.integers(0, n_cols, size=hi - lo, dtype=np.int32)
        val[lo:hi] = rng.random(hi - lo, dtype=np.float32) * np.float32(2.0) - np.float32(1.0)
    return CSR(n_rows, n_cols, rowptr.astype(np.int32), colind, val)


# --------------------------------------------------------------------------- #
# index-only helper used by tests that check sampled rows of a large result
# --------------------------------------------------------------------------- #
def row_slice(A: CSR, rows: np.ndarray) -> CSR:
    """The rectangular matrix made of the listed rows of A (all their nonzeros, same columns)."""
    rows = np.asarray(rows, dtype=np.int64)
    rp = A.rowptr.astype(np.int64)
    deg = rp[rows + 1] - rp[rows]
    new_ptr = np.zeros(rows.size + 1, dtype=np.int64)
    np.cumsum(deg, out=new_ptr[1:])
    idx = np.repeat(rp[rows] - new_ptr[:-1], deg) + np.arange(int(new_ptr[-1]), dtype=np.int64)
    return CSR(rows.size, A.n_cols, new_ptr.astype(np.int32), A.colind[idx].copy(), A.val[idx].copy())
