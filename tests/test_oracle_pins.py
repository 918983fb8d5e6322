"""Pins for the CPU oracle: every oracle function is checked against something other than
itself -- dense brute force, closed forms, library routines on textbook special cases,
hand-worked fixtures -- chosen so that a dropped term, a wrong index or a transposed
operand fails at least one test.  CPU only.
"""
import os

import numpy as np
import pytest
import scipy.sparse as sp
import scipy.special

import oracle
from paper_2511_17594_amd import workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def tiny_csr(n_rows, n_cols, mean_deg, seed, with_empty=True):
    rng = np.random.default_rng(seed)
    deg = rng.poisson(mean_deg, size=n_rows).clip(0, n_cols)
    if with_empty and n_rows > 2:
        deg[1] = 0
        deg[n_rows - 1] = 0
    A = W.csr_from_degrees(rng, deg, n_cols)
    return A, rng


def densify(A):
    """Dense copy of a CSR matrix built entry by entry (duplicates add)."""
    D = np.zeros((A.n_rows, A.n_cols), dtype=np.float64)
    for i in range(A.n_rows):
        for p in range(A.rowptr[i], A.rowptr[i + 1]):
            D[i, A.colind[p]] += float(A.val[p])
    return D


# ------------------------------------------------------------------ SpMM ---
@pytest.mark.parametrize("n_rows,n_cols,F", [(37, 37, 5), (64, 29, 8), (13, 50, 1)])
def test_spmm_equals_dense_matmul(n_rows, n_cols, F):
    A, rng = tiny_csr(n_rows, n_cols, 4.0, seed=n_rows)
    B = rng.standard_normal((n_cols, F)).astype(np.float32)
    C = oracle.spmm(A.rowptr, A.colind, A.val, B)
    ref = densify(A) @ B.astype(np.float64)
    np.testing.assert_allclose(C, ref, rtol=1e-13, atol=1e-13)
    assert np.all(C[1] == 0.0) and np.all(C[-1] == 0.0)          # empty rows give zeros


def test_spmm_identity_and_permutation_are_exact():
    n, F = 41, 7
    rng = np.random.default_rng(3)
    B = rng.standard_normal((n, F)).astype(np.float32)
    rowptr = np.arange(n + 1, dtype=np.int32)
    ones = np.ones(n, dtype=np.float32)
    C = oracle.spmm(rowptr, np.arange(n, dtype=np.int32), ones, B)
    assert np.array_equal(C, B.astype(np.float64))
    perm = rng.permutation(n).astype(np.int32)
    C = oracle.spmm(rowptr, perm, ones, B)
    assert np.array_equal(C, B[perm].astype(np.float64))


def test_spmm_diagonal_scaling_and_duplicates():
    n, F = 16, 3
    rng = np.random.default_rng(4)
    B = rng.standard_normal((n, F)).astype(np.float32)
    s = rng.uniform(-2, 2, n).astype(np.float32)
    C = oracle.spmm(np.arange(n + 1, dtype=np.int32), np.arange(n, dtype=np.int32), s, B)
    assert np.array_equal(C, s.astype(np.float64)[:, None] * B.astype(np.float64))
    # one row, the same column stored three times: the values add up
    C = oracle.spmm(np.array([0, 3], np.int32), np.array([2, 2, 2], np.int32),
                    np.array([1.0, 2.0, 4.0], np.float32), B)
    assert np.array_equal(C[0], 7.0 * B[2].astype(np.float64))


def test_spmm_row_normalised_times_ones():
    A, B, _, _ = W.config1_tiny(n=512, mean_deg=9.0, F=4)
    deg = A.degrees
    val = np.repeat(1.0 / np.maximum(deg, 1), deg).astype(np.float32)
    C = oracle.spmm(A.rowptr, A.colind, val, np.ones((512, 4), np.float32))
    expect = (deg > 0).astype(np.float64)[:, None] * np.ones((1, 4))
    np.testing.assert_allclose(C, expect, rtol=0, atol=1e-6)


def test_spmm_linearity_and_scipy_crosscheck():
    A, B, X, _ = W.config1_tiny(n=1024, mean_deg=16.0, F=32)
    C1 = oracle.spmm(A.rowptr, A.colind, A.val, B)
    C2 = oracle.spmm(A.rowptr, A.colind, A.val, X)
    # (B + X) is rounded to fp32 before the product, so compare through the fp32 sum itself
    S = (B + X).astype(np.float32)
    C12 = oracle.spmm(A.rowptr, A.colind, A.val, S)
    M = sp.csr_matrix((A.val.astype(np.float64), A.colind, A.rowptr), shape=(1024, 1024))
    np.testing.assert_allclose(C1, M @ B.astype(np.float64), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(C12, M @ S.astype(np.float64), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(C1 + C2, M @ (B.astype(np.float64) + X.astype(np.float64)), rtol=1e-12, atol=1e-12)


def test_spmm_bf16_operand_values():
    bits, vals = [], []
    for line in open(os.path.join(GOLDEN, "bf16_values.txt")):
        if line.startswith("#") or not line.strip():
            continue
        b, v = line.split()
        bits.append(int(b, 16))
        vals.append(float(v))
    n = len(bits)
    Bb = np.array(bits, dtype=np.uint16).reshape(n, 1)
    C = oracle.spmm(np.arange(n + 1, dtype=np.int32), np.arange(n, dtype=np.int32), np.ones(n, np.float32), Bb)
    assert np.array_equal(C[:, 0], np.array(vals))
    # the generators' bf16 helpers agree with the same table
    assert np.array_equal(W.bf16_bits_to_float(np.array(bits, np.uint16)).astype(np.float64), np.array(vals))
    assert np.array_equal(W.float_to_bf16_bits(np.array(vals, np.float32)), np.array(bits, np.uint16))
    # round to nearest even: 1 + 2^-8 is a tie between 0x3f80 and 0x3f81 -> even; just above goes up
    assert W.float_to_bf16_bits(np.array([1.0 + 2.0 ** -8], np.float32))[0] == 0x3F80
    assert W.float_to_bf16_bits(np.array([1.0 + 2.0 ** -8 + 2.0 ** -20], np.float32))[0] == 0x3F81
    assert W.float_to_bf16_bits(np.array([1.0 + 3 * 2.0 ** -8], np.float32))[0] == 0x3F82


def test_spmm_fp16_operand_values():
    """IEEE binary16 operands: the table holds the values the format's definition gives for each pattern."""
    bits, vals = [], []
    for line in open(os.path.join(GOLDEN, "f16_values.txt")):
        if line.startswith("#") or not line.strip():
            continue
        b, v = line.split()
        bits.append(int(b, 16))
        vals.append(float(v))
    n = len(bits)
    for u, v in zip(bits, vals):                       # the definition, written out
        sgn, e, f = (-1.0 if u >> 15 else 1.0), (u >> 10) & 31, u & 1023
        assert v == sgn * (2.0 ** (e - 15) * (1 + f / 1024) if e else 2.0 ** -14 * f / 1024)
    Bh = np.array(bits, dtype=np.uint16).view(np.float16).reshape(n, 1)
    C = oracle.spmm(np.arange(n + 1, dtype=np.int32), np.arange(n, dtype=np.int32), np.ones(n, np.float32), Bh)
    assert np.array_equal(C[:, 0], np.array(vals))
    out = oracle.sddmm(np.arange(n + 1, dtype=np.int32), np.arange(n, dtype=np.int32), Bh, np.ones((n, 1), np.float16))
    assert np.array_equal(out, np.array(vals))


# ----------------------------------------------------------------- SDDMM ---
@pytest.mark.parametrize("n_rows,n_cols,F", [(23, 23, 6), (31, 17, 9)])
def test_sddmm_equals_masked_dense_product(n_rows, n_cols, F):
    A, rng = tiny_csr(n_rows, n_cols, 3.0, seed=7 + n_rows)
    X = rng.standard_normal((n_rows, F)).astype(np.float32)
    Y = rng.standard_normal((n_cols, F)).astype(np.float32)
    out = oracle.sddmm(A.rowptr, A.colind, X, Y)
    full = X.astype(np.float64) @ Y.astype(np.float64).T          # [n_rows, n_cols]
    p = 0
    for i in range(n_rows):
        for q in range(A.rowptr[i], A.rowptr[i + 1]):
            assert abs(out[q] - full[i, A.colind[q]]) <= 1e-13 * (1 + abs(full[i, A.colind[q]]))
            p += 1
    assert p == A.nnz == out.shape[0]


def test_sddmm_special_cases():
    n, F = 19, 8
    rng = np.random.default_rng(11)
    X = rng.standard_normal((n, F)).astype(np.float32)
    eye_ptr, eye_col = np.arange(n + 1, dtype=np.int32), np.arange(n, dtype=np.int32)
    # identity pattern: out[i] = <X_i, Y_i>
    Y = rng.standard_normal((n, F)).astype(np.float32)
    out = oracle.sddmm(eye_ptr, eye_col, X, Y)
    np.testing.assert_allclose(out, np.einsum("if,if->i", X.astype(np.float64), Y.astype(np.float64)), rtol=1e-14)
    # F = 1 is a plain product x_i * y_j
    A, rng2 = tiny_csr(n, n, 3.0, seed=5)
    x = rng2.standard_normal((n, 1)).astype(np.float32)
    y = rng2.standard_normal((n, 1)).astype(np.float32)
    out = oracle.sddmm(A.rowptr, A.colind, x, y)
    rows = np.repeat(np.arange(n), A.degrees)
    assert np.array_equal(out, x[rows, 0].astype(np.float64) * y[A.colind, 0].astype(np.float64))
    # one-hot rows: X_i = e_(i mod F), Y_j = (j+1) * e_(j mod F): nonzero only where i = j (mod F)
    Xo = np.zeros((n, F), np.float32)
    Xo[np.arange(n), np.arange(n) % F] = 1
    Yo = np.zeros((n, F), np.float32)
    Yo[np.arange(n), np.arange(n) % F] = np.arange(1, n + 1)
    out = oracle.sddmm(A.rowptr, A.colind, Xo, Yo)
    expect = np.where(rows % F == A.colind % F, A.colind + 1.0, 0.0)
    assert np.array_equal(out, expect)
    # val plays no role: the function does not even take it


# --------------------------------------------------------------- softmax ---
def test_row_softmax_matches_library_softmax_per_row_and_head():
    A, rng = tiny_csr(40, 40, 5.0, seed=21)
    for H in (1, 3, 8):
        s = (4.0 * rng.standard_normal((A.nnz, H))).astype(np.float32)
        out = oracle.row_softmax(A.rowptr, s)
        for i in range(A.n_rows):
            p0, p1 = A.rowptr[i], A.rowptr[i + 1]
            if p1 > p0:
                ref = scipy.special.softmax(s[p0:p1].astype(np.float64), axis=0)
                np.testing.assert_allclose(out[p0:p1], ref, rtol=1e-13, atol=1e-300)
                np.testing.assert_allclose(out[p0:p1].sum(axis=0), 1.0, rtol=1e-13)


def test_row_softmax_closed_forms_and_stability():
    rowptr = np.array([0, 1, 1, 5, 9], np.int32)        # degrees 1, 0, 4, 4
    s = np.array([3.0, 2.0, 2.0, 2.0, 2.0, 1e4, -1e4, 1e4, 0.0], np.float32)
    out = oracle.row_softmax(rowptr, s)
    assert out[0] == 1.0                                 # single entry
    assert np.array_equal(out[1:5], np.full(4, 0.25))    # constant scores -> 1/deg
    assert np.all(np.isfinite(out))
    np.testing.assert_allclose(out[5:9], [0.5, 0.0, 0.5, 0.0], atol=1e-300)
    # shift invariance (shift chosen so that the fp32 sums are exact)
    s2 = np.array([0.5, 1.5, -2.0, 0.25, 1.0, 2.0, 3.0, 4.0, 5.0], np.float32)
    a = oracle.row_softmax(rowptr, s2)
    b = oracle.row_softmax(rowptr, s2 + np.float32(8.0))
    np.testing.assert_allclose(a, b, rtol=1e-14)
    # two-entry row: logistic closed form
    r = oracle.row_softmax(np.array([0, 2], np.int32), np.array([0.3, -1.1], np.float64))
    np.testing.assert_allclose(r[0], 1.0 / (1.0 + np.exp(-1.4)), rtol=1e-14)


# ------------------------------------------------------------- attention ---
def dense_attention(Q, K, V, scale):
    """Textbook softmax attention, per head, float64."""
    Q, K, V = (np.asarray(t, np.float64) for t in (Q, K, V))
    S = scale * np.einsum("ihk,jhk->hij", Q, K)
    P = scipy.special.softmax(S, axis=2)
    return np.einsum("hij,jhk->ihk", P, V)


def test_attention_full_pattern_is_dense_attention():
    n, H, d = 12, 3, 5
    rng = np.random.default_rng(31)
    Q, K, V = (rng.standard_normal((n, H, d)).astype(np.float32) for _ in range(3))
    rowptr = (np.arange(n + 1) * n).astype(np.int32)
    colind = np.tile(np.arange(n, dtype=np.int32), n)
    O = oracle.csr_attention(rowptr, colind, Q, K, V, scale=0.37)
    np.testing.assert_allclose(O, dense_attention(Q, K, V, 0.37), rtol=1e-12, atol=1e-13)
    # same through torch's CPU routine in float64
    torch = pytest.importorskip("torch")
    q, k, v = (torch.from_numpy(t.astype(np.float64)).permute(1, 0, 2) for t in (Q, K, V))
    ref = torch.nn.functional.scaled_dot_product_attention(q, k, v, scale=0.37).permute(1, 0, 2).numpy()
    np.testing.assert_allclose(O, ref, rtol=1e-10, atol=1e-12)


def test_attention_masked_pattern_equals_masked_dense_attention():
    n, H, d = 17, 2, 4
    A, rng = tiny_csr(n, n, 4.0, seed=33)
    Q, K, V = (rng.standard_normal((n, H, d)).astype(np.float32) for _ in range(3))
    O, S, P = oracle.csr_attention(A.rowptr, A.colind, Q, K, V, scale=0.5, return_scores=True)
    mask = np.zeros((n, n), bool)
    rows = np.repeat(np.arange(n), A.degrees)
    mask[rows, A.colind] = True
    Sd = 0.5 * np.einsum("ihk,jhk->hij", Q.astype(np.float64), K.astype(np.float64))
    Sd = np.where(mask[None], Sd, -np.inf)
    for i in range(n):
        if not mask[i].any():
            assert np.all(O[i] == 0.0)                   # empty row -> zeros
            continue
        Pd = scipy.special.softmax(Sd[:, i, :], axis=1)  # [H, n]
        ref = np.einsum("hj,jhk->hk", Pd, V.astype(np.float64))
        np.testing.assert_allclose(O[i], ref, rtol=1e-12, atol=1e-13)
    # stored scores are the scaled dot products in CSR order, probabilities sum to one per row/head
    np.testing.assert_allclose(S, Sd[:, rows, A.colind].T, rtol=1e-13, atol=1e-14)
    sums = np.add.reduceat(P, A.rowptr[:-1][A.degrees > 0], axis=0)
    np.testing.assert_allclose(sums, 1.0, rtol=1e-13)


def test_attention_identity_pattern_and_constant_values():
    n, H, d = 9, 2, 8
    Q, K, V = W.config5_attention(n, H, d, seed=1)
    eye_ptr, eye_col = np.arange(n + 1, dtype=np.int32), np.arange(n, dtype=np.int32)
    O = oracle.csr_attention(eye_ptr, eye_col, Q, K, V, scale=d ** -0.5)
    assert np.array_equal(O, W.bf16_bits_to_float(V).astype(np.float64))   # softmax of one score is 1
    A, _ = tiny_csr(n, n, 3.0, seed=2, with_empty=False)
    deg = np.maximum(A.degrees, 1)
    A2 = W.csr_from_degrees(np.random.default_rng(0), deg, n)
    Vc = np.zeros((n, H, d), np.float32)
    Vc[:, 0, :] = 1.5
    Vc[:, 1, :] = -0.25
    O = oracle.csr_attention(A2.rowptr, A2.colind, Q, K, W.float_to_bf16_bits(Vc).reshape(n, H, d), scale=1.0)
    np.testing.assert_allclose(O[:, 0, :], 1.5, rtol=1e-14)               # convex combination of a constant
    np.testing.assert_allclose(O[:, 1, :], -0.25, rtol=1e-14)


# --------------------------------------------------------- index metadata ---
def read_golden_partition():
    d = {}
    for line in open(os.path.join(GOLDEN, "hub_partition_small.txt")):
        if line.startswith("#") or not line.strip():
            continue
        k, *v = line.split()
        d[k] = np.array([int(x) for x in v], dtype=np.int64)
    return d


def test_hub_partition_hand_worked_case():
    g = read_golden_partition()
    rowptr = np.concatenate([[0], np.cumsum(g["degrees"])]).astype(np.int32)
    hub_rows, chunk_ptr, light_rows = oracle.hub_partition(rowptr, int(g["hub_t"][0]), int(g["hub_chunk"][0]))
    assert np.array_equal(hub_rows, g["hub_rows"])
    assert np.array_equal(chunk_ptr, g["chunk_ptr"])
    assert np.array_equal(light_rows, g["light_rows"])
    hist, mx = oracle.degree_histogram(rowptr)
    assert np.array_equal(hist[:4], g["hist"]) and hist[4:].sum() == 0 and mx == int(g["max_deg"][0])


@pytest.mark.parametrize("hub_t,chunk", [(8, 8), (16, 5), (1, 3), (1000, 7)])
def test_hub_partition_invariants(hub_t, chunk):
    rng = np.random.default_rng(hub_t)
    deg = W.powerlaw_degrees(rng, 3000, 2.1, 12.0, 600)
    deg[::17] = 0
    rowptr = np.concatenate([[0], np.cumsum(deg)]).astype(np.int32)
    hub_rows, chunk_ptr, light_rows = oracle.hub_partition(rowptr, hub_t, chunk)
    # brute force in Python integers
    hubs = [i for i in range(3000) if deg[i] >= hub_t]
    assert hub_rows.tolist() == hubs
    assert light_rows.tolist() == [i for i in range(3000) if deg[i] < hub_t]
    assert chunk_ptr[0] == 0 and np.all(np.diff(chunk_ptr) == [-(-int(deg[i]) // chunk) for i in hubs])
    # chunks tile every hub row exactly
    total = 0
    for k, r in enumerate(hubs):
        for t in range(chunk_ptr[k + 1] - chunk_ptr[k]):
            lo = rowptr[r] + t * chunk
            hi = min(rowptr[r] + (t + 1) * chunk, rowptr[r + 1])
            assert lo < hi
            total += hi - lo
    assert total == int(deg[hubs].sum()) if hubs else total == 0


def test_degree_histogram_brute_force():
    rng = np.random.default_rng(5)
    deg = np.concatenate([rng.integers(0, 70000, 500), [0, 1, 2, 3, 4, 65535, 65536, 65537]])
    rowptr = np.concatenate([[0], np.cumsum(deg)]).astype(np.int32)
    hist, mx = oracle.degree_histogram(rowptr)
    ref = np.zeros(33, np.int64)
    for x in deg.tolist():
        ref[int(x).bit_length()] += 1
    assert np.array_equal(hist, ref) and mx == deg.max()


def fnv1a64(data: bytes) -> int:
    h = 0xCBF29CE484222325
    for b in data:
        h = ((h ^ b) * 0x100000001B3) & 0xFFFFFFFFFFFFFFFF
    return h


def test_graph_signature_is_fnv1a_of_the_stated_stream():
    # the helper above is first pinned to the published vectors ...
    for line in open(os.path.join(GOLDEN, "fnv1a64_vectors.txt")):
        if line.startswith("#") or not line.strip():
            continue
        text, hx = line.rsplit(" ", 1)
        assert fnv1a64(text.strip('"').encode()) == int(hx, 16)
    # ... then applied to the byte stream the signature is defined over
    A = W.config2_powerlaw(n=5000, mean_deg=8.0, dmax=512, seed=3)
    hist, mx = oracle.degree_histogram(A.rowptr)
    seq = [A.n_rows, A.n_cols, A.nnz, mx] + hist.tolist() + [int(A.rowptr[(k * A.n_rows) // 1023]) for k in range(1024)]
    data = b"".join(int(v).to_bytes(8, "little", signed=True) for v in seq)
    assert oracle.graph_signature(A.rowptr, A.n_cols) == fnv1a64(data)
    # a different graph gets a different signature
    B = W.config2_powerlaw(n=5000, mean_deg=8.0, dmax=512, seed=4)
    assert oracle.graph_signature(B.rowptr, B.n_cols) != oracle.graph_signature(A.rowptr, A.n_cols)


# --------------------------------------------------------------- selector ---
def test_decide_guardrail_and_ties():
    assert oracle.decide([2.0, 1.0, 1.0, 3.0], 2.0, 0.95) == 1      # first strictly smallest wins ties
    assert oracle.decide([0.95], 1.0, 0.95) == 0                    # boundary t* == alpha * tb is accepted
    assert oracle.decide([0.951], 1.0, 0.95) == -1
    assert oracle.decide([], 1.0, 0.95) == -1                       # nothing to try -> baseline
    assert oracle.decide([1.5, 1.2], 1.0, 1.0) == -1


def test_decide_never_regresses_for_alpha_at_most_one():
    rng = np.random.default_rng(9)
    for _ in range(2000):
        k = int(rng.integers(0, 6))
        t = rng.uniform(0.1, 2.0, k)
        tb = float(rng.uniform(0.1, 2.0))
        alpha = float(rng.uniform(0.5, 1.0))
        c = oracle.decide(t, tb, alpha)
        chosen = tb if c < 0 else t[c]
        assert chosen <= tb                                          # Proposition 1
        if c >= 0:
            assert t[c] == t.min() and t[c] <= alpha * tb
        else:
            assert k == 0 or t.min() > alpha * tb


# ------------------------------------------------------------- adjoints ---
def test_transpose_matches_library_transpose_and_is_stable():
    A, rng = tiny_csr(37, 23, 4.0, seed=41)
    t_rowptr, t_colind, t_val, perm = oracle.csr_transpose(A.rowptr, A.colind, A.val, A.n_cols)
    M = sp.csr_matrix((A.val, A.colind, A.rowptr), shape=(37, 23))
    T = M.T.tocsr()
    T.sort_indices()
    assert np.array_equal(t_rowptr, T.indptr) and np.array_equal(t_colind, T.indices) and np.array_equal(t_val, T.data)
    assert np.array_equal(t_val, A.val[perm])
    rows = np.repeat(np.arange(37), A.degrees)
    assert np.array_equal(t_colind, rows[perm])
    # dense check of the use it is for: d/dB of C = A B is A^T dC
    dC = rng.standard_normal((37, 5)).astype(np.float32)
    dB = oracle.spmm(t_rowptr, t_colind, t_val, dC)
    np.testing.assert_allclose(dB, densify(A).T @ dC.astype(np.float64), rtol=1e-13, atol=1e-13)
    # hand-worked: rows {0: cols 2,0 (unsorted)}, {1: col 2}, {2: cols 2,2 (duplicate)}
    rp = np.array([0, 2, 3, 5], np.int32)
    ci = np.array([2, 0, 2, 2, 2], np.int32)
    va = np.array([1, 2, 3, 4, 5], np.float32)
    t_rowptr, t_colind, t_val, perm = oracle.csr_transpose(rp, ci, va, 3)
    assert t_rowptr.tolist() == [0, 1, 1, 5] and t_colind.tolist() == [0, 0, 1, 2, 2]
    assert t_val.tolist() == [2, 1, 3, 4, 5] and perm.tolist() == [1, 0, 2, 3, 4]


def test_softmax_backward_matches_autograd_and_finite_differences():
    torch = pytest.importorskip("torch")
    A, rng = tiny_csr(15, 15, 4.0, seed=43)
    H = 3
    s = rng.standard_normal((A.nnz, H))
    dP = rng.standard_normal((A.nnz, H))
    P = oracle.row_softmax(A.rowptr, s)
    dS = oracle.row_softmax_backward(A.rowptr, P, dP)
    for i in range(A.n_rows):
        p0, p1 = A.rowptr[i], A.rowptr[i + 1]
        if p1 == p0:
            continue
        x = torch.tensor(s[p0:p1], dtype=torch.float64, requires_grad=True)
        torch.softmax(x, dim=0).backward(torch.tensor(dP[p0:p1]))
        np.testing.assert_allclose(dS[p0:p1], x.grad.numpy(), rtol=1e-11, atol=1e-13)
    # central finite difference of sum(dP * softmax(s)) in one coordinate
    p, h, eps = int(A.rowptr[3]), 1, 1e-6
    sp_, sm_ = s.copy(), s.copy()
    sp_[p, h] += eps
    sm_[p, h] -= eps
    fd = ((oracle.row_softmax(A.rowptr, sp_) - oracle.row_softmax(A.rowptr, sm_)) * dP).sum() / (2 * eps)
    assert abs(fd - dS[p, h]) <= 1e-8
    # each row's gradient sums to zero (softmax is shift invariant)
    sums = np.add.reduceat(dS, A.rowptr[:-1][A.degrees > 0], axis=0)
    np.testing.assert_allclose(sums, 0.0, atol=1e-14)


def test_attention_backward_matches_autograd_of_dense_attention_and_finite_differences():
    """The three gradients against float64 autograd of the textbook masked dense attention, a central finite
    difference through the oracle's own forward, and two structural facts (a column nobody attends to gets no
    gradient; the identity pattern has P = 1, so dV = dO and dQ = dK = 0)."""
    torch = pytest.importorskip("torch")
    n, H, d, scale = 19, 3, 5, 0.4
    A, rng = tiny_csr(n, n, 4.0, seed=47)
    # make column 4 unused so that its K / V rows must receive exactly zero
    cols = [[int(c) for c in A.colind[A.rowptr[i]:A.rowptr[i + 1]] if c != 4] for i in range(n)]
    rowptr = np.concatenate([[0], np.cumsum([len(c) for c in cols])]).astype(np.int32)
    colind = np.array([c for row in cols for c in row], dtype=np.int32)
    Q, K, V = (rng.standard_normal((n, H, d)).astype(np.float32) for _ in range(3))
    dO = rng.standard_normal((n, H, d))
    dQ, dK, dV = oracle.csr_attention_backward(rowptr, colind, Q, K, V, dO, scale)

    tq, tk, tv = (torch.tensor(t, dtype=torch.float64, requires_grad=True) for t in (Q, K, V))
    mask = torch.zeros((n, n), dtype=torch.bool)
    rows = np.repeat(np.arange(n), np.diff(rowptr))
    mask[torch.from_numpy(rows), torch.from_numpy(colind.astype(np.int64))] = True
    S = scale * torch.einsum("ihk,jhk->hij", tq, tk)
    P = torch.nan_to_num(torch.softmax(S.masked_fill(~mask[None], float("-inf")), dim=2), nan=0.0)
    O = torch.einsum("hij,jhk->ihk", P, tv)
    (O * torch.tensor(dO)).sum().backward()
    np.testing.assert_allclose(dQ, tq.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(dK, tk.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(dV, tv.grad.numpy(), rtol=1e-10, atol=1e-12)
    assert np.all(dK[4] == 0.0) and np.all(dV[4] == 0.0)
    empty = np.diff(rowptr) == 0
    assert empty.any() and np.all(dQ[empty] == 0.0)

    def loss(q, k, v):
        return float((oracle.csr_attention(rowptr, colind, q, k, v, scale) * dO).sum())

    for which, grad in ((0, dQ), (1, dK), (2, dV)):
        i, h, c = 6, 1, 2
        ops_p, ops_m = [Q.copy(), K.copy(), V.copy()], [Q.copy(), K.copy(), V.copy()]
        base = float(ops_p[which][i, h, c])
        hi, lo = np.float32(base + 2.0 ** -7), np.float32(base - 2.0 ** -7)        # exactly representable steps
        ops_p[which][i, h, c], ops_m[which][i, h, c] = hi, lo
        fd = (loss(*ops_p) - loss(*ops_m)) / (float(hi) - float(lo))
        assert abs(fd - grad[i, h, c]) <= 2e-4 * max(1.0, abs(grad[i, h, c])), (which, fd, grad[i, h, c])

    eye_ptr, eye_col = np.arange(n + 1, dtype=np.int32), np.arange(n, dtype=np.int32)
    gq, gk, gv = oracle.csr_attention_backward(eye_ptr, eye_col, Q, K, V, dO, scale)
    assert np.array_equal(gv, dO) and np.all(gq == 0.0) and np.all(gk == 0.0)
