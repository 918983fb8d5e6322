"""GPU parity of the adjoint helpers (CSR transpose, value gather, row-softmax backward) against the oracle."""
import numpy as np
import pytest

import oracle
from paper_2511_17594_amd import workloads as W
from util import BACKWARD_FLOOR, dev, rel_l1_rows, rel_l1_segments

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch():
    import torch
    return torch


@pytest.fixture(scope="module")
def ab():
    from paper_2511_17594_amd import binding
    return binding


@pytest.fixture(scope="module")
def handle(ab):
    h = ab.Handle(0)
    yield h
    h.close()


def skew(n_rows, n_cols, seed):
    rng = np.random.default_rng(seed)
    deg = np.minimum(W.powerlaw_degrees(rng, n_rows, 2.1, 12.0, 2500), n_cols)
    deg[3::53] = 0
    return W.csr_from_degrees(rng, deg, n_cols)


def gpu_transpose(torch, handle, A, with_val=True, keep_perm=True):
    nnz = A.nnz
    t_rowptr = torch.full((A.n_cols + 1,), -1, dtype=torch.int32, device="cuda")
    t_colind = torch.full((max(nnz, 1),), -1, dtype=torch.int32, device="cuda")
    t_val = torch.full((max(nnz, 1),), float("nan"), dtype=torch.float32, device="cuda") if with_val else None
    perm = torch.full((max(nnz, 1),), -1, dtype=torch.int32, device="cuda") if keep_perm else None
    ws = torch.empty(handle.csr_transpose_workspace_bytes(A.n_rows, A.n_cols, nnz), dtype=torch.uint8, device="cuda")
    handle.csr_transpose(A.n_rows, A.n_cols, nnz, dev(A.rowptr, torch), dev(A.colind, torch),
                         dev(A.val, torch) if with_val else None, t_rowptr, t_colind, t_val, perm, ws)
    torch.cuda.synchronize()
    return t_rowptr, t_colind, t_val, perm


# column counts that take one, two, three and four 8-bit passes of the sort; nonzero counts from a fraction of a
# 4096-key tile to dozens of tiles with a ragged last one
@pytest.mark.parametrize("n_rows,n_cols", [(5003, 5003), (3000, 777), (400, 9001), (900, 200), (30011, 70001),
                                           (1500, (1 << 24) + 5), (37, 41), (9000, 1), (20000, 2)])
def test_transpose_bit_exact(torch, handle, ab, n_rows, n_cols):
    A = skew(n_rows, n_cols, n_rows)
    o_ptr, o_col, o_val, o_perm = oracle.csr_transpose(A.rowptr, A.colind, A.val, A.n_cols)
    t_rowptr, t_colind, t_val, perm = gpu_transpose(torch, handle, A)
    assert np.array_equal(t_rowptr.cpu().numpy(), o_ptr)
    assert np.array_equal(t_colind.cpu().numpy()[:A.nnz], o_col)
    assert np.array_equal(perm.cpu().numpy()[:A.nnz], o_perm)
    assert np.array_equal(t_val.cpu().numpy()[:A.nnz], o_val)
    # pattern only, permutation kept inside the workspace
    t_rowptr2, t_colind2, _, _ = gpu_transpose(torch, handle, A, with_val=False, keep_perm=False)
    assert torch.equal(t_rowptr2, t_rowptr) and torch.equal(t_colind2, t_colind)
    # gather carries per-nonzero rows of values (e.g. [nnz, H] probabilities) into the transposed order
    vals = torch.randn(A.nnz, 3, device="cuda")
    outv = torch.empty_like(vals)
    handle.gather_values(A.nnz, 3, perm, vals, outv)
    torch.cuda.synchronize()
    assert torch.equal(outv, vals[perm[:A.nnz].long()])


@pytest.mark.parametrize("nnz", [1, 63, 64, 4095, 4096, 4097, 3 * 4096])
def test_transpose_tile_boundaries_and_equal_keys(torch, handle, ab, nnz):
    """Nonzero counts around the sort's tile of 4096 keys; one case with a single column (all keys equal), one with
    every key distinct."""
    for kind in ("one_column", "distinct"):
        if kind == "one_column":
            A = W.CSR(nnz, 1, np.arange(nnz + 1, dtype=np.int32), np.zeros(nnz, np.int32), np.arange(nnz, dtype=np.float32))
        else:
            cols = np.random.default_rng(nnz).permutation(nnz).astype(np.int32)
            A = W.CSR(1, nnz, np.array([0, nnz], np.int32), cols, np.arange(nnz, dtype=np.float32))
        o_ptr, o_col, o_val, o_perm = oracle.csr_transpose(A.rowptr, A.colind, A.val, A.n_cols)
        t_rowptr, t_colind, t_val, perm = gpu_transpose(torch, handle, A)
        assert np.array_equal(t_rowptr.cpu().numpy(), o_ptr), kind
        assert np.array_equal(t_colind.cpu().numpy()[:nnz], o_col), kind
        assert np.array_equal(perm.cpu().numpy()[:nnz], o_perm), kind
        assert np.array_equal(t_val.cpu().numpy()[:nnz], o_val), kind


def test_transpose_degenerate(torch, handle, ab):
    A = W.CSR(7, 5, np.zeros(8, np.int32), np.zeros(0, np.int32), np.zeros(0, np.float32))
    t_rowptr, _, _, _ = gpu_transpose(torch, handle, A)
    assert np.array_equal(t_rowptr.cpu().numpy(), np.zeros(6, np.int32))
    # duplicates and unsorted columns keep storage order
    A = W.CSR(3, 3, np.array([0, 2, 3, 5], np.int32), np.array([2, 0, 2, 2, 2], np.int32), np.arange(1, 6, dtype=np.float32))
    t_rowptr, t_colind, t_val, perm = gpu_transpose(torch, handle, A)
    assert t_rowptr.tolist() == [0, 1, 1, 5] and t_colind.tolist() == [0, 0, 1, 2, 2]
    assert t_val.tolist() == [2, 1, 3, 4, 5] and perm.tolist() == [1, 0, 2, 3, 4]


def test_spmm_adjoint_through_the_transpose(torch, handle, ab):
    """d/dB of C = A B is A^T dC: SpMM on the transposed pattern against the oracle's definition."""
    A = skew(4000, 2500, 5)
    F = 48
    rng = np.random.default_rng(1)
    dC = rng.standard_normal((A.n_rows, F)).astype(np.float32)
    t_rowptr, t_colind, t_val, _ = gpu_transpose(torch, handle, A)
    dB = torch.full((A.n_cols, F), float("nan"), dtype=torch.float32, device="cuda")
    s = ab.Schedule(mapping=ab.MAP_WAVE_ROW, hub_t=256, hub_chunk=256)
    ws = torch.empty(handle.workspace_bytes(ab.OP_SPMM, A.n_cols, A.nnz, F, 1, s), dtype=torch.uint8, device="cuda")
    handle.spmm(A.n_cols, A.n_rows, t_rowptr, t_colind, t_val, dev(dC, torch), dB, F, sched=s, workspace=ws, nnz=A.nnz)
    torch.cuda.synchronize()
    o_ptr, o_col, o_val, _ = oracle.csr_transpose(A.rowptr, A.colind, A.val, A.n_cols)
    ref = oracle.spmm(o_ptr, o_col, o_val, dC)
    ref_abs = oracle.spmm(o_ptr, o_col, np.abs(o_val), np.abs(dC))
    assert rel_l1_rows(dB.cpu().numpy(), ref, ref_abs).max() <= 1e-5


@pytest.mark.parametrize("H,hub_t", [(1, 0), (4, 0), (8, 128), (3, 64), (70, 256)])
def test_softmax_backward(torch, handle, ab, H, hub_t):
    A = skew(3001, 3001, 11)
    rng = np.random.default_rng(H)
    s = (2.0 * rng.standard_normal((A.nnz, H))).astype(np.float32)
    P64 = oracle.row_softmax(A.rowptr, s)
    P = P64.astype(np.float32)
    dP = rng.standard_normal((A.nnz, H)).astype(np.float32)
    ref = oracle.row_softmax_backward(A.rowptr, P, dP)
    ref_abs = oracle.row_softmax_backward(A.rowptr, P, -np.abs(dP))      # all terms of one sign: magnitude of the terms
    d_rp, d_P, d_dP = dev(A.rowptr, torch), dev(P, torch), dev(dP, torch)
    dS = torch.full_like(d_dP, float("nan"))
    ws = torch.empty(handle.workspace_bytes(ab.OP_SOFTMAX, A.n_rows, A.nnz, 1, H, ab.Schedule(hub_t=hub_t)), dtype=torch.uint8,
                     device="cuda")
    handle.csr_row_softmax_backward(A.n_rows, A.nnz, d_rp, d_P, d_dP, dS, H=H, hub_t=hub_t, workspace=ws)
    torch.cuda.synchronize()
    got = dS.cpu().numpy()
    assert np.isfinite(got).all()
    scale = np.abs(P.astype(np.float64)) * (np.abs(dP.astype(np.float64)) + np.abs(ref_abs / np.maximum(P64, 1e-300) + np.abs(dP)))
    for h in range(H):
        err = rel_l1_segments(got[:, h], ref[:, h], A.rowptr, scale[:, h], floors=(BACKWARD_FLOOR, BACKWARD_FLOOR))
        assert err.max() <= 1e-5, (H, h, float(err.max()))
    # in place on dP
    handle.csr_row_softmax_backward(A.n_rows, A.nnz, d_rp, d_P, d_dP, d_dP, H=H, hub_t=hub_t, workspace=ws)
    torch.cuda.synchronize()
    assert np.array_equal(d_dP.cpu().numpy(), got)


def as_f64(t, shape):
    if t.dtype == np.uint16:
        return W.bf16_bits_to_float(t).reshape(shape).astype(np.float64)
    return np.asarray(t, dtype=np.float64).reshape(shape)


def gradient_term_magnitudes(A, Q, K, V, dO, scale):
    """The sums of the magnitudes of the terms of dQ, dK, dV (the same chain rule on absolute values, with the
    oracle's probabilities): the scale of the rounding error of a gradient that cancels, e.g. under a
    saturated softmax where dS = P (dP - sum P dP) is a difference of nearly equal numbers."""
    n, H, d = dO.shape
    _, _, P = oracle.csr_attention(A.rowptr, A.colind, Q, K, V, scale, return_scores=True)
    rows = np.repeat(np.arange(n), A.degrees)
    cols = A.colind.astype(np.int64)
    q, k, v, g = (np.abs(as_f64(t, (n, H, d))) for t in (Q, K, V, dO))
    adP = np.einsum("phk,phk->ph", g[rows], v[cols])
    rowdot = np.zeros((n, H))
    np.add.at(rowdot, rows, P * adP)
    adS = scale * P * (adP + rowdot[rows])
    mQ, mK, mV = (np.zeros((n, H, d)) for _ in range(3))
    np.add.at(mQ, rows, adS[:, :, None] * k[cols])
    np.add.at(mK, cols, adS[:, :, None] * q[rows])
    np.add.at(mV, cols, P[:, :, None] * g[rows])
    return mQ, mK, mV


@pytest.mark.parametrize("H,d,dtype,hub_t,qk_std", [
    (8, 64, "bf16", 256, 1.0), (8, 64, "bf16", 0, None), (2, 32, "f16", 128, 2.0), (1, 128, "bf16", 64, 1.0),
    (4, 16, "f32", 256, 1.0), (3, 16, "bf16", 512, 1.0), (8, 64, "f32", 0, 1.0),
])
@pytest.mark.parametrize("one_pass", [1, 0])
def test_attention_backward(torch, handle, ab, H, d, dtype, hub_t, qk_std, one_pass):
    """dQ, dK, dV of the library against the oracle's chain rule, on a skewed square pattern with hub rows in
    the pattern and in its transpose, empty rows, and columns nobody attends to; with the pattern-side half taken
    in one pass over K and V (where the shape has such kernels) and stage by stage."""
    from util import dtype_code
    n = 3001
    A = skew(n, n - 40, seed=900 + H + d)
    A = W.CSR(n, n, A.rowptr, A.colind, A.val)          # square, the last 40 columns never attended to
    Qb, Kb, Vb = W.config5_attention(n, H, d, seed=H * 10 + d, qk_std=qk_std)
    if dtype == "bf16":
        Q, K, V, tol = Qb, Kb, Vb, 2e-2
    elif dtype == "f16":
        Q, K, V = (W.bf16_bits_to_float(t).reshape(n, H, d).astype(np.float16) for t in (Qb, Kb, Vb))
        tol = 2e-2
    else:
        Q, K, V = (np.ascontiguousarray(W.bf16_bits_to_float(t).reshape(n, H, d) * np.float32(1.001), dtype=np.float32)
                   for t in (Qb, Kb, Vb))
        tol = 1e-4                                     # six fp32 stages stacked on each other
    scale = float(d) ** -0.5
    dO = np.random.default_rng(5).standard_normal((n, H, d)).astype(np.float32)
    ref = oracle.csr_attention_backward(A.rowptr, A.colind, Q, K, V, dO, scale)
    ref_abs = gradient_term_magnitudes(A, Q, K, V, dO, scale)
    t_rowptr, t_colind, _, perm = gpu_transpose(torch, handle, A, with_val=False)
    outs = [torch.full((n, H, d), float("nan"), dtype=torch.float32, device="cuda") for _ in range(3)]
    ws = torch.empty(handle.csr_attention_backward_workspace_bytes(n, A.nnz, H, d, hub_t), dtype=torch.uint8, device="cuda")
    print("attention backward H %d d %d %s hub %d one pass %d" % (H, d, dtype, hub_t, one_pass), flush=True)
    handle.set_param("attention_backward_fused", one_pass)
    handle.csr_attention_backward(n, dev(A.rowptr, torch), dev(A.colind, torch), t_rowptr, t_colind, perm,
                                  dev(Q, torch), dev(K, torch), dev(V, torch), dev(dO, torch), *outs, H, d, scale,
                                  in_dt=dtype_code(ab, Q), hub_t=hub_t, workspace=ws, nnz=A.nnz)
    torch.cuda.synchronize()
    handle.set_param("attention_backward_fused", 1)
    unused = np.setdiff1d(np.arange(n), A.colind)
    assert unused.size > 0
    for name, got_t, want, mag in zip(("dQ", "dK", "dV"), outs, ref, ref_abs):
        got = got_t.cpu().numpy()
        assert np.isfinite(got).all(), name
        err = rel_l1_rows(got.reshape(n * H, d), want.reshape(n * H, d), mag.reshape(n * H, d))
        # rows whose gradient vanishes (empty rows, unused columns) must be exactly zero; the rest within tolerance
        zero = np.abs(want.reshape(n * H, d)).sum(axis=1) == 0
        assert np.all(got.reshape(n * H, d)[zero] == 0.0), name
        assert err[~zero].max() <= tol, (name, float(err[~zero].max()), int(np.argmax(err * ~zero)))
        if dtype != "f32":
            assert err[~zero].max() <= 5e-4, (name, float(err[~zero].max()))     # exact inputs, fp32 arithmetic only
    assert np.all(outs[1].cpu().numpy()[unused] == 0.0) and np.all(outs[2].cpu().numpy()[unused] == 0.0)
    assert np.all(outs[0].cpu().numpy()[A.degrees == 0] == 0.0)
