"""The torch.ops.autosage operators: forward values and autograd gradients against dense float64
PyTorch CPU formulas (masked dense matmul / softmax / attention with autograd as the reference)."""
import numpy as np
import pytest

from paper_2511_17594_amd import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch():
    import torch
    return torch


@pytest.fixture(scope="module")
def ops(torch):
    from paper_2511_17594_amd import torch_ops
    return torch_ops


@pytest.fixture(scope="module")
def graph():
    rng = np.random.default_rng(3)
    n_rows, n_cols = 700, 900
    deg = rng.poisson(5.0, n_rows)
    deg[7] = 850                     # longer than a wavefront's index block many times over
    deg[11] = 0
    return W.csr_from_degrees(rng, deg, n_cols)


def rel(a, b):
    a, b = a.detach().double().cpu(), b.detach().double().cpu()
    return float((a - b).abs().sum() / b.abs().sum().clamp_min(1e-30))


def dense_of(torch, A, val):
    rows = torch.from_numpy(np.repeat(np.arange(A.n_rows), A.degrees))
    cols = torch.from_numpy(A.colind.astype(np.int64))
    D = torch.zeros((A.n_rows, A.n_cols), dtype=torch.float64)
    return D.index_put((rows, cols), val, accumulate=True), rows, cols


def test_ops_are_registered(torch, ops):
    for name in ("spmm_csr", "spmm_csr_split", "sddmm_csr", "csr_row_softmax", "csr_attention_forward"):
        assert hasattr(torch.ops.autosage, name)


@pytest.mark.parametrize("split", [False, True])
def test_spmm_forward_and_gradients(torch, ops, graph, split):
    A, F = graph, 24
    g = torch.Generator().manual_seed(1)
    val64 = torch.from_numpy(A.val.astype(np.float64)).requires_grad_(True)
    B64 = torch.randn(A.n_cols, F, dtype=torch.float64, generator=g).requires_grad_(True)
    Wt = torch.randn(A.n_rows, F, dtype=torch.float64, generator=g)
    D, _, _ = dense_of(torch, A, val64)
    (D @ B64 * Wt).sum().backward()
    rp, ci = torch.from_numpy(A.rowptr).cuda(), torch.from_numpy(A.colind).cuda()
    val = val64.detach().float().cuda().requires_grad_(True)
    B = B64.detach().float().cuda().requires_grad_(True)
    C = torch.ops.autosage.spmm_csr_split(rp, ci, val, B, 256) if split else torch.ops.autosage.spmm_csr(rp, ci, val, B)
    assert rel(C, D @ B64) <= 1e-5
    (C * Wt.float().cuda()).sum().backward()
    assert rel(B.grad, B64.grad) <= 1e-5 and rel(val.grad, val64.grad) <= 1e-5


def test_sddmm_forward_and_gradients(torch, ops, graph):
    A, F = graph, 20
    g = torch.Generator().manual_seed(2)
    X64 = torch.randn(A.n_rows, F, dtype=torch.float64, generator=g).requires_grad_(True)
    Y64 = torch.randn(A.n_cols, F, dtype=torch.float64, generator=g).requires_grad_(True)
    w = torch.randn(A.nnz, dtype=torch.float64, generator=g)
    _, rows, cols = dense_of(torch, A, torch.zeros(A.nnz, dtype=torch.float64))
    ref = (X64[rows] * Y64[cols]).sum(dim=1)
    (ref * w).sum().backward()
    rp, ci = torch.from_numpy(A.rowptr).cuda(), torch.from_numpy(A.colind).cuda()
    X = X64.detach().float().cuda().requires_grad_(True)
    Y = Y64.detach().float().cuda().requires_grad_(True)
    out = torch.ops.autosage.sddmm_csr(rp, ci, X, Y)
    assert rel(out, ref) <= 1e-5
    (out * w.float().cuda()).sum().backward()
    assert rel(X.grad, X64.grad) <= 1e-5 and rel(Y.grad, Y64.grad) <= 1e-5


def test_softmax_and_attention_gradients(torch, ops, graph):
    rng = np.random.default_rng(5)
    n = 600
    deg = rng.poisson(6.0, n)
    deg[5] = 580
    deg[9] = 0
    A = W.csr_from_degrees(rng, deg, n)
    H, d, scale = 2, 16, 0.25
    g = torch.Generator().manual_seed(3)
    Q64, K64, V64 = (torch.randn(n, H, d, dtype=torch.float64, generator=g).requires_grad_(True) for _ in range(3))
    Wt = torch.randn(n, H, d, dtype=torch.float64, generator=g)
    mask = torch.zeros((n, n), dtype=torch.bool)
    rows = torch.from_numpy(np.repeat(np.arange(n), A.degrees))
    cols = torch.from_numpy(A.colind.astype(np.int64))
    mask[rows, cols] = True
    S = scale * torch.einsum("ihk,jhk->hij", Q64, K64)
    S = S.masked_fill(~mask[None], float("-inf"))
    P = torch.softmax(S, dim=2)
    P = torch.nan_to_num(P, nan=0.0)                     # the empty row
    O_ref = torch.einsum("hij,jhk->ihk", P, V64)
    (O_ref * Wt).sum().backward()
    rp, ci = torch.from_numpy(A.rowptr).cuda(), torch.from_numpy(A.colind).cuda()
    Q, K, V = (t.detach().float().cuda().requires_grad_(True) for t in (Q64, K64, V64))
    O = torch.ops.autosage.csr_attention_forward(rp, ci, Q, K, V, scale)
    assert rel(O, O_ref) <= 2e-5
    (O * Wt.float().cuda()).sum().backward()
    assert rel(Q.grad, Q64.grad) <= 5e-5 and rel(K.grad, K64.grad) <= 5e-5 and rel(V.grad, V64.grad) <= 5e-5
    # row-softmax alone, two heads
    s64 = torch.randn(A.nnz, H, dtype=torch.float64, generator=g).requires_grad_(True)
    w = torch.randn(A.nnz, H, dtype=torch.float64, generator=g)
    dense = torch.full((H, n, n), float("-inf"), dtype=torch.float64)
    dense = dense.index_put((torch.arange(H)[:, None], rows[None], cols[None]), s64.T)
    Pd = torch.nan_to_num(torch.softmax(dense, dim=2), nan=0.0)
    ref = Pd[:, rows, cols].T
    (ref * w).sum().backward()
    s = s64.detach().float().cuda().requires_grad_(True)
    P_gpu = torch.ops.autosage.csr_row_softmax(rp, s)
    assert rel(P_gpu, ref) <= 1e-5
    (P_gpu * w.float().cuda()).sum().backward()
    assert rel(s.grad, s64.grad) <= 1e-5
    # bf16 operands: forward runs in the bf16 kernels, gradients come back in bf16
    Qb, Kb, Vb = (t.detach().to(torch.bfloat16).cuda().requires_grad_(True) for t in (Q64, K64, V64))
    Ob = torch.ops.autosage.csr_attention_forward(rp, ci, Qb, Kb, Vb, scale)
    assert rel(Ob, O_ref) <= 2e-2
    (Ob * Wt.float().cuda()).sum().backward()
    assert Qb.grad.dtype == torch.bfloat16 and rel(Qb.grad, Q64.grad) <= 3e-2 and rel(Vb.grad, V64.grad) <= 3e-2


def test_int64_indices_enter_through_the_narrowing_call(torch, ops, graph):
    """64-bit CSR index tensors are narrowed on the device: equal to the int32 originals bit for bit, and a
    value that does not fit the stated limit is an error, not a truncation."""
    from paper_2511_17594_amd import binding as ab
    A = graph
    rp64 = torch.from_numpy(A.rowptr.astype(np.int64)).cuda()
    ci64 = torch.from_numpy(A.colind.astype(np.int64)).cuda()
    rp, ci = ops.csr_indices_int32(rp64, ci64, A.n_cols)
    assert rp.dtype == torch.int32 and ci.dtype == torch.int32
    assert np.array_equal(rp.cpu().numpy(), A.rowptr) and np.array_equal(ci.cpu().numpy(), A.colind)
    same = ops.csr_indices_int32(rp, ci, A.n_cols)
    assert same[0] is rp and same[1] is ci
    with pytest.raises(ab.AutosageError):
        ops.csr_indices_int32(rp64, ci64, int(A.colind.max()))          # n_cols one too small for the largest column
    bad = rp64.clone()
    bad[3] = 2 ** 31 + 5
    with pytest.raises(ab.AutosageError):
        ops.csr_indices_int32(bad, ci64, A.n_cols)
    neg = ci64.clone()
    neg[0] = -1
    with pytest.raises(ab.AutosageError):
        ops.csr_indices_int32(rp64, neg, A.n_cols)
    empty = ops.csr_indices_int32(torch.zeros(1, dtype=torch.int64, device="cuda"),
                                  torch.zeros(0, dtype=torch.int64, device="cuda"), 5)
    assert empty[0].tolist() == [0] and empty[1].numel() == 0


def test_gradients_follow_the_pattern_when_index_memory_is_recycled(torch, ops):
    """Mini-batches with a fixed fan-out give one pattern after the other with the same number of nonzeros, the
    first freed before the second is allocated: the transposed-pattern cache and the library's per-address memory of
    degree features must never hand the second pattern the first one's transpose or features."""
    import oracle
    n, fan, F = 600, 8, 16
    rng = np.random.default_rng(5)
    seen_ptrs = []
    for batch in range(3):
        deg = np.full(n, fan, dtype=np.int64)
        A = W.csr_from_degrees(rng, deg, n)                      # same rows, columns and nonzeros every time
        assert A.nnz == n * fan
        B_h = rng.standard_normal((n, F)).astype(np.float32)
        Wt_h = rng.standard_normal((n, F)).astype(np.float32)
        rp, ci = torch.from_numpy(A.rowptr).cuda(), torch.from_numpy(A.colind).cuda()
        seen_ptrs.append((rp.data_ptr(), ci.data_ptr()))
        val = torch.from_numpy(A.val).cuda().requires_grad_(True)
        B = torch.from_numpy(B_h).cuda().requires_grad_(True)
        C = torch.ops.autosage.spmm_csr(rp, ci, val, B)
        (C * torch.from_numpy(Wt_h).cuda()).sum().backward()
        # dL/dB = A^T W through the oracle: SpMM on the oracle's own transpose of this batch's pattern
        t_rp, t_ci, t_val, _ = oracle.csr_transpose(A.rowptr, A.colind, A.val, n)
        want_dB = oracle.spmm(t_rp, t_ci, t_val, Wt_h)
        want_dval = oracle.sddmm(A.rowptr, A.colind, Wt_h, B_h)
        assert rel(B.grad, torch.from_numpy(want_dB)) <= 1e-5, batch
        assert rel(val.grad, torch.from_numpy(want_dval)) <= 1e-5, batch
        del rp, ci, val, B, C                                     # freed before the next batch is allocated
    # while an entry of either cache lives it pins its index tensors, so no two batches shared an address
    assert len(set(seen_ptrs)) == len(seen_ptrs)


def test_overwritten_rowptr_is_not_replayed(torch, ops):
    """A rowptr tensor overwritten in place with another graph of the same sizes: the operator notices the new
    tensor version, the library forgets the address, and the decision carries the new graph's signature."""
    import oracle
    n, F = 4096, 32
    rng = np.random.default_rng(6)
    deg1 = rng.poisson(6.0, n).astype(np.int64)
    deg2 = rng.permutation(deg1)                                  # same rows, same nonzeros, another graph
    A1, A2 = W.csr_from_degrees(rng, deg1, n), W.csr_from_degrees(rng, deg2, n)
    assert A1.nnz == A2.nnz and not np.array_equal(A1.rowptr, A2.rowptr)
    rp, ci = torch.from_numpy(A1.rowptr).cuda(), torch.from_numpy(A1.colind).cuda()
    val = torch.from_numpy(A1.val).cuda()
    B_h = rng.standard_normal((n, F)).astype(np.float32)
    B = torch.from_numpy(B_h).cuda()
    h = ops.handle(B.device)
    C1 = torch.ops.autosage.spmm_csr(rp, ci, val, B)
    sig1 = h.last_decision()["graph_sig"]
    assert int(sig1, 16) == oracle.graph_signature(A1.rowptr, n)
    rp.copy_(torch.from_numpy(A2.rowptr))
    ci.copy_(torch.from_numpy(A2.colind))
    val.copy_(torch.from_numpy(A2.val))
    C2 = torch.ops.autosage.spmm_csr(rp, ci, val, B)
    sig2 = h.last_decision()["graph_sig"]
    assert int(sig2, 16) == oracle.graph_signature(A2.rowptr, n) and sig2 != sig1
    assert rel(C1, torch.from_numpy(oracle.spmm(A1.rowptr, A1.colind, A1.val, B_h))) <= 1e-5
    assert rel(C2, torch.from_numpy(oracle.spmm(A2.rowptr, A2.colind, A2.val, B_h))) <= 1e-5
