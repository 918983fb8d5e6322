"""GPU parity at the full sizes of the five configurations, in the launch configuration the
benchmark times (schedule chosen by the selector), checked on sampled rows that the oracle
computes one by one, plus properties that hold at any size.  Configs 3 and 4 are synthetic
stand-ins shaped like the paper's two real graphs (same rows / nonzeros / degree character)."""
import numpy as np
import pytest

import oracle
from paper_2511_17594_amd import workloads as W
from util import dev, rel_l1_rows, rel_l1_segments

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


def sample_rows(A, k, seed):
    """k random rows plus the 16 rows of largest degree."""
    rng = np.random.default_rng(seed)
    rows = rng.choice(A.n_rows, size=min(k, A.n_rows), replace=False)
    top = np.argsort(A.degrees)[-16:]
    return np.unique(np.concatenate([rows, top]))


def check_spmm(torch, ab, handle, A, d_csr, F, rows, seed, sched=None):
    rng = np.random.default_rng(seed)
    B = rng.standard_normal((A.n_cols, F), dtype=np.float32)
    dB = dev(B, torch)
    C = torch.full((A.n_rows, F), float("nan"), dtype=torch.float32, device="cuda")
    ws = torch.empty(handle.workspace_bytes(ab.OP_SPMM, A.n_rows, A.nnz, F), dtype=torch.uint8, device="cuda")
    handle.spmm(A.n_rows, A.n_cols, *d_csr, dB, C, F, sched=sched, workspace=ws)
    torch.cuda.synchronize()
    got = C[torch.from_numpy(rows).cuda()].cpu().numpy()
    assert bool(torch.isfinite(C).all())
    As = W.row_slice(A, rows)
    ref = oracle.spmm(As.rowptr, As.colind, As.val, B)
    ref_abs = oracle.spmm(As.rowptr, As.colind, np.abs(As.val), np.abs(B))
    err = rel_l1_rows(got, ref, ref_abs)
    assert err.max() <= 1e-5, (F, float(err.max()), int(rows[err.argmax()]))
    return C


def check_sddmm(torch, ab, handle, A, d_csr, F, rows, seed, sched=None):
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((A.n_rows, F), dtype=np.float32)
    Y = rng.standard_normal((A.n_cols, F), dtype=np.float32)
    out = torch.full((A.nnz,), float("nan"), dtype=torch.float32, device="cuda")
    ws = torch.empty(handle.workspace_bytes(ab.OP_SDDMM, A.n_rows, A.nnz, F), dtype=torch.uint8, device="cuda")
    handle.sddmm(A.n_rows, A.n_cols, d_csr[0], d_csr[1], dev(X, torch), dev(Y, torch), out, F, sched=sched, workspace=ws)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(out).all())
    As = W.row_slice(A, rows)
    rp = A.rowptr.astype(np.int64)
    idx = np.concatenate([np.arange(rp[r], rp[r + 1]) for r in rows]) if rows.size else np.zeros(0, np.int64)
    got = out[torch.from_numpy(idx).cuda()].cpu().numpy()
    Xs = np.ascontiguousarray(X[rows])
    ref = oracle.sddmm(As.rowptr, As.colind, Xs, Y)
    ref_abs = oracle.sddmm(As.rowptr, As.colind, np.abs(Xs), np.abs(Y))
    err = rel_l1_segments(got, ref, As.rowptr, ref_abs)
    assert err.max() <= 1e-5, (F, float(err.max()), int(rows[err.argmax()]))


def test_config1_tiny_full_compare(torch, ab, handle):
    A, B, X, Y = W.config1_tiny()
    assert A.n_rows == 4096 and abs(A.nnz / 4096 - 16) < 1
    d_csr = (dev(A.rowptr, torch), dev(A.colind, torch), dev(A.val, torch))
    C = torch.empty((4096, 32), dtype=torch.float32, device="cuda")
    out = torch.empty(A.nnz, dtype=torch.float32, device="cuda")
    ws = torch.empty(handle.workspace_bytes(ab.OP_SPMM, 4096, A.nnz, 32), dtype=torch.uint8, device="cuda")
    handle.spmm(4096, 4096, *d_csr, dev(B, torch), C, 32, workspace=ws)
    handle.sddmm(4096, 4096, d_csr[0], d_csr[1], dev(X, torch), dev(Y, torch), out, 32, workspace=ws)
    torch.cuda.synchronize()
    ref = oracle.spmm(A.rowptr, A.colind, A.val, B)
    ref_abs = oracle.spmm(A.rowptr, A.colind, np.abs(A.val), np.abs(B))
    assert rel_l1_rows(C.cpu().numpy(), ref, ref_abs).max() <= 1e-5
    ref = oracle.sddmm(A.rowptr, A.colind, X, Y)
    ref_abs = oracle.sddmm(A.rowptr, A.colind, np.abs(X), np.abs(Y))
    assert rel_l1_segments(out.cpu().numpy(), ref, A.rowptr, ref_abs).max() <= 1e-5


@pytest.fixture(scope="module")
def config2():
    A = W.config2_powerlaw()
    assert A.n_rows == 262144 and A.nnz == 262144 * 32 and A.degrees.max() == 65536
    return A


@pytest.mark.parametrize("F", [8, 64, 256])
def test_config2_powerlaw_full_size(torch, ab, handle, config2, F):
    A = config2
    d_csr = (dev(A.rowptr, torch), dev(A.colind, torch), dev(A.val, torch))
    rows = sample_rows(A, 1500, F)
    check_spmm(torch, ab, handle, A, d_csr, F, rows, seed=F)
    assert handle.last_decision()["choice"]["hub_t"] > 0             # 65536-long rows must not stay on one wavefront
    check_sddmm(torch, ab, handle, A, d_csr, F, rows, seed=F + 1)
    # the fallback itself is also correct at full size (one width is enough: it is slow on the hub rows)
    if F == 64:
        check_spmm(torch, ab, handle, A, d_csr, F, rows, seed=F, sched=ab.baseline_schedule())
    # metadata at full size, bit exact
    n = A.n_rows
    hub_rows = torch.empty(n, dtype=torch.int32, device="cuda")
    chunk_ptr = torch.empty(n + 1, dtype=torch.int32, device="cuda")
    light_rows = torch.empty(n, dtype=torch.int32, device="cuda")
    ws = torch.empty(1 << 20, dtype=torch.uint8, device="cuda")
    nh, nl = handle.hub_partition(n, d_csr[0], 1024, 1024, hub_rows, chunk_ptr, light_rows, ws)
    o_hub, o_ptr, o_light = oracle.hub_partition(A.rowptr, 1024, 1024)
    assert np.array_equal(hub_rows.cpu().numpy()[:nh], o_hub) and np.array_equal(chunk_ptr.cpu().numpy()[:nh + 1], o_ptr)
    assert np.array_equal(light_rows.cpu().numpy()[:nl], o_light)
    hist, mx, nnz, sig = handle.graph_features(n, n, d_csr[0])
    assert sig == oracle.graph_signature(A.rowptr, n) and mx == 65536 and nnz == A.nnz


def test_config5_attention_full_size(torch, ab, handle, config2):
    A, H, d = config2, 8, 64
    scale = d ** -0.5
    rows = sample_rows(A, 600, 5)
    As = W.row_slice(A, rows)
    for qk_std in (None, 1.0):                                           # the config's flat softmax and a peaked one
        Q, K, V = W.config5_attention(A.n_rows, H, d, seed=0, qk_std=qk_std)
        d_in = [dev(t, torch) for t in (A.rowptr, A.colind, Q, K, V)]
        ref = oracle.csr_attention(As.rowptr, As.colind, np.ascontiguousarray(Q[rows]), K, V, scale)
        vmax = float(np.abs(W.bf16_bits_to_float(V)).max())
        for sched in (None, ab.Schedule(mapping=ab.MAP_WAVE_ROW, hub_t=1024, hub_chunk=1024)):   # default, three stages
            O = torch.full((A.n_rows, H, d), float("nan"), dtype=torch.float32, device="cuda")
            ws = torch.empty(handle.workspace_bytes(ab.OP_ATTENTION, A.n_rows, A.nnz, d, H, sched), dtype=torch.uint8,
                             device="cuda")
            handle.csr_attention(A.n_rows, *d_in, O, H, d, scale, sched=sched, workspace=ws)
            torch.cuda.synchronize()
            if sched is None:
                assert handle.last_decision()["choice"]["hub_t"] > 0          # the selector splits the 65536-long rows
            assert bool(torch.isfinite(O).all())
            got = O[torch.from_numpy(rows).cuda()].cpu().numpy()
            err = rel_l1_rows(got.reshape(-1, d), ref.reshape(-1, d))
            assert err.max() <= 2e-2, (qk_std, float(err.max()))
            # every output row is a convex combination of V rows: bounded by the extreme V value
            assert float(O.abs().max()) <= vmax * (1 + 1e-5)
            del O, ws


def test_config3_community_full_size(torch, ab, handle):
    A = W.config3_community()
    assert A.n_rows == 232965 and abs(A.nnz / 114.6e6 - 1) < 0.03
    d_csr = (dev(A.rowptr, torch), dev(A.colind, torch), dev(A.val, torch))
    rows = sample_rows(A, 300, 3)
    for F in (128, 602):
        check_spmm(torch, ab, handle, A, d_csr, F, rows, seed=F)
    # val = 1/deg(i): A times the all-ones matrix is all ones (any size, no oracle needed)
    F = 32
    ones = torch.ones((A.n_cols, F), dtype=torch.float32, device="cuda")
    C = torch.empty((A.n_rows, F), dtype=torch.float32, device="cuda")
    ws = torch.empty(handle.workspace_bytes(ab.OP_SPMM, A.n_rows, A.nnz, F), dtype=torch.uint8, device="cuda")
    handle.spmm(A.n_rows, A.n_cols, *d_csr, ones, C, F, workspace=ws)
    torch.cuda.synchronize()
    assert float((C - 1.0).abs().max()) <= 2e-5


def test_config4_large_sparse_full_size(torch, ab, handle):
    A = W.config4_large()
    assert A.n_rows == 2449029 and abs(A.nnz / 123.7e6 - 1) < 0.03
    d_csr = (dev(A.rowptr, torch), dev(A.colind, torch), dev(A.val, torch))
    rows = sample_rows(A, 1500, 4)
    check_spmm(torch, ab, handle, A, d_csr, 100, rows, seed=100)
    check_sddmm(torch, ab, handle, A, d_csr, 16, rows, seed=16)
    check_sddmm(torch, ab, handle, A, d_csr, 128, rows, seed=128)
    # bf16 dense operands with fp32 accumulation (the paper's mixed-precision extension), F = 128
    rng = np.random.default_rng(7)
    F = 128
    Bb = W.float_to_bf16_bits(rng.standard_normal((A.n_cols, F), dtype=np.float32)).reshape(A.n_cols, F)
    Xb = W.float_to_bf16_bits(rng.standard_normal((A.n_rows, F), dtype=np.float32)).reshape(A.n_rows, F)
    dB, dX = dev(Bb, torch), dev(Xb, torch)
    C = torch.full((A.n_rows, F), float("nan"), dtype=torch.float32, device="cuda")
    out = torch.full((A.nnz,), float("nan"), dtype=torch.float32, device="cuda")
    ws = torch.empty(handle.workspace_bytes(ab.OP_SPMM, A.n_rows, A.nnz, F), dtype=torch.uint8, device="cuda")
    handle.spmm(A.n_rows, A.n_cols, *d_csr, dB, C, F, dt=ab.BF16, workspace=ws)
    handle.sddmm(A.n_rows, A.n_cols, d_csr[0], d_csr[1], dX, dB, out, F, dt=ab.BF16, workspace=ws)
    torch.cuda.synchronize()
    As = W.row_slice(A, rows)
    absb = lambda x: x & np.uint16(0x7FFF)
    ref = oracle.spmm(As.rowptr, As.colind, As.val, Bb)
    ref_abs = oracle.spmm(As.rowptr, As.colind, np.abs(As.val), absb(Bb))
    got = C[torch.from_numpy(rows).cuda()].cpu().numpy()
    assert rel_l1_rows(got, ref, ref_abs).max() <= 2e-2
    rp = A.rowptr.astype(np.int64)
    idx = np.concatenate([np.arange(rp[r], rp[r + 1]) for r in rows])
    Xs = np.ascontiguousarray(Xb[rows])
    ref = oracle.sddmm(As.rowptr, As.colind, Xs, Bb)
    ref_abs = oracle.sddmm(As.rowptr, As.colind, absb(Xs), absb(Bb))
    got = out[torch.from_numpy(idx).cuda()].cpu().numpy()
    assert rel_l1_segments(got, ref, As.rowptr, ref_abs).max() <= 2e-2
