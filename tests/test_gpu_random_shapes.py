"""Seeded random sweep of shapes and schedules against the oracle: rectangular matrices, empty rows, rows with
duplicate and unsorted columns, one long row, random widths, element types, mappings, vector widths, unrolls,
split thresholds and chunk lengths.  A schedule the library declares unsupported for a shape is skipped; a
schedule it accepts must match the oracle to the tolerance of its element type."""
import numpy as np
import pytest

import oracle
from paper_2511_17594_amd import workloads as W
from util import dev, dtype_code, rel_l1_rows, rel_l1_segments

pytestmark = pytest.mark.gpu

WIDTHS = [1, 2, 3, 4, 7, 8, 12, 16, 24, 32, 40, 64, 96, 100, 128, 130, 192, 256, 300, 512]


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


def random_matrix(rng):
    n_rows, n_cols = int(rng.integers(1, 2500)), int(rng.integers(1, 2500))
    kind = rng.integers(0, 3)
    if kind == 0:
        deg = rng.poisson(rng.uniform(0.5, 40.0), size=n_rows)
    elif kind == 1 and n_rows >= 50:
        deg = W.powerlaw_degrees(rng, n_rows, 2.1, float(rng.uniform(2.0, 30.0)), None)
    else:
        deg = rng.integers(0, 3, size=n_rows)
    deg = np.minimum(deg, n_cols).astype(np.int64)
    deg[rng.integers(0, n_rows, size=max(1, n_rows // 10))] = 0                 # empty rows
    deg[rng.integers(0, n_rows)] = min(n_cols, int(rng.integers(200, 4000)))    # one long row
    A = W.csr_from_degrees(rng, deg, n_cols)
    if A.nnz and rng.random() < 0.5:                                             # duplicates and unsorted rows
        ci = A.colind.copy()
        pick = rng.integers(0, A.nnz, size=max(1, A.nnz // 20))
        ci[pick] = ci[np.maximum(pick - 1, 0)]
        rp = A.rowptr.astype(np.int64)
        r = int(np.argmax(deg))
        ci[rp[r]:rp[r + 1]] = ci[rp[r]:rp[r + 1]][::-1]
        A = W.CSR(A.n_rows, A.n_cols, A.rowptr, np.ascontiguousarray(ci), A.val)
    return A


def random_schedule(rng, ab):
    s = ab.Schedule()
    s.mapping = int(rng.choice([0, 1, 1, 1, 2]))
    s.vec_bytes = int(rng.choice([0, 0, 4, 8, 16])) if s.mapping else 0
    s.unroll = int(rng.choice([0, 1, 2, 4, 8])) if s.mapping else 0
    s.waves_per_wg = int(rng.choice([0, 1, 2, 4, 8, 16]))
    s.hub_t = int(rng.choice([0, 0, 64, 100, 256, 1000]))
    s.hub_chunk = int(rng.choice([0, 64, 77, 512])) if s.hub_t else 0
    s.xcd_remap = int(rng.integers(0, 2))
    s.f_tile = int(rng.choice([0, 0, 0, 32, 64])) if s.mapping == 1 else (64 if s.mapping == 0 else 0)
    return s


def operands(rng, rows, F, kind):
    x = rng.standard_normal((rows, F)).astype(np.float32)
    if kind == "bf16":
        return W.float_to_bf16_bits(x).reshape(rows, F), (lambda t: t & np.uint16(0x7FFF))
    if kind == "f16":
        return x.astype(np.float16), np.abs
    return x, np.abs


@pytest.mark.parametrize("seed", range(48))
def test_random_shape_and_schedule(torch, ab, handle, seed):
    rng = np.random.default_rng(9000 + seed)
    A = random_matrix(rng)
    F = int(rng.choice(WIDTHS))
    kind = str(rng.choice(["f32", "f32", "bf16", "f16"]))
    tol = 1e-5                                                   # 16-bit inputs are exact on both sides
    B, absf = operands(rng, A.n_cols, F, kind)
    X, _ = operands(rng, A.n_rows, F, kind)
    s = random_schedule(rng, ab)
    tag = (seed, A.n_rows, A.n_cols, A.nnz, F, kind, s.as_dict())
    print(tag, flush=True)
    d_rp, d_ci, d_v, d_B, d_X = (dev(t, torch) for t in (A.rowptr, A.colind, A.val, B, X))
    dt = dtype_code(ab, B)
    for op in ("spmm", "sddmm"):
        try:
            nbytes = handle.workspace_bytes(ab.OP_SPMM if op == "spmm" else ab.OP_SDDMM, A.n_rows, A.nnz, F, 1, s)
            ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
            if op == "spmm":
                C = torch.full((A.n_rows, F), float("nan"), dtype=torch.float32, device="cuda")
                handle.spmm(A.n_rows, A.n_cols, d_rp, d_ci, d_v, d_B, C, F, dt=dt, sched=s, workspace=ws, nnz=A.nnz)
            else:
                out = torch.full((max(A.nnz, 1),), float("nan"), dtype=torch.float32, device="cuda")
                handle.sddmm(A.n_rows, A.n_cols, d_rp, d_ci, d_X, d_B, out, F, dt=dt, sched=s, workspace=ws, nnz=A.nnz)
        except ab.AutosageError as e:
            assert e.status in (ab.ERR_UNSUPPORTED, ab.ERR_INVALID_ARG), tag          # a shape this schedule has no kernel for
            print("   %s: schedule refused (%s)" % (op, e), flush=True)
            continue
        torch.cuda.synchronize()
        if op == "spmm":
            ref = oracle.spmm(A.rowptr, A.colind, A.val, B)
            mag = oracle.spmm(A.rowptr, A.colind, np.abs(A.val), absf(B))
            got = C.cpu().numpy()
            assert np.isfinite(got).all(), tag
            assert rel_l1_rows(got, ref, mag, terms=A.degrees).max() <= tol, (op,) + tag
        elif A.nnz:
            ref = oracle.sddmm(A.rowptr, A.colind, X, B)
            mag = oracle.sddmm(A.rowptr, A.colind, absf(X), absf(B))
            got = out.cpu().numpy()[:A.nnz]
            assert np.isfinite(got).all(), tag
            assert rel_l1_segments(got, ref, A.rowptr, mag, terms=F).max() <= tol, (op,) + tag


@pytest.mark.parametrize("seed", range(16))
def test_random_softmax_and_attention(torch, ab, handle, seed):
    rng = np.random.default_rng(9500 + seed)
    n = int(rng.integers(50, 1500))
    deg = np.minimum(W.powerlaw_degrees(rng, n, 2.1, float(rng.uniform(2.0, 25.0)), None), n).astype(np.int64)
    deg[rng.integers(0, n, size=max(1, n // 8))] = 0
    deg[rng.integers(0, n)] = min(n, int(rng.integers(100, 1400)))
    A = W.csr_from_degrees(rng, deg, n)
    H = int(rng.choice([1, 2, 3, 4, 8, 16]))
    hub_t = int(rng.choice([0, 64, 128, 500]))
    group = int(rng.choice([-1, 0, 0, 1, 4, 16, 64]))
    print((seed, n, A.nnz, H, hub_t, group), flush=True)
    d_rp, d_ci = dev(A.rowptr, torch), dev(A.colind, torch)
    # row-softmax with a forced lane-group size, in its own handle
    h2 = ab.Handle(0)
    try:
        h2.set_param("softmax_group", group)
        s = (4.0 * rng.standard_normal((A.nnz, H))).astype(np.float32)
        d_s = dev(s, torch) if A.nnz else torch.empty((0, H), device="cuda")
        out = torch.full_like(d_s, float("nan"))
        ws = torch.empty(h2.workspace_bytes(ab.OP_SOFTMAX, n, A.nnz, 1, H, ab.Schedule(hub_t=hub_t)), dtype=torch.uint8, device="cuda")
        h2.csr_row_softmax(n, A.nnz, d_rp, d_s, out, H, hub_t, 0, workspace=ws)
        torch.cuda.synchronize()
        if A.nnz:
            ref = oracle.row_softmax(A.rowptr, s)
            got = out.cpu().numpy()
            for hh in range(H):
                assert rel_l1_segments(got[:, hh], ref[:, hh], A.rowptr).max() <= 1e-5, (seed, hh)
    finally:
        h2.close()
    # attention on the same pattern: a head shape the single pass has kernels for, both pipelines
    Hh, d = [(8, 64), (4, 32), (2, 32), (1, 128), (16, 8), (4, 16)][seed % 6]
    Q, K, V = W.config5_attention(n, Hh, d, seed=seed, qk_std=1.0)
    scale = float(d) ** -0.5
    ref = oracle.csr_attention(A.rowptr, A.colind, Q, K, V, scale)
    for mapping in (ab.MAP_FUSED, ab.MAP_WAVE_ROW):
        sc = ab.Schedule(mapping=mapping, waves_per_wg=4, hub_t=hub_t, hub_chunk=0)
        O = torch.full((n, Hh, d), float("nan"), dtype=torch.float32, device="cuda")
        try:
            ws = torch.empty(handle.workspace_bytes(ab.OP_ATTENTION, n, A.nnz, d, Hh, sc), dtype=torch.uint8, device="cuda")
            handle.csr_attention(n, d_rp, d_ci, dev(Q, torch), dev(K, torch), dev(V, torch), O, Hh, d, scale, sched=sc,
                                 workspace=ws, nnz=A.nnz)
        except ab.AutosageError as e:
            assert e.status == ab.ERR_UNSUPPORTED, (seed, mapping)
            continue
        torch.cuda.synchronize()
        got = O.cpu().numpy()
        assert np.isfinite(got).all(), (seed, mapping)
        assert rel_l1_rows(got.reshape(-1, d), ref.reshape(-1, d)).max() <= 2e-2, (seed, mapping)


@pytest.mark.parametrize("seed", range(12))
def test_random_shape_through_the_selector(torch, ab, seed):
    """The same random inputs with sched = NULL: whatever the probes make the selector pick must match the oracle,
    the decision must follow the rule on its own logged times, and a second call must replay it."""
    rng = np.random.default_rng(9800 + seed)
    A = random_matrix(rng)
    F = int(rng.choice(WIDTHS))
    kind = str(rng.choice(["f32", "bf16", "f16"]))
    B, absf = operands(rng, A.n_cols, F, kind)
    X, _ = operands(rng, A.n_rows, F, kind)
    print((seed, A.n_rows, A.n_cols, A.nnz, F, kind), flush=True)
    d_rp, d_ci, d_v, d_B, d_X = (dev(t, torch) for t in (A.rowptr, A.colind, A.val, B, X))
    dt = dtype_code(ab, B)
    h = ab.Handle(0)
    try:
        ws = torch.empty(h.workspace_bytes(ab.OP_SPMM, A.n_rows, A.nnz, F), dtype=torch.uint8, device="cuda")
        C = torch.full((A.n_rows, F), float("nan"), dtype=torch.float32, device="cuda")
        out = torch.full((max(A.nnz, 1),), float("nan"), dtype=torch.float32, device="cuda")
        for op in ("spmm", "sddmm"):
            for call in range(2):
                if op == "spmm":
                    h.spmm(A.n_rows, A.n_cols, d_rp, d_ci, d_v, d_B, C, F, dt=dt, workspace=ws, nnz=A.nnz)
                else:
                    h.sddmm(A.n_rows, A.n_cols, d_rp, d_ci, d_X, d_B, out, F, dt=dt, workspace=ws, nnz=A.nnz)
                d = h.last_decision()
                assert d["cache_hit"] is (call == 1), (op, call, d)
                if call == 0:
                    t = [c["t_ms"] if c["t_ms"] is not None else float("inf") for c in d["candidates"]]
                    assert d["choice_index"] == oracle.decide(t, d["t_baseline_ms"], d["alpha"]), (op, d)
            torch.cuda.synchronize()
        assert rel_l1_rows(C.cpu().numpy(), oracle.spmm(A.rowptr, A.colind, A.val, B),
                           oracle.spmm(A.rowptr, A.colind, np.abs(A.val), absf(B)), terms=A.degrees).max() <= 1e-5
        assert rel_l1_segments(out.cpu().numpy()[:A.nnz], oracle.sddmm(A.rowptr, A.colind, X, B), A.rowptr,
                               oracle.sddmm(A.rowptr, A.colind, absf(X), absf(B)), terms=F).max() <= 1e-5
    finally:
        h.close()
