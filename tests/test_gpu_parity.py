"""GPU parity: the HIP library (through its C ABI) against the CPU oracle, element by element,
on seeded inputs small enough for the oracle yet spanning several tiles, ragged tails, hub rows
and empty rows.  Tolerances (per-row L1-scaled relative error): 1e-5 for fp32 operands, 2e-2 for
bf16 operands with fp32 accumulation; integer metadata must match bit for bit.
"""
import numpy as np
import pytest

import oracle
from paper_2511_17594_amd import workloads as W
from util import BACKWARD_FLOOR, dev, dtype_code, rel_l1_rows, rel_l1_segments

pytestmark = pytest.mark.gpu

TOL_F32 = 1e-5
TOL_BF16 = 2e-2


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


@pytest.fixture(scope="module")
def skew_graph():
    """Power-law graph with hub rows (max degree 3000), empty rows and a ragged last row block."""
    rng = np.random.default_rng(17)
    n = 6007
    deg = W.powerlaw_degrees(rng, n, 2.1, 14.0, 3000)
    deg[5::97] = 0
    deg[11] = 3000
    deg[n - 1] = 777
    return W.csr_from_degrees(rng, deg, n)


def sched_of(ab, **kw):
    s = ab.Schedule()
    for k, v in kw.items():
        setattr(s, k, v)
    return s


def workspace(torch, handle, ab, op, A, F, H=1, sched=None):
    nbytes = handle.workspace_bytes(op, A.n_rows, A.nnz, F, H, sched)
    return torch.empty(nbytes, dtype=torch.uint8, device="cuda")


def run_spmm(torch, handle, ab, A, B, sched, dt=None):
    F = B.shape[1]
    dt = dtype_code(ab, B)
    d_rp, d_ci, d_v, d_B = dev(A.rowptr, torch), dev(A.colind, torch), dev(A.val, torch), dev(B, torch)
    C = torch.full((A.n_rows, F), float("nan"), dtype=torch.float32, device="cuda")
    ws = workspace(torch, handle, ab, ab.OP_SPMM, A, F, 1, sched)
    handle.spmm(A.n_rows, A.n_cols, d_rp, d_ci, d_v, d_B, C, F, dt=dt, sched=sched, workspace=ws)
    torch.cuda.synchronize()
    return C.cpu().numpy()


def run_sddmm(torch, handle, ab, A, X, Y, sched):
    F = X.shape[1]
    dt = dtype_code(ab, X)
    d_rp, d_ci = dev(A.rowptr, torch), dev(A.colind, torch)
    out = torch.full((max(A.nnz, 1),), float("nan"), dtype=torch.float32, device="cuda")
    ws = workspace(torch, handle, ab, ab.OP_SDDMM, A, F, 1, sched)
    handle.sddmm(A.n_rows, A.n_cols, d_rp, d_ci, dev(X, torch), dev(Y, torch), out, F, dt=dt, sched=sched, workspace=ws,
                 nnz=A.nnz)
    torch.cuda.synchronize()
    return out.cpu().numpy()[:A.nnz]


SCHEDULES = [
    dict(mapping=0),                                              # plain fallback
    dict(mapping=0, hub_t=256),
    dict(mapping=1),                                              # wave per row, widest vectors
    dict(mapping=1, vec_bytes=4, unroll=2),
    dict(mapping=1, hub_t=256, hub_chunk=128, unroll=8, xcd_remap=1),
    dict(mapping=1, hub_t=512, waves_per_wg=8),
    dict(mapping=2),                                              # several rows per wavefront
    dict(mapping=2, hub_t=1024, unroll=2, xcd_remap=1, waves_per_wg=2),
    dict(mapping=1, f_tile=64, hub_t=256, xcd_remap=1),           # narrow feature tiles (SDDMM: one launch per tile)
    dict(mapping=1, f_tile=32, vec_bytes=4),
]


@pytest.mark.parametrize("F", [1, 2, 8, 16, 32, 33, 64, 100, 128, 256, 602, 1024])
def test_spmm_f32_schedules(torch, handle, ab, skew_graph, F):
    A = skew_graph
    rng = np.random.default_rng(F)
    B = rng.standard_normal((A.n_cols, F)).astype(np.float32)
    ref = oracle.spmm(A.rowptr, A.colind, A.val, B)
    ref_abs = oracle.spmm(A.rowptr, A.colind, np.abs(A.val), np.abs(B))
    ran = 0
    for kw in SCHEDULES:
        s = sched_of(ab, **kw)
        try:
            C = run_spmm(torch, handle, ab, A, B, s)
        except ab.AutosageError as e:
            assert e.status == ab.ERR_UNSUPPORTED and kw.get("mapping") == 2, (kw, str(e))
            continue                                              # multi-row needs the row to fit 32 lanes
        ran += 1
        err = rel_l1_rows(C, ref, ref_abs, terms=A.degrees)
        assert np.isfinite(C).all(), kw
        assert err.max() <= TOL_F32, (kw, F, float(err.max()), int(err.argmax()))
        assert np.all(C[A.degrees == 0] == 0.0), kw               # empty rows are exactly zero
    assert ran >= 6


@pytest.mark.parametrize("F", [1, 4, 16, 32, 36, 64, 128, 200, 256, 602])
def test_sddmm_f32_schedules(torch, handle, ab, skew_graph, F):
    A = skew_graph
    rng = np.random.default_rng(1000 + F)
    X = rng.standard_normal((A.n_rows, F)).astype(np.float32)
    Y = rng.standard_normal((A.n_cols, F)).astype(np.float32)
    ref = oracle.sddmm(A.rowptr, A.colind, X, Y)
    ref_abs = oracle.sddmm(A.rowptr, A.colind, np.abs(X), np.abs(Y))
    ran = 0
    for kw in SCHEDULES:
        s = sched_of(ab, **kw)
        try:
            out = run_sddmm(torch, handle, ab, A, X, Y, s)
        except ab.AutosageError as e:
            # multi-row needs the row to fit 32 lanes; a dot product of more than 512 four-byte lanes has no kernel
            too_wide = kw.get("vec_bytes") == 4 and F > 512
            assert e.status == ab.ERR_UNSUPPORTED and (kw.get("mapping") == 2 or too_wide), (kw, str(e))
            continue
        ran += 1
        assert np.isfinite(out).all(), kw
        err = rel_l1_segments(out, ref, A.rowptr, ref_abs, terms=F)
        assert err.max() <= TOL_F32, (kw, F, float(err.max()), int(err.argmax()))
    assert ran >= 5


@pytest.mark.parametrize("kind,F", [("f32", 32), ("f32", 64), ("f32", 100), ("f32", 128), ("f32", 256), ("f32", 36),
                                     ("bf16", 64), ("bf16", 128), ("bf16", 256), ("bf16", 512), ("f16", 128)])
def test_sddmm_narrow_lane_groups(torch, handle, ab, skew_graph, kind, F):
    """SDDMM with a dense row shared by fewer lanes (each holding several 16-byte vectors): every group size that has
    kernels for the width, with and without hub split and narrow feature tiles, against the oracle; shapes without
    kernels are refused, and so is the knob on SpMM."""
    A = skew_graph
    rng = np.random.default_rng(1500 + F)
    X = rng.standard_normal((A.n_rows, F)).astype(np.float32)
    Y = rng.standard_normal((A.n_cols, F)).astype(np.float32)
    if kind == "bf16":
        X, Y = (W.float_to_bf16_bits(t).reshape(t.shape) for t in (X, Y))
        absf = lambda t: t & np.uint16(0x7FFF)
    elif kind == "f16":
        X, Y = X.astype(np.float16), Y.astype(np.float16)
        absf = np.abs
    else:
        absf = np.abs
    ref = oracle.sddmm(A.rowptr, A.colind, X, Y)
    ref_abs = oracle.sddmm(A.rowptr, A.colind, absf(X), absf(Y))
    vec = 4 if kind == "f32" else 8
    ran = 0
    for lanes in (4, 8, 16, 32):
        for kw in (dict(), dict(hub_t=256, hub_chunk=512, xcd_remap=1), dict(f_tile=256 // (16 // vec), hub_t=128, unroll=2)):
            s = sched_of(ab, mapping=1, group_lanes=lanes, **kw)
            tile = min(kw.get("f_tile", F), F)
            full = 1                                           # lanes one vector per lane would take for the tile
            while full * vec < tile:
                full *= 2
            k = full // lanes if lanes < full else 1
            legal = F % vec == 0 and (lanes >= full or (full <= 64 and (lanes, k) in
                                                      ((32, 2), (16, 2), (16, 4), (8, 2), (8, 4), (8, 8), (4, 4), (4, 8))))
            try:
                out = run_sddmm(torch, handle, ab, A, X, Y, s)
            except ab.AutosageError as e:
                assert e.status == ab.ERR_UNSUPPORTED and not legal, (kind, F, lanes, kw, str(e))
                continue
            assert legal, (kind, F, lanes, kw)
            ran += 1
            assert np.isfinite(out).all(), (lanes, kw)
            err = rel_l1_segments(out, ref, A.rowptr, ref_abs, terms=F)
            assert err.max() <= (TOL_F32 if kind == "f32" else 1e-4), (kind, F, lanes, kw, float(err.max()))
    assert ran >= (3 if F % vec == 0 else 0)
    with pytest.raises(ab.AutosageError) as e:                  # the knob belongs to SDDMM
        run_spmm(torch, handle, ab, A, Y, sched_of(ab, mapping=1, group_lanes=8))
    assert e.value.status == ab.ERR_UNSUPPORTED


@pytest.mark.parametrize("half", ["bf16", "f16"])
@pytest.mark.parametrize("F", [8, 30, 64, 128, 520])
def test_spmm_sddmm_bf16_operands(torch, handle, ab, skew_graph, F, half):
    A = skew_graph
    rng = np.random.default_rng(2000 + F)
    B32 = rng.standard_normal((A.n_cols, F)).astype(np.float32)
    X32 = rng.standard_normal((A.n_rows, F)).astype(np.float32)
    if half == "bf16":
        B = W.float_to_bf16_bits(B32).reshape(A.n_cols, F)
        X = W.float_to_bf16_bits(X32).reshape(A.n_rows, F)
        absb = lambda t: (t & np.uint16(0x7FFF))                  # |x| of a bf16 bit pattern
    else:
        B, X, absb = B32.astype(np.float16), X32.astype(np.float16), np.abs
        B[3, 0], B[4, 0], X[2, 0] = np.float16(6.0e-8), np.float16(65504.0), np.float16(-6.1e-5)   # subnormal, largest
    ref_c = oracle.spmm(A.rowptr, A.colind, A.val, B)
    ref_s = oracle.sddmm(A.rowptr, A.colind, X, B)
    abs_c = oracle.spmm(A.rowptr, A.colind, np.abs(A.val), absb(B))
    abs_s = oracle.sddmm(A.rowptr, A.colind, absb(X), absb(B))
    for kw in (dict(mapping=0), dict(mapping=1), dict(mapping=1, hub_t=256, vec_bytes=4), dict(mapping=2, hub_t=512)):
        s = sched_of(ab, **kw)
        try:
            C = run_spmm(torch, handle, ab, A, B, s)
            out = run_sddmm(torch, handle, ab, A, X, B, s)
        except ab.AutosageError as e:
            assert e.status == ab.ERR_UNSUPPORTED and kw.get("mapping") == 2, (kw, str(e))
            continue
        # the 16-bit inputs are exact in both paths, so only fp32 accumulation differs
        assert rel_l1_rows(C, ref_c, abs_c, terms=A.degrees).max() <= TOL_F32, kw
        assert rel_l1_segments(out, ref_s, A.rowptr, abs_s, terms=F).max() <= TOL_F32, kw


@pytest.mark.parametrize("H,hub_t", [(1, 0), (1, 128), (3, 0), (3, 64), (8, 0), (8, 256), (70, 128)])
def test_row_softmax(torch, handle, ab, skew_graph, H, hub_t):
    A = skew_graph
    rng = np.random.default_rng(3000 + H)
    s = (3.0 * rng.standard_normal((A.nnz, H))).astype(np.float32)
    s[A.rowptr[11]:A.rowptr[11] + 5] = 60.0                     # a few dominant scores in the hub row
    ref = oracle.row_softmax(A.rowptr, s)
    d_rp, d_s = dev(A.rowptr, torch), dev(s, torch)
    out = torch.full_like(d_s, float("nan"))
    ws = torch.empty(handle.workspace_bytes(ab.OP_SOFTMAX, A.n_rows, A.nnz, 1, H,
                                            sched_of(ab, hub_t=hub_t)), dtype=torch.uint8, device="cuda")
    handle.csr_row_softmax(A.n_rows, A.nnz, d_rp, d_s, out, H=H, hub_t=hub_t, workspace=ws)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    assert np.isfinite(got).all()
    for h in range(H):
        err = rel_l1_segments(got[:, h], ref[:, h], A.rowptr)
        assert err.max() <= TOL_F32, (H, h, float(err.max()))
    # in place
    handle.csr_row_softmax(A.n_rows, A.nnz, d_rp, d_s, d_s, H=H, hub_t=hub_t, workspace=ws)
    torch.cuda.synchronize()
    assert np.array_equal(d_s.cpu().numpy(), got)


@pytest.mark.parametrize("H,group,hub_t", [
    (1, 1, 0), (1, 4, 128), (1, 64, 0), (2, 2, 64), (2, 16, 0), (4, 1, 0), (4, 8, 256), (8, 2, 0), (8, 16, 128),
    (8, 64, 1024), (16, 4, 64), (64, 16, 0), (128, 1, 128), (256, 64, 512), (8, -1, 128), (4, 0, 0),
])
def test_row_softmax_lane_groups(torch, ab, skew_graph, H, group, hub_t):
    """Every lane-group size of the row-softmax (several rows per wavefront, rows that fit one wavefront's
    registers, rows read twice, hub chunks with vector loads) and the one-row-per-wavefront kernels
    (group < 0), forward and backward, against the oracle; then the same call on arrays that start one
    float past a 16-byte boundary, which must fall back to scalar loads and give the same result."""
    A = skew_graph
    rng = np.random.default_rng(3100 + H)
    s = (3.0 * rng.standard_normal((A.nnz, H))).astype(np.float32)
    s[A.rowptr[11] + 1000:A.rowptr[11] + 1003] = 40.0             # dominant scores in the second chunk of the hub row
    ref = oracle.row_softmax(A.rowptr, s)
    dP = rng.standard_normal((A.nnz, H)).astype(np.float32)
    P32 = ref.astype(np.float32)
    ref_b = oracle.row_softmax_backward(A.rowptr, P32, dP)
    mag_b = np.abs(P32.astype(np.float64)) * (np.abs(dP) + np.abs(oracle.row_softmax_backward(A.rowptr, P32, -np.abs(dP))
                                                                  / np.maximum(ref, 1e-300) + np.abs(dP)))
    h = ab.Handle(0)
    try:
        h.set_param("softmax_group", group)
        d_rp = dev(A.rowptr, torch)
        ws = torch.empty(h.workspace_bytes(ab.OP_SOFTMAX, A.n_rows, A.nnz, 1, H, sched_of(ab, hub_t=hub_t)),
                         dtype=torch.uint8, device="cuda")
        results = []
        for shift in (0, 1):                                       # 0: aligned; 1: one float past the alignment
            pad = torch.zeros(A.nnz * H + 4, device="cuda")
            d_s, out, d_P, d_dP, dS = (pad.clone() for _ in range(5))
            view = lambda t: t[shift:shift + A.nnz * H].view(A.nnz, H)
            view(d_s).copy_(dev(s, torch)); view(d_P).copy_(dev(P32, torch)); view(d_dP).copy_(dev(dP, torch))
            view(out).fill_(float("nan")); view(dS).fill_(float("nan"))
            h.csr_row_softmax(A.n_rows, A.nnz, d_rp, view(d_s), view(out), H=H, hub_t=hub_t, workspace=ws)
            h.csr_row_softmax_backward(A.n_rows, A.nnz, d_rp, view(d_P), view(d_dP), view(dS), H=H, hub_t=hub_t, workspace=ws)
            torch.cuda.synchronize()
            got, got_b = view(out).cpu().numpy(), view(dS).cpu().numpy()
            assert np.isfinite(got).all() and np.isfinite(got_b).all()
            assert float(out[:shift].abs().sum() + out[shift + A.nnz * H:].abs().sum()) == 0.0     # nothing outside
            assert float(dS[:shift].abs().sum() + dS[shift + A.nnz * H:].abs().sum()) == 0.0
            for hh in range(0, H, max(1, H // 8)):
                assert rel_l1_segments(got[:, hh], ref[:, hh], A.rowptr).max() <= TOL_F32, (H, group, shift, hh)
                assert rel_l1_segments(got_b[:, hh], ref_b[:, hh], A.rowptr, mag_b[:, hh], floors=(BACKWARD_FLOOR, BACKWARD_FLOOR)).max() <= TOL_F32, (H, group, shift, hh)
            # in place
            h.csr_row_softmax(A.n_rows, A.nnz, d_rp, view(d_s), view(d_s), H=H, hub_t=hub_t, workspace=ws)
            torch.cuda.synchronize()
            assert np.array_equal(view(d_s).cpu().numpy(), got)
            results.append(got)
        if H == 1 or group < 0:
            assert np.array_equal(results[0], results[1])          # scalar loads either way: same kernel, same bits
    finally:
        h.close()


@pytest.mark.parametrize("H,d,dtype,qk_std,hub_t", [
    (8, 64, "bf16", None, 256), (8, 64, "bf16", 1.0, 0), (2, 32, "bf16", 1.0, 128), (1, 128, "bf16", 1.0, 64),
    (3, 16, "bf16", 2.0, 512), (4, 16, "f32", 1.0, 256), (8, 64, "f32", 1.0, 0), (16, 8, "bf16", 1.0, 256),
    (8, 64, "f16", 1.0, 256), (2, 32, "f16", 2.0, 0),
])
def test_csr_attention(torch, handle, ab, skew_graph, H, d, dtype, qk_std, hub_t):
    A = skew_graph
    Qb, Kb, Vb = W.config5_attention(A.n_rows, H, d, seed=H * 100 + d, qk_std=qk_std)
    if dtype == "f32":
        Q, K, V = (W.bf16_bits_to_float(t).reshape(A.n_rows, H, d) * np.float32(1.001) for t in (Qb, Kb, Vb))
        Q, K, V = (np.ascontiguousarray(t, dtype=np.float32) for t in (Q, K, V))
        tol, dt = TOL_F32 * 4, ab.F32         # three fp32 stages stacked on each other
    elif dtype == "f16":
        Q, K, V = (W.bf16_bits_to_float(t).reshape(A.n_rows, H, d).astype(np.float16) for t in (Qb, Kb, Vb))
        tol, dt = TOL_BF16, ab.F16
    else:
        Q, K, V, tol, dt = Qb, Kb, Vb, TOL_BF16, ab.BF16
    scale = float(d) ** -0.5
    ref = oracle.csr_attention(A.rowptr, A.colind, Q, K, V, scale)
    d_in = [dev(t, torch) for t in (A.rowptr, A.colind, Q, K, V)]
    for mapping in (ab.MAP_WAVE_ROW, ab.MAP_FUSED):                # three stages, and the single pass
        s = sched_of(ab, mapping=mapping, hub_t=hub_t, hub_chunk=hub_t)
        O = torch.full((A.n_rows, H, d), float("nan"), dtype=torch.float32, device="cuda")
        ws = torch.empty(handle.workspace_bytes(ab.OP_ATTENTION, A.n_rows, A.nnz, d, H, s), dtype=torch.uint8, device="cuda")
        handle.csr_attention(A.n_rows, d_in[0], d_in[1], d_in[2], d_in[3], d_in[4], O, H, d, scale, in_dt=dt, sched=s,
                             workspace=ws, nnz=A.nnz)
        torch.cuda.synchronize()
        got = O.cpu().numpy()
        assert np.isfinite(got).all(), mapping
        err = rel_l1_rows(got.reshape(A.n_rows * H, d), ref.reshape(A.n_rows * H, d))
        assert err.max() <= tol, (mapping, H, d, dtype, float(err.max()), int(err.argmax()))
        assert np.all(got[A.degrees == 0] == 0.0), mapping
        # the bf16 path is in fact far inside its tolerance: inputs are exact, only fp32 rounding differs
        if dtype != "f32":
            assert err.max() <= 1e-4, mapping


@pytest.mark.parametrize("H,d,dtype,heads_tile,hub_t", [
    (8, 64, "bf16", 2, 256), (8, 64, "bf16", 4, 0), (8, 64, "bf16", 1, 128), (6, 32, "bf16", 3, 256),
    (16, 8, "bf16", 8, 256), (8, 64, "f32", 2, 256), (8, 16, "f16", 4, 64), (12, 64, "bf16", 4, 512),
])
def test_csr_attention_head_tiles(torch, handle, ab, skew_graph, H, d, dtype, heads_tile, hub_t):
    """The single pass with the heads walked in tiles (grid rows of the launch): same oracle, and the same bits as the
    untiled single pass whenever a tile has the lane shape of the whole (a head's lanes never see another head)."""
    A = skew_graph
    Qb, Kb, Vb = W.config5_attention(A.n_rows, H, d, seed=H * 10 + d, qk_std=1.0)
    if dtype == "f32":
        Q, K, V = (np.ascontiguousarray(W.bf16_bits_to_float(t).reshape(A.n_rows, H, d) * np.float32(1.001), dtype=np.float32)
                   for t in (Qb, Kb, Vb))
        tol, dt = TOL_F32 * 4, ab.F32
    elif dtype == "f16":
        Q, K, V = (W.bf16_bits_to_float(t).reshape(A.n_rows, H, d).astype(np.float16) for t in (Qb, Kb, Vb))
        tol, dt = 1e-4, ab.F16
    else:
        Q, K, V, tol, dt = Qb, Kb, Vb, 1e-4, ab.BF16
    scale = float(d) ** -0.5
    ref = oracle.csr_attention(A.rowptr, A.colind, Q, K, V, scale)
    d_in = [dev(t, torch) for t in (A.rowptr, A.colind, Q, K, V)]
    s = sched_of(ab, mapping=ab.MAP_FUSED, hub_t=hub_t, hub_chunk=hub_t, f_tile=heads_tile * d)
    O = torch.full((A.n_rows, H, d), float("nan"), dtype=torch.float32, device="cuda")
    ws = torch.empty(handle.workspace_bytes(ab.OP_ATTENTION, A.n_rows, A.nnz, d, H, s), dtype=torch.uint8, device="cuda")
    handle.csr_attention(A.n_rows, *d_in, O, H, d, scale, in_dt=dt, sched=s, workspace=ws, nnz=A.nnz)
    torch.cuda.synchronize()
    got = O.cpu().numpy()
    assert np.isfinite(got).all()
    err = rel_l1_rows(got.reshape(A.n_rows * H, d), ref.reshape(A.n_rows * H, d))
    assert err.max() <= tol, (H, d, dtype, heads_tile, float(err.max()), int(err.argmax()))
    assert np.all(got[A.degrees == 0] == 0.0)
    # a tile size that does not divide the head count, or is no multiple of d, is refused
    for bad in (d * H + d // 2, (H - 1) * d if H > 2 and H % (H - 1) else d // 2):
        with pytest.raises(ab.AutosageError) as e:
            handle.csr_attention(A.n_rows, *d_in, O, H, d, scale, in_dt=dt, nnz=A.nnz, workspace=ws,
                                 sched=sched_of(ab, mapping=ab.MAP_FUSED, hub_t=hub_t, hub_chunk=hub_t, f_tile=bad))
        assert e.value.status == ab.ERR_UNSUPPORTED


def test_csr_attention_unsupported_shapes(torch, handle, ab, skew_graph):
    A = skew_graph
    rp, ci = dev(A.rowptr, torch), dev(A.colind, torch)
    ws = torch.empty(1 << 24, dtype=torch.uint8, device="cuda")

    def call(H, d, mapping):
        Q = torch.zeros((A.n_rows, H, d), dtype=torch.bfloat16, device="cuda")
        O = torch.zeros((A.n_rows, H, d), dtype=torch.float32, device="cuda")
        handle.csr_attention(A.n_rows, rp, ci, Q, Q, Q, O, H, d, 1.0, sched=sched_of(ab, mapping=mapping), workspace=ws,
                             nnz=A.nnz)

    with pytest.raises(ab.AutosageError) as ei:
        call(4, 12, ab.MAP_WAVE_ROW)              # 24-byte head rows cannot take 16-byte lane loads
    assert ei.value.status == ab.ERR_UNSUPPORTED
    with pytest.raises(ab.AutosageError) as ei:
        call(32, 64, ab.MAP_FUSED)                # 32 heads x 8 lanes = four register passes: single pass not built
    assert ei.value.status == ab.ERR_UNSUPPORTED
    with pytest.raises(ab.AutosageError) as ei:
        call(8, 64, ab.MAP_MULTI_ROW)             # not an attention pipeline
    assert ei.value.status == ab.ERR_UNSUPPORTED
    torch.cuda.synchronize()


@pytest.mark.parametrize("hub_t,chunk", [(64, 64), (256, 100), (1, 7), (5000, 64)])
def test_hub_partition_and_features_bit_exact(torch, handle, ab, skew_graph, hub_t, chunk):
    A = skew_graph
    n = A.n_rows
    d_rp = dev(A.rowptr, torch)
    hub_rows = torch.full((n,), -1, dtype=torch.int32, device="cuda")
    chunk_ptr = torch.full((n + 1,), -1, dtype=torch.int32, device="cuda")
    light_rows = torch.full((n,), -1, dtype=torch.int32, device="cuda")
    ws = torch.empty(1 << 20, dtype=torch.uint8, device="cuda")
    nh, nl = handle.hub_partition(n, d_rp, hub_t, chunk, hub_rows, chunk_ptr, light_rows, ws)
    o_hub, o_ptr, o_light = oracle.hub_partition(A.rowptr, hub_t, chunk)
    assert nh == o_hub.shape[0] and nl == o_light.shape[0]
    assert np.array_equal(hub_rows.cpu().numpy()[:nh], o_hub)
    assert np.array_equal(chunk_ptr.cpu().numpy()[:nh + 1], o_ptr)
    assert np.array_equal(light_rows.cpu().numpy()[:nl], o_light)
    hist, mx, nnz, sig = handle.graph_features(n, A.n_cols, d_rp)
    o_hist, o_mx = oracle.degree_histogram(A.rowptr)
    assert hist == o_hist.tolist() and mx == o_mx and nnz == A.nnz
    assert sig == oracle.graph_signature(A.rowptr, A.n_cols)


def test_edge_cases(torch, handle, ab):
    F = 20
    rng = np.random.default_rng(5)
    # all rows empty -> zeros; SDDMM and softmax write nothing
    A = W.CSR(50, 40, np.zeros(51, np.int32), np.zeros(0, np.int32), np.zeros(0, np.float32))
    B = rng.standard_normal((40, F)).astype(np.float32)
    for kw in (dict(mapping=0), dict(mapping=1, hub_t=64), dict(mapping=2)):
        C = run_spmm(torch, handle, ab, A, B, sched_of(ab, **kw))
        assert np.all(C == 0.0)
    # zero rows: nothing to do
    handle.spmm(0, 40, dev(np.zeros(1, np.int32), torch), None, None, None,
                torch.empty((0, F), device="cuda"), F, sched=sched_of(ab, mapping=1), nnz=0)
    # one row holding every column once, rectangular, padded leading dimensions, hub path with a single chunk
    n_cols = 300
    A = W.CSR(1, n_cols, np.array([0, n_cols], np.int32), np.arange(n_cols, dtype=np.int32),
              rng.uniform(-1, 1, n_cols).astype(np.float32))
    Bp = rng.standard_normal((n_cols, F + 12)).astype(np.float32)
    ref = oracle.spmm(A.rowptr, A.colind, A.val, np.ascontiguousarray(Bp[:, :F]))
    for kw in (dict(mapping=0), dict(mapping=1), dict(mapping=1, hub_t=64, hub_chunk=64), dict(mapping=2)):
        s = sched_of(ab, **kw)
        Cp = torch.full((1, F + 4), 7.0, dtype=torch.float32, device="cuda")
        ws = workspace(torch, handle, ab, ab.OP_SPMM, A, F, 1, s)
        handle.spmm(1, n_cols, dev(A.rowptr, torch), dev(A.colind, torch), dev(A.val, torch), dev(Bp, torch), Cp, F,
                    sched=s, workspace=ws, ldb=F + 12, ldc=F + 4)
        torch.cuda.synchronize()
        got = Cp.cpu().numpy()
        assert rel_l1_rows(got[:, :F], ref).max() <= TOL_F32, kw
        assert np.all(got[:, F:] == 7.0), kw                         # padding columns untouched
    # misaligned dense base pointer: 16-byte loads are refused, the automatic width falls back and stays correct
    A2, B2, X2, Y2 = W.config1_tiny(n=512, mean_deg=9.0, F=32)
    ref = oracle.spmm(A2.rowptr, A2.colind, A2.val, B2)
    flat = torch.empty(512 * 32 + 1, dtype=torch.float32, device="cuda")
    Bm = flat[1:].view(512, 32)
    Bm.copy_(torch.from_numpy(B2))
    C = torch.empty((512, 32), dtype=torch.float32, device="cuda")
    args = (512, 512, dev(A2.rowptr, torch), dev(A2.colind, torch), dev(A2.val, torch), Bm, C, 32)
    with pytest.raises(ab.AutosageError) as ei:
        handle.spmm(*args, sched=sched_of(ab, mapping=1, vec_bytes=16))
    assert ei.value.status == ab.ERR_UNSUPPORTED
    handle.spmm(*args, sched=sched_of(ab, mapping=1))
    torch.cuda.synchronize()
    assert rel_l1_rows(C.cpu().numpy(), ref).max() <= TOL_F32
    # invalid arguments are rejected before any launch
    with pytest.raises(ab.AutosageError) as ei:
        handle.spmm(*args[:7], 0, sched=sched_of(ab, mapping=1))
    assert ei.value.status == ab.ERR_INVALID_ARG
    with pytest.raises(ab.AutosageError) as ei:
        handle.spmm(*args, sched=sched_of(ab, mapping=1, hub_t=512), workspace=None)
    assert ei.value.status == ab.ERR_WORKSPACE_TOO_SMALL
    with pytest.raises(ab.AutosageError) as ei:
        handle.spmm(*args, sched=sched_of(ab, mapping=7))
    assert ei.value.status == ab.ERR_INVALID_ARG
    # CSR validation
    assert handle.validate_csr(512, 512, A2.nnz, dev(A2.rowptr, torch), dev(A2.colind, torch))
    bad = A2.colind.copy()
    bad[7] = 512
    assert not handle.validate_csr(512, 512, A2.nnz, dev(A2.rowptr, torch), dev(bad, torch))
    badp = A2.rowptr.copy()
    badp[100] = badp[101] + 1
    assert not handle.validate_csr(512, 512, A2.nnz, dev(badp, torch), dev(A2.colind, torch))


def test_fixed_schedule_is_bit_reproducible(torch, handle, ab, skew_graph):
    A = skew_graph
    rng = np.random.default_rng(77)
    B = rng.standard_normal((A.n_cols, 64)).astype(np.float32)
    s = sched_of(ab, mapping=1, hub_t=256, hub_chunk=256)
    C1 = run_spmm(torch, handle, ab, A, B, s)
    C2 = run_spmm(torch, handle, ab, A, B, s)
    assert np.array_equal(C1, C2)


@pytest.mark.parametrize("fmt", ["bf16", "f16"])
def test_16_bit_operands_are_decoded_exactly(torch, handle, ab, fmt):
    """Identity pattern with unit values: C must equal the 16-bit operand's values bit for bit (the tables hold
    what the two formats define, subnormals and the largest finite value included)."""
    import os
    golden = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "%s_values.txt" % fmt)
    rows = [l.split() for l in open(golden) if l.strip() and not l.startswith("#")]
    bits = np.array([int(b, 16) for b, _ in rows], dtype=np.uint16)
    vals = np.array([float(v) for _, v in rows], dtype=np.float32)
    n = bits.size
    A = W.CSR(n, n, np.arange(n + 1, dtype=np.int32), np.arange(n, dtype=np.int32), np.ones(n, np.float32))
    for F, kw in ((8, dict(mapping=1, vec_bytes=16)), (8, dict(mapping=2)), (4, dict(mapping=1, vec_bytes=8)),
                  (6, dict(mapping=1, vec_bytes=4)), (3, dict(mapping=1, vec_bytes=2)), (5, dict(mapping=0))):
        B = np.repeat(bits[:, None], F, axis=1)
        B = B if fmt == "bf16" else B.view(np.float16)
        C = run_spmm(torch, handle, ab, A, np.ascontiguousarray(B), sched_of(ab, **kw))
        assert np.array_equal(C, np.repeat(vals[:, None], F, axis=1)), (fmt, F, kw)
