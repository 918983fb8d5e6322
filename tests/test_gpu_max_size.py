"""The library's size limit: a matrix with exactly AUTOSAGE_MAX_NNZ = 2^31 - 2^20 stored entries whose last
row is long and ends at the last position.  Positions are int32 inside the kernels; this input puts every
`position + step` of the row, hub and softmax kernels next to the top of that range.  Sampled rows (first,
empty, hub, random, last) are compared with the oracle one by one; one entry past the limit is an error."""
import numpy as np
import pytest

import oracle
from paper_2511_17594_amd import workloads as W
from util import dev, rel_l1_rows, rel_l1_segments

pytestmark = pytest.mark.gpu

MAX_NNZ = (1 << 31) - (1 << 20)
F = 8


@pytest.fixture(scope="module")
def torch():
    import torch
    return torch


@pytest.fixture(scope="module")
def ab():
    from paper_2511_17594_amd import binding
    return binding


@pytest.fixture(scope="module")
def big(torch):
    print("generating %d nonzeros on the host" % MAX_NNZ, flush=True)
    A = W.largest_input(MAX_NNZ)
    assert A.nnz == MAX_NNZ and A.rowptr.dtype == np.int32 and int(A.rowptr[-1]) == MAX_NNZ
    assert A.colind.size == MAX_NNZ and A.val.size == MAX_NNZ
    assert int(A.colind.min()) >= 0 and int(A.colind.max()) < A.n_cols
    d = (dev(A.rowptr, torch), dev(A.colind, torch), dev(A.val, torch))
    rng = np.random.default_rng(11)
    rows = np.unique(np.concatenate([np.arange(9), rng.choice(A.n_rows, 40, replace=False),
                                     np.arange(A.n_rows - 3, A.n_rows)]))
    return A, d, rows, W.row_slice(A, rows)


def schedules(ab):
    return [
        ("wave-row, hub 4096, longest chunk", ab.Schedule(mapping=ab.MAP_WAVE_ROW, hub_t=4096, hub_chunk=1 << 20)),
        ("wave-row, hub 1024 = chunk, 16 waves", ab.Schedule(mapping=ab.MAP_WAVE_ROW, hub_t=1024, waves_per_wg=16)),
        ("multi-row, hub 2048, chunk 64", ab.Schedule(mapping=ab.MAP_MULTI_ROW, hub_t=2048, hub_chunk=64)),
    ]


def test_spmm_at_the_size_limit(torch, ab, big):
    A, d, rows, As = big
    h = ab.Handle(0)
    rng = np.random.default_rng(1)
    B = rng.standard_normal((A.n_cols, F), dtype=np.float32)
    dB = dev(B, torch)
    ref = oracle.spmm(As.rowptr, As.colind, As.val, B)
    ref_abs = oracle.spmm(As.rowptr, As.colind, np.abs(As.val), np.abs(B))
    sel = torch.from_numpy(rows).cuda()
    for name, s in schedules(ab) + [("selector", None)]:
        print("spmm:", name, flush=True)
        C = torch.full((A.n_rows, F), float("nan"), dtype=torch.float32, device="cuda")
        ws = torch.empty(h.workspace_bytes(ab.OP_SPMM, A.n_rows, A.nnz, F, 1, s), dtype=torch.uint8, device="cuda")
        h.spmm(A.n_rows, A.n_cols, *d, dB, C, F, sched=s, workspace=ws)
        torch.cuda.synchronize()
        assert bool(torch.isfinite(C).all()), name
        err = rel_l1_rows(C[sel].cpu().numpy(), ref, ref_abs, terms=As.degrees)
        assert err.max() <= 1e-5, (name, float(err.max()), int(rows[err.argmax()]))
        assert float(C[5].abs().max()) == 0.0                      # the empty row
    with pytest.raises(ab.AutosageError) as ei:                      # one entry more is refused before any launch
        h.spmm(A.n_rows, A.n_cols, *d, dB, C, F, sched=schedules(ab)[0][1], workspace=ws, nnz=MAX_NNZ + 1)
    assert ei.value.status == ab.ERR_INVALID_ARG
    h.close()


def test_sddmm_and_softmax_at_the_size_limit(torch, ab, big):
    A, d, rows, As = big
    h = ab.Handle(0)
    rng = np.random.default_rng(2)
    X = rng.standard_normal((A.n_rows, F), dtype=np.float32)
    Y = rng.standard_normal((A.n_cols, F), dtype=np.float32)
    dX, dY = dev(X, torch), dev(Y, torch)
    Xs = np.ascontiguousarray(X[rows])
    ref = oracle.sddmm(As.rowptr, As.colind, Xs, Y)
    ref_abs = oracle.sddmm(As.rowptr, As.colind, np.abs(Xs), np.abs(Y))
    rp = A.rowptr.astype(np.int64)
    idx = torch.from_numpy(np.concatenate([np.arange(rp[r], rp[r + 1]) for r in rows])).cuda()
    out = torch.empty(A.nnz, dtype=torch.float32, device="cuda")
    for name, s in schedules(ab):
        print("sddmm:", name, flush=True)
        out.fill_(float("nan"))
        ws = torch.empty(h.workspace_bytes(ab.OP_SDDMM, A.n_rows, A.nnz, F, 1, s), dtype=torch.uint8, device="cuda")
        h.sddmm(A.n_rows, A.n_cols, d[0], d[1], dX, dY, out, F, sched=s, workspace=ws)
        torch.cuda.synchronize()
        assert bool(torch.isfinite(out).all()), name
        err = rel_l1_segments(out[idx].cpu().numpy(), ref, As.rowptr, ref_abs, terms=F)
        assert err.max() <= 1e-5, (name, float(err.max()), int(rows[err.argmax()]))

    # row-softmax of the stored values (scores = val), written into `out`
    ref_p = oracle.row_softmax(As.rowptr, As.val)
    for hub_t, chunk in ((0, 0), (1024, 0), (4096, 1 << 20)):
        print("softmax: hub_t %d chunk %d" % (hub_t, chunk), flush=True)
        out.fill_(float("nan"))
        ws = torch.empty(h.workspace_bytes(ab.OP_SOFTMAX, A.n_rows, A.nnz, 1, 1, ab.Schedule(hub_t=hub_t, hub_chunk=chunk)),
                         dtype=torch.uint8, device="cuda")
        h.csr_row_softmax(A.n_rows, A.nnz, d[0], d[2], out, 1, hub_t, chunk, workspace=ws)
        torch.cuda.synchronize()
        assert bool(torch.isfinite(out).all())
        got = out[idx].cpu().numpy()
        err = rel_l1_segments(got, ref_p, As.rowptr)
        assert err.max() <= 1e-5, (hub_t, float(err.max()), int(rows[err.argmax()]))
    h.close()
