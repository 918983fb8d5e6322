"""GPU tests of the input-aware selector: probe -> guardrail -> cache -> replay, through the C ABI."""
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
def graph():
    return W.config2_powerlaw(n=40000, mean_deg=24.0, dmax=8192, seed=5)


def ops(torch, ab, A, F, seed=0):
    rng = np.random.default_rng(seed)
    B = rng.standard_normal((A.n_cols, F)).astype(np.float32)
    X = rng.standard_normal((A.n_rows, F)).astype(np.float32)
    return B, X


def timed(torch, fn, iters=7):
    fn()
    torch.cuda.synchronize()
    ts = []
    for _ in range(iters):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        fn()
        e1.record()
        e1.synchronize()
        ts.append(e0.elapsed_time(e1))
    return float(np.median(ts))


def test_decide_probe_guardrail_cache_replay(torch, ab, graph, tmp_path):
    A, F = graph, 64
    B, X = ops(torch, ab, A, F)
    h = ab.Handle(0)
    rp, ci, va, dB, dX = (dev(t, torch) for t in (A.rowptr, A.colind, A.val, B, X))
    C = torch.empty((A.n_rows, F), dtype=torch.float32, device="cuda")
    out = torch.empty(A.nnz, dtype=torch.float32, device="cuda")
    ws = torch.empty(h.workspace_bytes(ab.OP_SPMM, A.n_rows, A.nnz, F), dtype=torch.uint8, device="cuda")

    # cold: probes run, the decision obeys the rule on the measured times
    s1 = h.decide(ab.OP_SPMM, A.n_rows, A.n_cols, rp, ci, va, dB, None, C, F, workspace=ws)
    d1 = h.last_decision()
    assert d1["cache_hit"] is False and d1["replay_miss"] is False
    assert d1["graph_sig"] == "%016x" % oracle.graph_signature(A.rowptr, A.n_cols)
    ranked = [c for c in d1["candidates"] if not c.get("refinement")]
    refined = [c for c in d1["candidates"] if c.get("refinement")]
    assert 1 <= len(ranked) <= 4 and len(refined) <= 8 and d1["probe_rows"] >= 512
    assert d1["candidates"][:len(ranked)] == ranked                          # the refinement rounds come after the ranked k
    keys = [(c["sched"]["mapping"], c["sched"]["hub_t"], c["sched"]["xcd_remap"], c["sched"]["vec_bytes"]) for c in ranked]
    assert len(set(keys)) == len(keys)                       # the ranked candidates differ in more than the unroll depth
    scheds = [tuple(sorted(c["sched"].items())) for c in d1["candidates"]]
    assert len(set(scheds)) == len(scheds)                   # no schedule is probed twice
    t = [c["t_ms"] if c["t_ms"] is not None else float("inf") for c in d1["candidates"]]
    assert d1["choice_index"] == oracle.decide(t, d1["t_baseline_ms"], d1["alpha"])
    if d1["choice_index"] >= 0 and not d1.get("confirm", {}).get("demoted", False):
        # the rule's pick, unless the full-input run-off put the best ranked candidate back in front of a refined one
        runoff = d1.get("confirm", {}).get("runoff", {})
        kept = runoff["index"] if runoff.get("switched") else d1["choice_index"]
        assert d1["choice"] == d1["candidates"][kept]["sched"]
        assert t[kept] <= d1["alpha"] * d1["t_baseline_ms"]                     # Proposition 1 on the probe times
        if runoff:
            assert d1["candidates"][d1["choice_index"]].get("refinement") and not d1["candidates"][runoff["index"]].get("refinement")
            assert runoff["switched"] is (runoff["t_ms"] < runoff["t_refined_ms"])
    else:
        assert d1["choice"]["mapping"] == ab.MAP_PLAIN

    # warm: same key -> cache hit, same schedule, nothing is timed
    s2 = h.decide(ab.OP_SPMM, A.n_rows, A.n_cols, rp, ci, va, dB, None, C, F, workspace=ws)
    d2 = h.last_decision()
    assert d2["cache_hit"] is True and s2.as_dict() == s1.as_dict() and "candidates" not in d2
    # op and F are part of the key
    h.decide(ab.OP_SDDMM, A.n_rows, A.n_cols, rp, ci, None, dX, dB, out, F, workspace=ws)
    assert h.last_decision()["cache_hit"] is False

    # persistent cache: save, load into a fresh handle in replay-only mode -> hit without probing
    path = str(tmp_path / "sched_cache.txt")
    h.cache_save(path)
    h2 = ab.Handle(0)
    h2.set_param("replay_only", 1)
    h2.cache_load(path)
    s3 = h2.decide(ab.OP_SPMM, A.n_rows, A.n_cols, rp, ci, va, dB, None, C, F, workspace=ws)
    assert h2.last_decision()["cache_hit"] is True and s3.as_dict() == s1.as_dict()
    # replay-only miss (another F): the baseline runs and the miss is recorded
    B2 = torch.randn(A.n_cols, 32, device="cuda")
    C2 = torch.empty((A.n_rows, 32), dtype=torch.float32, device="cuda")
    s4 = h2.decide(ab.OP_SPMM, A.n_rows, A.n_cols, rp, ci, va, B2, None, C2, 32, workspace=ws)
    d4 = h2.last_decision()
    assert d4["replay_miss"] is True and s4.mapping == ab.MAP_PLAIN and s4.hub_t == 0
    h.close()
    h2.close()


@pytest.mark.parametrize("F", [16, 64, 256])
def test_auto_path_matches_oracle_and_is_not_slower_than_fallback(torch, ab, graph, F):
    A = graph
    B, X = ops(torch, ab, A, F, seed=F)
    h = ab.Handle(0)
    rp, ci, va, dB, dX = (dev(t, torch) for t in (A.rowptr, A.colind, A.val, B, X))
    C = torch.full((A.n_rows, F), float("nan"), dtype=torch.float32, device="cuda")
    out = torch.full((A.nnz,), float("nan"), dtype=torch.float32, device="cuda")
    ws = torch.empty(h.workspace_bytes(ab.OP_SPMM, A.n_rows, A.nnz, F), dtype=torch.uint8, device="cuda")
    h.spmm(A.n_rows, A.n_cols, rp, ci, va, dB, C, F, workspace=ws)            # sched = None -> selector
    d_sp = h.last_decision()
    h.sddmm(A.n_rows, A.n_cols, rp, ci, dX, dB, out, F, workspace=ws)
    d_sd = h.last_decision()
    torch.cuda.synchronize()
    ref = oracle.spmm(A.rowptr, A.colind, A.val, B)
    ref_abs = oracle.spmm(A.rowptr, A.colind, np.abs(A.val), np.abs(B))
    assert rel_l1_rows(C.cpu().numpy(), ref, ref_abs, terms=A.degrees).max() <= 1e-5
    ref = oracle.sddmm(A.rowptr, A.colind, X, B)
    ref_abs = oracle.sddmm(A.rowptr, A.colind, np.abs(X), np.abs(B))
    assert rel_l1_segments(out.cpu().numpy(), ref, A.rowptr, ref_abs, terms=F).max() <= 1e-5
    # the skewed graph must not end on the fallback, and the choice must not lose to it on the full input
    assert d_sp["choice"]["mapping"] != ab.MAP_PLAIN and d_sd["choice"]["mapping"] != ab.MAP_PLAIN
    base = ab.baseline_schedule()
    t_auto = timed(torch, lambda: h.spmm(A.n_rows, A.n_cols, rp, ci, va, dB, C, F, workspace=ws))
    t_base = timed(torch, lambda: h.spmm(A.n_rows, A.n_cols, rp, ci, va, dB, C, F, sched=base, workspace=ws))
    assert t_auto <= 1.05 * t_base, (t_auto, t_base)
    t_auto = timed(torch, lambda: h.sddmm(A.n_rows, A.n_cols, rp, ci, dX, dB, out, F, workspace=ws))
    t_base = timed(torch, lambda: h.sddmm(A.n_rows, A.n_cols, rp, ci, dX, dB, out, F, sched=base, workspace=ws))
    assert t_auto <= 1.05 * t_base, (t_auto, t_base)
    h.close()


def test_guardrail_falls_back_when_alpha_is_unreachable(torch, ab, graph):
    A, F = graph, 32
    B, _ = ops(torch, ab, A, F)
    h = ab.Handle(0)
    h.set_param("alpha", 1e-6)               # no candidate can be a million times faster than the baseline
    rp, ci, va, dB = (dev(t, torch) for t in (A.rowptr, A.colind, A.val, B))
    C = torch.empty((A.n_rows, F), dtype=torch.float32, device="cuda")
    ws = torch.empty(h.workspace_bytes(ab.OP_SPMM, A.n_rows, A.nnz, F), dtype=torch.uint8, device="cuda")
    s = h.decide(ab.OP_SPMM, A.n_rows, A.n_cols, rp, ci, va, dB, None, C, F, workspace=ws)
    d = h.last_decision()
    assert d["choice_index"] == -1 and s.mapping == ab.MAP_PLAIN and s.as_dict() == ab.baseline_schedule().as_dict()
    h.close()


def test_attention_decision(torch, ab, graph):
    A, H, d = graph, 4, 32
    Q, K, V = W.config5_attention(A.n_rows, H, d, seed=3, qk_std=1.0)
    h = ab.Handle(0)
    rp, ci, dQ, dK, dV = (dev(t, torch) for t in (A.rowptr, A.colind, Q, K, V))
    O = torch.full((A.n_rows, H, d), float("nan"), dtype=torch.float32, device="cuda")
    ws = torch.empty(h.workspace_bytes(ab.OP_ATTENTION, A.n_rows, A.nnz, d, H), dtype=torch.uint8, device="cuda")
    scale = d ** -0.5
    s1 = h.decide_attention(A.n_rows, rp, ci, dQ, dK, dV, O, H, d, scale, workspace=ws)
    d1 = h.last_decision()
    assert d1["cache_hit"] is False and d1["op"] == ab.OP_ATTENTION and d1["H"] == H and d1["F"] == d
    kinds = {c["sched"]["mapping"] for c in d1["candidates"]}
    assert ab.MAP_FUSED in kinds and ab.MAP_WAVE_ROW in kinds        # both pipelines are among the probed candidates
    t = [c["t_ms"] if c["t_ms"] is not None else float("inf") for c in d1["candidates"]]
    assert d1["choice_index"] == oracle.decide(t, d1["t_baseline_ms"], d1["alpha"])
    assert s1.mapping in (ab.MAP_FUSED, ab.MAP_WAVE_ROW) and s1.hub_t > 0     # 8192-long rows: never the unsplit baseline
    # the compute call with sched = NULL replays the decision and matches the oracle
    h.csr_attention(A.n_rows, rp, ci, dQ, dK, dV, O, H, d, scale, workspace=ws)
    assert h.last_decision()["cache_hit"] is True
    torch.cuda.synchronize()
    ref = oracle.csr_attention(A.rowptr, A.colind, Q, K, V, scale)
    err = rel_l1_rows(O.cpu().numpy().reshape(-1, d), ref.reshape(-1, d))
    assert err.max() <= 2e-2
    # another head count is another key
    Q2, K2, V2 = W.config5_attention(A.n_rows, 2, d, seed=4)
    O2 = torch.empty((A.n_rows, 2, d), dtype=torch.float32, device="cuda")
    h.decide_attention(A.n_rows, rp, ci, dev(Q2, torch), dev(K2, torch), dev(V2, torch), O2, 2, d, scale, workspace=ws)
    assert h.last_decision()["cache_hit"] is False
    h.close()


def test_replayed_decision_falls_back_when_alignment_changes(torch, ab, graph):
    A, F = graph, 64
    B, _ = ops(torch, ab, A, F, seed=9)
    h = ab.Handle(0)
    rp, ci, va = (dev(t, torch) for t in (A.rowptr, A.colind, A.val))
    C = torch.empty((A.n_rows, F), dtype=torch.float32, device="cuda")
    ws = torch.empty(h.workspace_bytes(ab.OP_SPMM, A.n_rows, A.nnz, F), dtype=torch.uint8, device="cuda")
    dB = dev(B, torch)
    h.spmm(A.n_rows, A.n_cols, rp, ci, va, dB, C, F, workspace=ws)
    assert h.last_decision()["choice"]["vec_bytes"] == 16
    # the same graph and width with a dense operand that is only 4-byte aligned: the cached 16-byte schedule
    # cannot run, the call silently uses the baseline and stays correct
    flat = torch.empty(A.n_cols * F + 1, dtype=torch.float32, device="cuda")
    Bm = flat[1:].view(A.n_cols, F)
    Bm.copy_(dB)
    C2 = torch.full_like(C, float("nan"))
    h.spmm(A.n_rows, A.n_cols, rp, ci, va, Bm, C2, F, workspace=ws)
    assert h.last_decision()["cache_hit"] is True
    torch.cuda.synchronize()
    ref = oracle.spmm(A.rowptr, A.colind, A.val, B)
    ref_abs = oracle.spmm(A.rowptr, A.colind, np.abs(A.val), np.abs(B))
    assert rel_l1_rows(C2.cpu().numpy(), ref, ref_abs, terms=A.degrees).max() <= 1e-5
    h.close()


@pytest.mark.parametrize("op_name", ["spmm", "sddmm"])
def test_baseline_light_row_bound_is_below_the_baseline_and_decides_alike(torch, ab, graph, op_name):
    """The selector's cheap baseline time (rows of >= 1024 entries left out) is a lower bound of the baseline's
    time on the same sample, so the rule applied to it (Proposition 1: t* <= alpha * t_b) can only be stricter."""
    A, F = graph, 64
    assert A.degrees.max() >= 1024
    B, X = ops(torch, ab, A, F)
    rp, ci, va, dB, dX = (dev(t, torch) for t in (A.rowptr, A.colind, A.val, B, X))
    C = torch.empty((A.n_rows, F), dtype=torch.float32, device="cuda")
    out = torch.empty(A.nnz, dtype=torch.float32, device="cuda")
    logs = {}
    for bound in (1, 0):
        h = ab.Handle(0)
        h.set_param("baseline_bound", bound)
        ws = torch.empty(h.workspace_bytes(ab.OP_SPMM, A.n_rows, A.nnz, F), dtype=torch.uint8, device="cuda")
        if op_name == "spmm":
            h.decide(ab.OP_SPMM, A.n_rows, A.n_cols, rp, ci, va, dB, None, C, F, workspace=ws)
        else:
            h.decide(ab.OP_SDDMM, A.n_rows, A.n_cols, rp, ci, None, dX, dB, out, F, workspace=ws)
        d = h.last_decision()
        h.close()
        t = [c["t_ms"] if c["t_ms"] is not None else float("inf") for c in d["candidates"]]
        assert d["choice_index"] == oracle.decide(t, d["t_baseline_ms"], d["alpha"])
        logs[bound] = d
    assert logs[1]["baseline_light_rows_only"] is True and logs[0]["baseline_light_rows_only"] is False
    # the bound leaves the longest rows out: it is the smaller time (generous margin for timer noise)
    assert logs[1]["t_baseline_ms"] <= 1.25 * logs[0]["t_baseline_ms"]
    # accepted against the bound => accepted against the whole baseline
    if logs[1]["choice_index"] >= 0:
        assert min(c["t_ms"] for c in logs[1]["candidates"]) <= logs[1]["alpha"] * 1.25 * logs[0]["t_baseline_ms"]
