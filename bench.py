#!/usr/bin/env python3
"""Benchmark of the CSR SpMM / SDDMM / CSR-attention hot path on one MI355X.

One *step* is one pass of the whole hot path over the power-law skew stressor (N = 262144,
mean 32 nonzeros per row, hub rows up to 65536): SpMM and SDDMM at F = 64 in fp32 with the
schedule the selector chose (replayed from its cache; the plan/hub partition runs inside
every call), and the multi-head CSR attention (H = 8, d = 64, bf16 operands, fp32 scores and
accumulators; SDDMM -> row-softmax -> SpMM in the pipeline form and hub threshold the selector chose).  All inputs are resident in HBM before the timed region.

Prints one JSON line: whole-step GFLOP/s (2*nnz*F per SpMM/SDDMM, 4*nnz*H*d for attention),
the roofline of the dominant kernel measured with HIP events inside the timed region, and the
CPU oracle timed on the host cores as a reported baseline.  Everything else goes to stderr.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def stage_bytes(stage, N, F, H, d, light_nnz, hub_nnz, n_chunks):
    """Algorithmic bytes of one launch of a stage (every gathered dense row counted once per nonzero)."""
    rp = 4 * (N + 1)
    HD = H * d
    table = {
        # per nonzero: colind + val (8 B) + one fp32 row of B; per row: one fp32 row of C
        "spmm_rows": light_nnz * (8 + 4 * F) + N * 4 * F + rp,
        "spmm_hub": hub_nnz * (8 + 4 * F) + 2 * n_chunks * 4 * F,
        # per nonzero: colind (4 B) + one fp32 row of Y + one fp32 result; per row: one row of X
        "sddmm_rows": light_nnz * (4 + 4 * F + 4) + N * 4 * F + rp,
        "sddmm_hub": hub_nnz * (4 + 4 * F + 4),
        # attention, bf16 operands: K or V row = 2*H*d B, scores [nnz, H] fp32
        "attn_sddmm_rows": light_nnz * (4 + 2 * HD + 4 * H) + N * 2 * HD + rp,
        "attn_sddmm_hub": hub_nnz * (4 + 2 * HD + 4 * H),
        "attn_spmm_rows": light_nnz * (4 + 4 * H + 2 * HD) + N * 4 * HD + rp,
        "attn_spmm_hub": hub_nnz * (4 + 4 * H + 2 * HD) + 2 * n_chunks * 4 * HD,
        # single pass: colind + one K row + one V row per nonzero; per row: Q row read, fp32 O row written
        "attn_fused_rows": light_nnz * (4 + 4 * HD) + N * (2 * HD + 4 * HD) + rp,
        "attn_fused_hub": hub_nnz * (4 + 4 * HD) + 2 * n_chunks * 4 * (HD + 2 * H),
        "softmax_rows": light_nnz * 8 * H + rp,
        "softmax_hub": hub_nnz * 12 * H,
        "hub_partition": 2 * rp,
    }
    return table.get(stage)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--no-sweep", action="store_true", help="skip the per-F table written to stderr")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--n", type=int, default=262144, help="rows of the power-law graph (default: the full config)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 1 GiB device-to-device copy three times (known traffic for counter scaling)")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build measures one GPU only; multi-GPU sharding is a design note, not code. "
            "Run with --gpus 1.")
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2511_17594_amd.binding as ab
    from paper_2511_17594_amd import workloads as W

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    F, H, d = 64, 8, 64
    t0 = time.time()
    A = W.config2_powerlaw(n=args.n)
    N, nnz = A.n_rows, A.nnz
    rng = W.rng_for(0, 2, 7)
    B = W.dense_operand(rng, N, F)
    X = W.dense_operand(rng, N, F)
    Y = W.dense_operand(rng, N, F)
    Q, K, V = W.config5_attention(N, H, d, seed=0)
    log("inputs: N=%d nnz=%d max_deg=%d generated in %.1f s" % (N, nnz, int(A.degrees.max()), time.time() - t0))

    def dev(a):
        a = np.ascontiguousarray(a)
        return torch.from_numpy(a.view(np.int16) if a.dtype == np.uint16 else a).cuda()

    rp, ci, va = dev(A.rowptr), dev(A.colind), dev(A.val)
    dB, dX, dY, dQ, dK, dV = (dev(t) for t in (B, X, Y, Q, K, V))
    C = torch.empty((N, F), dtype=torch.float32, device="cuda")
    out = torch.empty(nnz, dtype=torch.float32, device="cuda")
    O = torch.empty((N, H, d), dtype=torch.float32, device="cuda")
    h = ab.Handle(0)
    ws_bytes = max(h.workspace_bytes(ab.OP_SPMM, N, nnz, 256), h.workspace_bytes(ab.OP_ATTENTION, N, nnz, d, H))
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    scale = float(d) ** -0.5
    stream = torch.cuda.current_stream()

    def step():
        h.spmm(N, N, rp, ci, va, dB, C, F, workspace=ws, stream=stream)
        h.sddmm(N, N, rp, ci, dX, dY, out, F, workspace=ws, stream=stream)
        h.csr_attention(N, rp, ci, dQ, dK, dV, O, H, d, scale, workspace=ws, stream=stream)

    if args.copy_calibration:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)                  # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst

    # cold call: the selector probes and caches (reported, not part of the timed region)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    h.spmm(N, N, rp, ci, va, dB, C, F, workspace=ws, stream=stream)
    torch.cuda.synchronize()
    cold_spmm_ms = (time.perf_counter() - t0) * 1e3
    dec_spmm = h.last_decision()
    t0 = time.perf_counter()
    h.sddmm(N, N, rp, ci, dX, dY, out, F, workspace=ws, stream=stream)
    torch.cuda.synchronize()
    cold_sddmm_ms = (time.perf_counter() - t0) * 1e3
    dec_sddmm = h.last_decision()
    t0 = time.perf_counter()
    h.csr_attention(N, rp, ci, dQ, dK, dV, O, H, d, scale, workspace=ws, stream=stream)
    torch.cuda.synchronize()
    cold_attn_ms = (time.perf_counter() - t0) * 1e3
    dec_attn = h.last_decision()
    log("selector attn : %s (cold call %.2f ms)" % (dec_attn.get("choice"), cold_attn_ms))
    log("selector spmm : %s (cold call %.2f ms)" % (dec_spmm.get("choice"), cold_spmm_ms))
    log("selector sddmm: %s (cold call %.2f ms)" % (dec_sddmm.get("choice"), cold_sddmm_ms))

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    h.profile_begin()                       # per-kernel HIP events on the launch stream, inside the timed region
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    stages = h.profile_read()
    ms_per_step = elapsed * 1e3 / args.steps
    flops_step = 2.0 * nnz * F * 2 + 4.0 * nnz * H * d
    value = flops_step / (ms_per_step * 1e-3) / 1e9

    # roofline of the dominant kernel stage
    deg = A.degrees

    def split(hub_t):
        if hub_t <= 0:
            return nnz, 0, 0
        hub = deg >= hub_t
        hub_nnz = int(deg[hub].sum())
        return nnz - hub_nnz, hub_nnz, int(np.ceil(deg[hub] / hub_t).sum())

    hub_of = {"spmm": dec_spmm["choice"]["hub_t"], "sddmm": dec_sddmm["choice"]["hub_t"], "attn": dec_attn["choice"]["hub_t"], "softmax": dec_attn["choice"]["hub_t"]}
    per_stage = {}
    for name, rec in stages.items():
        key = "attn" if name.startswith("attn") else name.split("_")[0]
        light_nnz, hub_nnz, n_chunks = split(hub_of.get(key, 0))
        b = stage_bytes(name, N, F, H, d, light_nnz, hub_nnz, n_chunks)
        avg_ms = rec["total_ms"] / rec["calls"]
        per_stage[name] = {"avg_ms": avg_ms, "calls": rec["calls"], "alg_bytes": b,
                           "gbs": None if b is None else b / avg_ms / 1e6}
    dom = max(per_stage, key=lambda k: per_stage[k]["avg_ms"] * per_stage[k]["calls"])
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic.txt")     # from the committed rocprofv3 --pmc summaries
    if os.path.exists(tpath) and N == 262144:
        for ln in open(tpath):
            parts = ln.split()
            if len(parts) == 2 and parts[0] == dom and parts[1].isdigit():
                traffic = int(parts[1])
    roofline = {"bound": "hbm", "kernel": dom, "achieved": per_stage[dom]["gbs"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": per_stage[dom]["gbs"] / HBM_PEAK_GBS, "traffic": traffic,
                "avg_launch_ms": per_stage[dom]["avg_ms"], "alg_bytes_per_launch": per_stage[dom]["alg_bytes"]}
    for name in sorted(per_stage, key=lambda k: -per_stage[k]["avg_ms"]):
        s = per_stage[name]
        log("stage %-16s %8.4f ms/launch  %6.0f GB/s algorithmic (%.0f%% of 8 TB/s)"
            % (name, s["avg_ms"], s["gbs"] or 0, 100 * (s["gbs"] or 0) / HBM_PEAK_GBS))

    # per-op steady-state numbers at the step's width, and an F sweep (stderr only)
    def timed(fn, iters=10):
        fn()
        torch.cuda.synchronize()
        ts = []
        for _ in range(iters):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            fn()
            e1.record(stream)
            e1.synchronize()
            ts.append(e0.elapsed_time(e1))
        return float(np.median(ts))

    detail = {}
    widths = [F] if args.no_sweep else [8, 16, 32, 64, 128, 256]
    base = ab.baseline_schedule()
    for f in widths:
        Bf = dB if f == F else torch.randn(N, f, device="cuda")
        Xf = dX if f == F else torch.randn(N, f, device="cuda")
        Cf = torch.empty((N, f), dtype=torch.float32, device="cuda")
        bg = 4 * (N + 1) + 8 * nnz + nnz * f * 4 + N * f * 4
        t_sp = timed(lambda: h.spmm(N, N, rp, ci, va, Bf, Cf, f, workspace=ws, stream=stream))
        ch_sp = h.last_decision().get("choice")
        t_sd = timed(lambda: h.sddmm(N, N, rp, ci, Xf, Bf, out, f, workspace=ws, stream=stream))
        ch_sd = h.last_decision().get("choice")
        t_fb = timed(lambda: h.spmm(N, N, rp, ci, va, Bf, Cf, f, sched=base, workspace=ws, stream=stream), iters=3)
        t_fd = timed(lambda: h.sddmm(N, N, rp, ci, Xf, Bf, out, f, sched=base, workspace=ws, stream=stream), iters=3)
        detail["F%d" % f] = {
            "spmm_ms": t_sp, "spmm_gflops": 2.0 * nnz * f / t_sp / 1e6, "spmm_gbs": bg / t_sp / 1e6,
            "spmm_frac_hbm": bg / t_sp / 1e6 / HBM_PEAK_GBS, "spmm_fallback_ms": t_fb, "spmm_hub_t": ch_sp["hub_t"],
            "spmm_mapping": ch_sp["mapping"],
            "sddmm_ms": t_sd, "sddmm_gflops": 2.0 * nnz * f / t_sd / 1e6, "sddmm_gbs": bg / t_sd / 1e6,
            "sddmm_frac_hbm": bg / t_sd / 1e6 / HBM_PEAK_GBS, "sddmm_fallback_ms": t_fd, "sddmm_hub_t": ch_sd["hub_t"],
            "sddmm_mapping": ch_sd["mapping"],
        }
        log("F=%-3d spmm %.3f ms %.0f GFLOP/s %.0f GB/s (%.0f%%) fallback %.3f ms | sddmm %.3f ms %.0f GFLOP/s %.0f GB/s (%.0f%%) "
            "fallback %.3f ms" % (f, t_sp, 2.0 * nnz * f / t_sp / 1e6, bg / t_sp / 1e6, 100 * bg / t_sp / 1e6 / HBM_PEAK_GBS,
                                  t_fb, t_sd, 2.0 * nnz * f / t_sd / 1e6, bg / t_sd / 1e6,
                                  100 * bg / t_sd / 1e6 / HBM_PEAK_GBS, t_fd))
    # what this device's memory system sustains for plain streams (read, copy, in-place update), 1 GiB each
    n_probe = 1 << 30
    pa = torch.empty(n_probe, dtype=torch.uint8, device="cuda")
    pb = torch.empty(n_probe, dtype=torch.uint8, device="cuda")
    pa.zero_()
    pb.zero_()
    psum = torch.empty(h.stream_probe_dst_bytes(), dtype=torch.uint8, device="cuda")
    measured = {
        "read_gbs": n_probe / timed(lambda: h.stream_probe(ab.STREAM_READ, pa, psum, n_probe, stream=stream)) / 1e6,
        "copy_gbs": 2 * n_probe / timed(lambda: h.stream_probe(ab.STREAM_COPY, pa, pb, n_probe, stream=stream)) / 1e6,
        "inplace_gbs": 2 * n_probe / timed(lambda: h.stream_probe(ab.STREAM_INPLACE, None, pb, n_probe, stream=stream)) / 1e6,
        "bytes": n_probe,
    }
    del pa, pb, psum
    roofline["measured_stream"] = measured
    roofline["frac_of_measured_read"] = roofline["achieved"] / measured["read_gbs"]
    log("plain streams over 1 GiB: read %.0f GB/s, copy %.0f GB/s (read + written), in place %.0f GB/s; dominant kernel at "
        "%.0f%% of the measured read rate" % (measured["read_gbs"], measured["copy_gbs"], measured["inplace_gbs"],
                                              100 * roofline["frac_of_measured_read"]))
    t_attn = timed(lambda: h.csr_attention(N, rp, ci, dQ, dK, dV, O, H, d, scale, workspace=ws, stream=stream))
    detail["attention_ms"] = t_attn
    log("csr_attention H=%d d=%d bf16: %.3f ms/call" % (H, d, t_attn))
    if not args.no_sweep:
        try:                                  # the vendor's sparse library on the same buffers, as a reported reference only
            from paper_2511_17594_amd import vendor
            vs = vendor.Session(torch)
            Cv = torch.empty_like(C)
            t_algs = vs.spmm_times(N, N, rp, ci, va, dB, Cv, iters=3)
            t_vsd = vs.sddmm_time(N, N, rp, ci, dX, dB, torch.zeros_like(out), iters=3)
            vs.close()
            detail["hipsparse_spmm_F64_ms"] = t_algs
            detail["hipsparse_sddmm_F64_ms"] = t_vsd
            log("hipSPARSE at F=64: SpMM %s ms, SDDMM %s ms"
                % ({k: round(v, 3) for k, v in t_algs.items()}, "n/a" if t_vsd is None else "%.3f" % t_vsd))
            del Cv
        except Exception as e:                # pragma: no cover
            log("hipSPARSE unavailable: %r" % (e,))

    # the same cold calls on a fresh handle (empty cache) now that the kernels' code objects are loaded: what a
    # long-running process pays when it meets a new graph
    # (skipped with --no-sweep: the profile summaries take the last dispatches of a kernel for the timed steps)
    cold_loaded = {}
    h2 = ab.Handle(0)
    for name, fn in () if args.no_sweep else (("spmm", lambda: h2.spmm(N, N, rp, ci, va, dB, C, F, workspace=ws, stream=stream)),
                     ("sddmm", lambda: h2.sddmm(N, N, rp, ci, dX, dY, out, F, workspace=ws, stream=stream)),
                     ("attention", lambda: h2.csr_attention(N, rp, ci, dQ, dK, dV, O, H, d, scale, workspace=ws, stream=stream))):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        fn()
        torch.cuda.synchronize()
        cold_loaded[name] = (time.perf_counter() - t0) * 1e3
    h2.close()
    log("cold calls with the code objects loaded: %s" % {k: round(v, 2) for k, v in cold_loaded.items()})

    # CPU baseline: the oracle as it stands, on the host cores, same step
    cpu = None
    if not args.no_cpu:
        import oracle
        # bounded sample: the step itself on the whole graph, repeated until about 12 s of CPU work (at most 16 times)
        reps, t_sp, t_at = 0, 0.0, 0.0
        while reps < 16 and t_sp + t_at < 12.0:
            t0 = time.perf_counter()
            oracle.spmm(A.rowptr, A.colind, A.val, B)
            oracle.sddmm(A.rowptr, A.colind, X, Y)
            t1 = time.perf_counter()
            oracle.csr_attention(A.rowptr, A.colind, Q, K, V, scale)
            t2 = time.perf_counter()
            t_sp += t1 - t0
            t_at += t2 - t1
            reps += 1
        cpu = {"value": reps * flops_step / (t_sp + t_at) / 1e9, "unit": "GFLOP/s", "cores": oracle.num_threads(),
               "kind": "oracle",
               "sample": "the whole step (all %d rows, %d nonzeros), %d repetition(s): SpMM+SDDMM %.1f s, attention %.1f s"
                         % (N, nnz, reps, t_sp, t_at)}
        log("cpu oracle: %.2f GFLOP/s on %d threads (%s)" % (cpu["value"], cpu["cores"], cpu["sample"]))

    line = {
        "metric": "CSR SpMM+SDDMM (F=64, fp32) + CSR attention (H=8, d=64, bf16) step throughput, 2*nnz*F flops",
        "value": value, "unit": "GFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32 (SpMM/SDDMM), bf16 operands with f32 accumulation (attention)", "data": "synthetic",
        "config": {"workload": "power-law skew stressor N=%d nnz=%d (Pareto exponent 2.1, mean 32, clip 65536), "
                               "SpMM+SDDMM F=64 fp32 + CSR attention H=8 d=64 bf16" % (N, nnz),
                   "N": N, "nnz": nnz, "F": F, "H": H, "d": d},
        "roofline": roofline,
        "cpu_baseline": cpu,
        "selector": {"spmm": dec_spmm.get("choice"), "sddmm": dec_sddmm.get("choice"), "attention": dec_attn.get("choice"),
                     "cold_call_ms": {"spmm": cold_spmm_ms, "sddmm": cold_sddmm_ms, "attention": cold_attn_ms},
                     "cold_call_code_loaded_ms": cold_loaded},
        "stages": {k: {"avg_ms": v["avg_ms"], "gbs": v["gbs"]} for k, v in per_stage.items()},
        "detail": detail,
    }
    h.close()
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
