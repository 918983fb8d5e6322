"""Feature-width sweep of SpMM / SDDMM on one of the synthetic workloads, printed as a Markdown table.

    python -m paper_2511_17594_amd.sweep --workload config2 [--widths 8,16,32,64,128,256] [--vendor]

For every width: the selector's choice (cold call, then steady state from its cache), time (median of
`--iters` HIP-event timings), GFLOP/s = 2*nnz*F/t, algorithmic GB/s (every gathered dense row counted
once per nonzero; `--dtype bf16` / `f16` halve the bytes of a gathered row) and its fraction of the
8 TB/s HBM peak, the rate in compulsory bytes (every array touched exactly once), and the guardrail's
fallback kernel on the same input.  `--vendor` adds hipSPARSE on the same buffers (its fastest CSR SpMM
algorithm and its SDDMM, called directly through `vendor.py`).
`--attention` prints the CSR-attention table instead (H = 8, d = 64, 16-bit operands from `--dtype`, default
bf16): the selector's choice, the single pass and the three-stage pipeline at fixed split thresholds, and
the backward call; bytes are the algorithmic ones (a K and a V row per nonzero, plus 16 bytes per score and
head for the three stages; backward: K, V, Q rows and an fp32 dO row per nonzero, 32 bytes per score and head).  `--softmax` prints the row-softmax table instead (forward and backward, H = 1 and 8, over split
thresholds): 8 bytes per score forward (read + write), 12 backward (P, dP read, dS written).
Workloads: config1..4 (the benchmark configurations), er (Erdos-Renyi N = 200000, p = 2e-5, the shape of
the paper's extreme-sparsity stressor) and hubsplit_5k / hubsplit_12k (N = 20000, a few rows of degree
5000 / 12000, the rest 64 / 32: the shape of the paper's split-versus-baseline table; the number of hub
rows is not given there, 32 is used).
`--transpose` times the CSR transpose of the pattern (pattern only, permutation kept).
`--column-slices S` measures what processing the pattern in S column ranges would cost, with the library's own
kernels: the pattern is cut on the host into S patterns that hold the nonzeros of one column range each (so the
slice of the gathered operand a launch touches is 1/S of it and can stay in the Infinity Cache), every slice is
decided by the selector on its own, and the S launches are timed back to back beside the unsliced call.  For SDDMM
that is the whole sliced operation (every nonzero is written once either way); for SpMM and the single-pass
attention it leaves out the merge of the S partial results per row, so the figure is a lower bound of the sliced
form's time.
"""
from __future__ import annotations

import argparse
import sys
import time

import numpy as np

HBM_PEAK_GBS = 8000.0

DEFAULT_WIDTHS = {
    "config1": [32], "config2": [8, 16, 32, 64, 128, 256], "config3": [32, 64, 128, 256, 602],
    "config4": [16, 32, 100, 128], "er": [64, 128, 256], "hubsplit_5k": [128], "hubsplit_12k": [128],
}


def make_workload(name):
    from . import workloads as W
    if name == "config1":
        return W.config1_tiny()[0]
    if name == "config2":
        return W.config2_powerlaw()
    if name == "config3":
        return W.config3_community()
    if name == "config4":
        return W.config4_large()
    if name == "er":
        return W.er_graph(200000, 2e-5, seed=0, config_id=7)
    if name == "hubsplit_5k":
        return W.hub_split_graph(20000, 32, 5000, 64)
    if name == "hubsplit_12k":
        return W.hub_split_graph(20000, 32, 12000, 32)
    raise SystemExit("unknown workload %r" % name)


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--workload", default="config2", choices=sorted(DEFAULT_WIDTHS))
    ap.add_argument("--widths", default=None)
    ap.add_argument("--iters", type=int, default=10)
    ap.add_argument("--vendor", action="store_true")
    ap.add_argument("--no-sddmm", action="store_true")
    ap.add_argument("--dtype", default="f32", choices=["f32", "bf16", "f16"], help="element type of the dense input operands")
    ap.add_argument("--softmax", action="store_true", help="row-softmax forward / backward table instead of SpMM / SDDMM")
    ap.add_argument("--attention", action="store_true", help="CSR attention (forward and backward) table instead of SpMM / SDDMM")
    ap.add_argument("--schedule", action="append", default=[],
                    help="run this explicit schedule instead of the selector's choice, e.g. mapping=1,hub_t=512,hub_chunk=2048,"
                         "group_lanes=8 (fields of autosage_schedule_t; may be given several times: one table row each)")
    ap.add_argument("--no-fallback", action="store_true", help="do not time the guardrail's fallback kernel")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="first run a plain 1 GiB device-to-device copy three times (known traffic for profiler counter scaling)")
    ap.add_argument("--transpose", action="store_true", help="time the CSR transpose of the pattern (sort passes, index kernels)")
    ap.add_argument("--column-slices", type=int, default=0,
                    help="time the pattern cut into this many column ranges, one launch per range, beside the unsliced call")
    args = ap.parse_args(argv)

    import torch
    from . import binding as ab

    widths = [int(x) for x in args.widths.split(",")] if args.widths else DEFAULT_WIDTHS[args.workload]
    t0 = time.time()
    A = make_workload(args.workload)
    N, M, nnz = A.n_rows, A.n_cols, A.nnz
    deg = A.degrees
    print("workload %s: rows %d, nnz %d, degree mean %.1f / median %d / max %d (generated in %.1f s)"
          % (args.workload, N, nnz, deg.mean(), int(np.median(deg)), int(deg.max()), time.time() - t0), file=sys.stderr)
    rp = torch.from_numpy(A.rowptr).cuda()
    ci = torch.from_numpy(A.colind).cuda()
    va = torch.from_numpy(A.val).cuda()
    h = ab.Handle(0)
    stream = torch.cuda.current_stream()
    base = ab.baseline_schedule()
    explicit = [ab.Schedule(**{k: int(v) for k, v in (kv.split("=") for kv in text.split(","))}) for text in args.schedule]
    if args.copy_calibration:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)                  # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst

    def timed(fn, iters):
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

    def short(c):
        m = {0: "plain", 1: "wave-row", 2: "multi-row"}[c["mapping"]]
        return "%s v%d u%d hub %d%s%s%s%s" % (m, c["vec_bytes"], c["unroll"], c["hub_t"],
                                              "/%d" % c["hub_chunk"] if c["hub_t"] else "",
                                              " tile %d" % c["f_tile"] if c["f_tile"] else "",
                                              " lanes %d" % c["group_lanes"] if c.get("group_lanes") else "",
                                              " xcd" if c["xcd_remap"] else "")

    def column_slices(S):
        """The S patterns that hold the nonzeros of one column range each, as device CSR arrays."""
        rows = np.repeat(np.arange(N, dtype=np.int32), deg)
        out = []
        for k in range(S):
            lo, hi = (M * k) // S, (M * (k + 1)) // S
            keep = (A.colind >= lo) & (A.colind < hi)
            rp_k = np.zeros(N + 1, dtype=np.int64)
            np.cumsum(np.bincount(rows[keep], minlength=N), out=rp_k[1:])
            out.append((int(keep.sum()), torch.from_numpy(rp_k.astype(np.int32)).cuda(), torch.from_numpy(A.colind[keep]).cuda(),
                        torch.from_numpy(A.val[keep]).cuda()))
        return out

    if args.transpose:
        t_rp = torch.empty(M + 1, dtype=torch.int32, device="cuda")
        t_ci = torch.empty(max(nnz, 1), dtype=torch.int32, device="cuda")
        perm = torch.empty(max(nnz, 1), dtype=torch.int32, device="cuda")
        wst = torch.empty(h.csr_transpose_workspace_bytes(N, M, nnz), dtype=torch.uint8, device="cuda")
        t = timed(lambda: h.csr_transpose(N, M, nnz, rp, ci, None, t_rp, t_ci, None, perm, wst, stream=stream), args.iters)
        passes = (max(1, int(M - 1).bit_length()) + 7) // 8
        print("| workload | nnz | columns | 8-bit passes | ms | 10^9 keys/s | workspace MB |")
        print("|---|---|---|---|---|---|---|")
        print("| %s | %d | %d | %d | %.3f | %.2f | %.0f |" % (args.workload, nnz, M, passes, t, nnz / t / 1e6, wst.numel() / 1e6), flush=True)
        h.close()
        return

    if args.column_slices > 1:
        S = args.column_slices
        parts = column_slices(S)
        print("| op | F | column ranges | gathered operand per range MB | unsliced ms | sliced ms | sliced / unsliced | what the sliced figure leaves out |")
        print("|---|---|---|---|---|---|---|---|")
        if args.attention:
            H, d = 8, 64
            half = torch.float16 if args.dtype == "f16" else torch.bfloat16
            in_dt = ab.F16 if args.dtype == "f16" else ab.BF16
            g = torch.Generator(device="cuda").manual_seed(5)
            Q, K, V = (torch.randn((N, H, d), device="cuda", generator=g).mul_(d ** -0.25).to(half) for _ in range(3))
            O = torch.empty((N, H, d), device="cuda")
            ws = torch.empty(h.workspace_bytes(ab.OP_ATTENTION, N, nnz, d, H), dtype=torch.uint8, device="cuda")
            call = lambda n_k, rp_k, ci_k: h.csr_attention(N, rp_k, ci_k, Q, K, V, O, H, d, d ** -0.5, in_dt=in_dt, workspace=ws,
                                                           stream=stream, nnz=n_k)
            t_full = timed(lambda: call(nnz, rp, ci), args.iters)
            t_cut = timed(lambda: [call(n_k, rp_k, ci_k) for n_k, rp_k, ci_k, _ in parts], args.iters)
            print("| attention (H = %d, d = %d, %s) | %d | %d | %.0f | %.3f | %.3f | %.2f | merging S running-softmax states per row |"
                  % (H, d, "f16" if args.dtype == "f16" else "bf16", H * d, S, 2.0 * N * H * d * 2 / S / 1e6, t_full, t_cut,
                     t_cut / t_full), flush=True)
            h.close()
            return
        dt = {"f32": ab.F32, "bf16": ab.BF16, "f16": ab.F16}[args.dtype]
        esz = 4 if args.dtype == "f32" else 2
        for F in widths:
            g = torch.Generator(device="cuda").manual_seed(F)
            B = torch.randn((M, F), device="cuda", generator=g)
            X = torch.randn((N, F), device="cuda", generator=g)
            if args.dtype != "f32":
                half = torch.bfloat16 if args.dtype == "bf16" else torch.float16
                B, X = B.to(half), X.to(half)
            C = torch.empty((N, F), device="cuda")
            out = torch.empty(max(nnz, 1), device="cuda")
            ws = torch.empty(h.workspace_bytes(ab.OP_SPMM, N, nnz, F), dtype=torch.uint8, device="cuda")
            spmm = lambda n_k, rp_k, ci_k, va_k: h.spmm(N, M, rp_k, ci_k, va_k, B, C, F, dt=dt, workspace=ws, stream=stream)
            sddmm = lambda n_k, rp_k, ci_k, va_k: h.sddmm(N, M, rp_k, ci_k, X, B, out, F, dt=dt, workspace=ws, stream=stream, nnz=n_k)
            for name, fn, left_out in (("SpMM", spmm, "adding S partial rows of C"), ("SDDMM", sddmm, "nothing")):
                if name == "SDDMM" and args.no_sddmm:
                    continue
                t_full = timed(lambda: fn(nnz, rp, ci, va), args.iters)
                t_cut = timed(lambda: [fn(*part) for part in parts], args.iters)
                print("| %s | %d | %d | %.0f | %.3f | %.3f | %.2f | %s |" % (name, F, S, M * F * esz / S / 1e6, t_full, t_cut,
                                                                       t_cut / t_full, left_out), flush=True)
            del B, X, C, out, ws
        h.close()
        return

    if args.attention:
        if N != M:
            raise SystemExit("attention needs a square pattern")
        H, d = 8, 64
        half = {"f32": torch.bfloat16, "bf16": torch.bfloat16, "f16": torch.float16}[args.dtype]
        in_dt = ab.F16 if args.dtype == "f16" else ab.BF16
        g = torch.Generator(device="cuda").manual_seed(5)
        Q, K, V = (torch.randn((N, H, d), device="cuda", generator=g).mul_(d ** -0.25).to(half) for _ in range(3))
        O = torch.empty((N, H, d), device="cuda")
        scale = d ** -0.5
        HD, e = H * d, 2
        b_fused = 4 * (N + 1) + 4 * nnz + 2.0 * nnz * HD * e + N * HD * e + N * HD * 4
        b_three = b_fused + 16.0 * nnz * H + 8 * (N + 1) + 8 * nnz
        ws = torch.empty(h.workspace_bytes(ab.OP_ATTENTION, N, nnz, d, H), dtype=torch.uint8, device="cuda")
        print("| pipeline | split threshold | ms | GFLOP/s (4·nnz·H·d) | algorithmic GB | GB/s | of 8 TB/s |")
        print("|---|---|---|---|---|---|---|")

        def row(label, hub_t, t, nbytes):
            print("| %s | %s | %.3f | %.0f | %.2f | %.0f | %.0f %% |" % (label, hub_t, t, 4.0 * nnz * HD / t / 1e6, nbytes / 1e9,
                                                                nbytes / t / 1e6, 100 * nbytes / t / 1e6 / HBM_PEAK_GBS), flush=True)

        torch.cuda.synchronize()
        t0 = time.perf_counter()
        h.csr_attention(N, rp, ci, Q, K, V, O, H, d, scale, in_dt=in_dt, workspace=ws, stream=stream)
        torch.cuda.synchronize()
        cold = (time.perf_counter() - t0) * 1e3
        ch = h.last_decision().get("choice")
        t = timed(lambda: h.csr_attention(N, rp, ci, Q, K, V, O, H, d, scale, in_dt=in_dt, workspace=ws, stream=stream), args.iters)
        fused = ch["mapping"] == ab.MAP_FUSED
        row("selector's choice (%s, cold call %.0f ms)" % ("single pass" if fused else "three stages", cold), ch["hub_t"], t,
            b_fused if fused else b_three)
        thresholds = [256, 1024] if deg.max() >= 4096 else [0, 1024]
        for mapping, label, nbytes in ((ab.MAP_FUSED, "single pass", b_fused), (ab.MAP_WAVE_ROW, "three stages", b_three)):
            for hub_t in thresholds:
                sc = ab.Schedule(mapping=mapping, waves_per_wg=4, hub_t=hub_t, hub_chunk=4 * hub_t if mapping == ab.MAP_FUSED else 0)
                wsx = torch.empty(h.workspace_bytes(ab.OP_ATTENTION, N, nnz, d, H, sc), dtype=torch.uint8, device="cuda")
                fn = lambda: h.csr_attention(N, rp, ci, Q, K, V, O, H, d, scale, in_dt=in_dt, sched=sc, workspace=wsx, stream=stream)
                row(label, hub_t, timed(fn, args.iters), nbytes)
                del wsx
        # backward: the chain rule through the three stages on the pattern and on its transpose
        t_rp = torch.empty(N + 1, dtype=torch.int32, device="cuda")
        t_ci = torch.empty(nnz, dtype=torch.int32, device="cuda")
        perm = torch.empty(nnz, dtype=torch.int32, device="cuda")
        wst = torch.empty(h.csr_transpose_workspace_bytes(N, N, nnz), dtype=torch.uint8, device="cuda")
        h.csr_transpose(N, N, nnz, rp, ci, None, t_rp, t_ci, None, perm, wst, stream=stream)
        del wst
        dO = torch.randn((N, H, d), device="cuda", generator=g)
        dQ, dK, dV = (torch.empty((N, H, d), device="cuda") for _ in range(3))
        hub_b = 512 if deg.max() >= 4096 else 0
        wsb = torch.empty(h.csr_attention_backward_workspace_bytes(N, nnz, H, d, hub_b), dtype=torch.uint8, device="cuda")
        tb = timed(lambda: h.csr_attention_backward(N, rp, ci, t_rp, t_ci, perm, Q, K, V, dO, dQ, dK, dV, H, d, scale, in_dt=in_dt,
                                                    hub_t=hub_b, workspace=wsb, stream=stream, nnz=nnz), max(3, args.iters // 2))
        # gathered rows: K and V once (16-bit, one pass for dQ, P and dS), Q once (16-bit) and dO once (fp32) on the
        # transposed side; scores: 8 passes of [nnz, H] fp32 (s and dP written, read, P and dS written and read once more)
        b_bwd = nnz * HD * (3.0 * e + 4.0) + 8.0 * 4 * nnz * H + 4.0 * nnz + 5.0 * N * HD * 4
        print("| backward | %d | %.3f | %.0f | %.2f | %.0f | %.0f %% |" % (hub_b, tb, 10.0 * nnz * HD / tb / 1e6, b_bwd / 1e9, b_bwd / tb / 1e6,
                                                                      100 * b_bwd / tb / 1e6 / HBM_PEAK_GBS), flush=True)
        h.close()
        return

    if args.softmax:
        print("| H | split threshold | forward ms | GB/s | of 8 TB/s | backward ms | GB/s | of 8 TB/s |")
        print("|---|---|---|---|---|---|---|---|")
        for H in (1, 8):
            g = torch.Generator(device="cuda").manual_seed(H)
            s_in = 3.0 * torch.randn((nnz, H), device="cuda", generator=g)
            P = torch.empty_like(s_in)
            dP = torch.randn((nnz, H), device="cuda", generator=g)
            dS = torch.empty_like(s_in)
            for hub_t in (0, 512, 1024, 4096):
                if hub_t == 0 and deg.max() > 100000:
                    continue                                    # one wavefront on a row that long takes tens of ms
                ws = torch.empty(h.workspace_bytes(ab.OP_SOFTMAX, N, nnz, 1, H, ab.Schedule(hub_t=hub_t)), dtype=torch.uint8,
                                 device="cuda")
                tf = timed(lambda: h.csr_row_softmax(N, nnz, rp, s_in, P, H, hub_t, 0, workspace=ws, stream=stream), args.iters)
                tb = timed(lambda: h.csr_row_softmax_backward(N, nnz, rp, P, dP, dS, H, hub_t, 0, workspace=ws, stream=stream),
                           args.iters)
                bf, bb = 8.0 * nnz * H + 4 * (N + 1), 12.0 * nnz * H + 4 * (N + 1)
                print("| %d | %d | %.3f | %.0f | %.0f %% | %.3f | %.0f | %.0f %% |"
                      % (H, hub_t, tf, bf / tf / 1e6, 100 * bf / tf / 1e6 / HBM_PEAK_GBS, tb, bb / tb / 1e6,
                         100 * bb / tb / 1e6 / HBM_PEAK_GBS), flush=True)
        h.close()
        return

    print("| op | F | ms | GFLOP/s | GB/s | of 8 TB/s | compulsory GB/s | fallback ms | speed-up | cold call ms | selector's choice |")
    print("|---|---|---|---|---|---|---|---|---|---|---|")
    for F in widths:
        g = torch.Generator(device="cuda").manual_seed(F)
        B = torch.randn((M, F), device="cuda", generator=g)
        X = torch.randn((N, F), device="cuda", generator=g)
        if args.dtype != "f32":
            half = torch.bfloat16 if args.dtype == "bf16" else torch.float16
            B, X = B.to(half), X.to(half)
        C = torch.empty((N, F), device="cuda")
        out = torch.empty(max(nnz, 1), device="cuda")
        ws = torch.empty(h.workspace_bytes(ab.OP_SPMM, N, nnz, F), dtype=torch.uint8, device="cuda")
        esz = 4 if args.dtype == "f32" else 2
        dt = {"f32": ab.F32, "bf16": ab.BF16, "f16": ab.F16}[args.dtype]
        bg = 4 * (N + 1) + 8 * nnz + nnz * F * esz + N * F * 4
        # compulsory bytes (every array touched once): SpMM reads B and writes C, SDDMM reads X and Y and writes out
        bmin = {"SpMM": 4 * (N + 1) + 8 * nnz + M * F * esz + N * F * 4,
                "SDDMM": 4 * (N + 1) + 4 * nnz + (N + M) * F * esz + 4 * nnz}
        ops = [("SpMM", lambda s: h.spmm(N, M, rp, ci, va, B, C, F, dt=dt, sched=s, workspace=ws, stream=stream))]
        if not args.no_sddmm:
            ops.append(("SDDMM", lambda s: h.sddmm(N, M, rp, ci, X, B, out, F, dt=dt, sched=s, workspace=ws, stream=stream,
                                                   nnz=nnz)))
        for name, fn in ops:
            for sched in explicit or [None]:
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                try:
                    fn(sched)
                except ab.AutosageError as e:
                    print("| %s | %d | | | | | | | | | refused: %s |" % (name, F, short(sched.as_dict())), flush=True)
                    continue
                torch.cuda.synchronize()
                cold = (time.perf_counter() - t0) * 1e3
                choice = h.last_decision().get("choice") if sched is None else sched.as_dict()
                t = timed(lambda: fn(sched), args.iters)
                tb = float("nan") if args.no_fallback else timed(lambda: fn(base), 3)
                print("| %s | %d | %.3f | %.0f | %.0f | %.0f %% | %.0f | %.3f | %.2fx | %.1f | %s%s |"
                      % (name, F, t, 2.0 * nnz * F / t / 1e6, bg / t / 1e6, 100 * bg / t / 1e6 / HBM_PEAK_GBS, bmin[name] / t / 1e6,
                         tb, tb / t, cold, "" if sched is None else "given: ", short(choice)), flush=True)
        if args.vendor and args.dtype == "f32":
            try:
                from . import vendor
                vs = vendor.Session(torch)
                algs = vs.spmm_times(N, M, rp, ci, va, B, C, iters=3)
                tsd = vs.sddmm_time(N, M, rp, ci, X, B, out, iters=3)
                vs.close()
                rows = [("hipSPARSE SpMM (%s)" % min(algs, key=algs.get), min(algs.values()), "SpMM")] if algs else []
                if tsd is not None:
                    rows.append(("hipSPARSE SDDMM", tsd, "SDDMM"))
                for label, tv, kind in rows:
                    print("| %s | %d | %.3f | %.0f | %.0f | %.0f %% | %.0f | | | | |"
                          % (label, F, tv, 2.0 * nnz * F / tv / 1e6, bg / tv / 1e6, 100 * bg / tv / 1e6 / HBM_PEAK_GBS,
                             bmin[kind] / tv / 1e6), flush=True)
            except Exception as e:                      # pragma: no cover
                print("hipSPARSE unavailable: %r" % (e,), file=sys.stderr)
        del B, X, C, out, ws
    h.close()


if __name__ == "__main__":
    main()
