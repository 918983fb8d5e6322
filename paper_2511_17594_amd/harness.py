"""Ablation harness: guardrail, vector width, hub threshold and probe budget, as CSV files with sidecars.

    python -m paper_2511_17594_amd.harness --out results/ --workload config2 --widths 32,64,128 \
        [--ops spmm,sddmm] [--ablate alpha,vec,hubt,probe] [--dtype f32]

Follows the paper's Ablations section (guardrail sensitivity, vectorised versus scalar loads where the
scheduler's kernel is chosen, split threshold versus the measured heavy-row fraction) and its probe
overhead study (sample fraction and per-candidate cap, cold call versus steady-state replay).  Every
CSV gets a `.meta.json` sidecar (device, CU count, torch / HIP versions, AUTOSAGE_* environment, command
line, workload statistics) and every run leaves `<workload>.cache`, the selector's decisions under its
default parameters, which `AUTOSAGE_CACHE=<file> AUTOSAGE_REPLAY_ONLY=1` replays without probing, and
`<workload>_decisions.jsonl`, one decision log per selector call.  Times are medians of `--iters`
HIP-event timings after a warm-up call.
"""
from __future__ import annotations

import argparse
import csv
import json
import os
import sys
import time

import numpy as np

from .sweep import DEFAULT_WIDTHS, make_workload

ALPHAS = [0.80, 0.90, 0.95, 0.98, 1.00]
HUB_TS = [0, 128, 256, 512, 1024, 2048, 4096, 8192]
PROBE_FRACS = [0.01, 0.02, 0.03, 0.05]
PROBE_CAPS = [0.5, 1.0]


def write_csv(path, header, rows, meta):
    with open(path, "w", newline="") as f:
        w = csv.writer(f)
        w.writerow(header)
        w.writerows(rows)
    with open(path + ".meta.json", "w") as f:
        json.dump(meta, f, indent=1, sort_keys=True)
    print("wrote %s (%d rows)" % (path, len(rows)), file=sys.stderr, flush=True)


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--out", required=True, help="directory for the CSV files")
    ap.add_argument("--workload", default="config2", choices=sorted(DEFAULT_WIDTHS))
    ap.add_argument("--widths", default=None)
    ap.add_argument("--ops", default="spmm,sddmm")
    ap.add_argument("--ablate", default="alpha,vec,hubt,probe")
    ap.add_argument("--dtype", default="f32", choices=["f32", "bf16", "f16"])
    ap.add_argument("--iters", type=int, default=10)
    args = ap.parse_args(argv)

    import torch
    from . import binding as ab

    os.makedirs(args.out, exist_ok=True)
    widths = [int(x) for x in args.widths.split(",")] if args.widths else DEFAULT_WIDTHS[args.workload]
    ops = [o for o in args.ops.split(",") if o]
    which = set(args.ablate.split(","))
    A = make_workload(args.workload)
    N, M, nnz = A.n_rows, A.n_cols, A.nnz
    deg = A.degrees
    rp = torch.from_numpy(A.rowptr).cuda()
    ci = torch.from_numpy(A.colind).cuda()
    va = torch.from_numpy(A.val).cuda()
    stream = torch.cuda.current_stream()
    props = torch.cuda.get_device_properties(0)
    meta = {
        "command": "python -m paper_2511_17594_amd.harness " + " ".join(sys.argv[1:]), "utc": time.strftime("%Y-%m-%dT%H:%M:%SZ", time.gmtime()),
        "device": props.name, "arch": getattr(props, "gcnArchName", ""), "compute_units": props.multi_processor_count,
        "hbm_bytes": props.total_memory, "torch": torch.__version__, "hip": torch.version.hip,
        "library": os.path.basename(ab.LIB_PATH), "env": {k: v for k, v in os.environ.items() if k.startswith("AUTOSAGE_")},
        "workload": {"name": args.workload, "n_rows": N, "n_cols": M, "nnz": nnz, "degree_mean": float(deg.mean()),
                     "degree_median": float(np.median(deg)), "degree_max": int(deg.max())},
        "dtype": args.dtype, "iters": args.iters, "timing": "median of HIP-event timings after one warm-up call",
    }
    h = ab.Handle(0)
    h_replay = ab.Handle(0)          # sees one default-parameter decision per (op, F): its cache is the one saved
    meta["device_sig"] = None
    base = ab.baseline_schedule()
    dt = {"f32": ab.F32, "bf16": ab.BF16, "f16": ab.F16}[args.dtype]
    decisions = open(os.path.join(args.out, "%s_decisions.jsonl" % args.workload), "w")

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

    def cold(fn):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        fn(None)
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3
        d = h.last_decision()
        if meta["device_sig"] is None:
            meta["device_sig"] = d.get("device_sig")
        decisions.write(json.dumps(d) + "\n")
        return ms, d

    def sched_from(c, **over):
        s = ab.Schedule(c["mapping"], c["f_tile"], c["waves_per_wg"], c["vec_bytes"], c["unroll"], c["hub_t"],
                        c["hub_chunk"], c["xcd_remap"])
        for k, v in over.items():
            setattr(s, k, v)
        return s

    rows_alpha, rows_vec, rows_hub, rows_probe = [], [], [], []
    for F in widths:
        g = torch.Generator(device="cuda").manual_seed(F)
        B = torch.randn((M, F), device="cuda", generator=g)
        X = torch.randn((N, F), device="cuda", generator=g)
        if args.dtype != "f32":
            half = torch.bfloat16 if args.dtype == "bf16" else torch.float16
            B, X = B.to(half), X.to(half)
        C = torch.empty((N, F), device="cuda")
        out = torch.empty(max(nnz, 1), device="cuda")
        box = {"ws": torch.empty(h.workspace_bytes(ab.OP_SPMM, N, nnz, F), dtype=torch.uint8, device="cuda")}

        def workspace_for(op_id, s):
            need = h.workspace_bytes(op_id, N, nnz, F, sched=s) if s is not None else 0
            if need > box["ws"].numel():
                box["ws"] = torch.empty(need, dtype=torch.uint8, device="cuda")
            return box["ws"]

        calls = {
            "spmm": lambda s, hh=None: (hh or h).spmm(N, M, rp, ci, va, B, C, F, dt=dt, sched=s,
                                                     workspace=workspace_for(ab.OP_SPMM, s), stream=stream),
            "sddmm": lambda s, hh=None: (hh or h).sddmm(N, M, rp, ci, X, B, out, F, dt=dt, sched=s,
                                                       workspace=workspace_for(ab.OP_SDDMM, s), stream=stream, nnz=nnz),
        }
        for op in ops:
            fn = calls[op]
            t_base = timed(lambda: fn(base), 3)
            h.set_param("alpha", 0.95)
            h.cache_clear()
            _, d0 = cold(fn)
            choice = d0["choice"]
            fn(None, h_replay)

            if "alpha" in which:
                # Guardrail sensitivity: same probes, the acceptance threshold moves.
                for a in ALPHAS:
                    h.set_param("alpha", a)
                    h.cache_clear()
                    ms_cold, d = cold(fn)
                    t = timed(lambda: fn(None), args.iters)
                    cands = d.get("candidates", [])
                    t_star = min((c["t_ms"] for c in cands), default=float("nan"))
                    rows_alpha.append([args.workload, op, F, a, d.get("t_baseline_ms"), t_star,
                                       int(d["choice"]["mapping"] != base.mapping), "%.4f" % t, "%.4f" % t_base,
                                       "%.3f" % (t_base / t), "%.2f" % ms_cold, json.dumps(d["choice"])])
                h.set_param("alpha", 0.95)

            if "vec" in which and choice["mapping"] != base.mapping:
                # Vector loads against 4-byte (fp32) / 2-byte (bf16) scalar loads, everything else as chosen.
                scalar = 4 if args.dtype == "f32" else 2
                t_on = timed(lambda: fn(sched_from(choice)), args.iters)
                t_off, off_map = None, None
                # the multi-row mapping has no scalar form at widths of a whole wavefront: use wave-per-row there
                for mp in (choice["mapping"], ab.MAP_WAVE_ROW):
                    try:
                        t_off = timed(lambda: fn(sched_from(choice, vec_bytes=scalar, mapping=mp)), args.iters)
                        off_map = mp
                        break
                    except ab.AutosageError:
                        continue
                rows_vec.append([args.workload, op, F, choice["mapping"], choice["vec_bytes"], "%.4f" % t_on,
                                 off_map if off_map is not None else "", "%.4f" % t_off if t_off else "unsupported",
                                 "%.3f" % (t_off / t_on) if t_off else ""])

            if "hubt" in which:
                for ht in HUB_TS:
                    heavy = deg >= ht if ht > 0 else np.zeros_like(deg, dtype=bool)
                    s = sched_from(choice if choice["mapping"] != base.mapping else
                                   {"mapping": ab.MAP_WAVE_ROW, "f_tile": 0, "waves_per_wg": 4, "vec_bytes": 0, "unroll": 4,
                                    "hub_t": 0, "hub_chunk": 0, "xcd_remap": 0}, hub_t=ht, hub_chunk=ht)
                    try:
                        t = timed(lambda: fn(s), max(3, args.iters // 2))
                    except ab.AutosageError as e:
                        rows_hub.append([args.workload, op, F, ht, int(heavy.sum()), "", "unsupported: %s" % e, "", ""])
                        continue
                    rows_hub.append([args.workload, op, F, ht, int(heavy.sum()),
                                     "%.4f" % (float(deg[heavy].sum()) / max(nnz, 1)), "%.4f" % t, "%.4f" % t_base,
                                     "%.3f" % (t_base / t)])

            if "probe" in which:
                for cap in PROBE_CAPS:
                    for frac in PROBE_FRACS:
                        h.set_param("probe_frac", frac)
                        h.set_param("probe_cap_ms", cap)
                        h.cache_clear()
                        ms_cold, d = cold(fn)
                        t = timed(lambda: fn(None), args.iters)
                        rows_probe.append([args.workload, op, F, frac, cap, d.get("probe_rows"), "%.2f" % ms_cold,
                                           d.get("probe_wall_ms"), "%.4f" % t, "%.1f" % (ms_cold / t),
                                           "%.3f" % (t_base / t), json.dumps(d["choice"])])
                h.set_param("probe_frac", 0.02)
                h.set_param("probe_cap_ms", 1.0)
            print("done %s F=%d" % (op, F), file=sys.stderr, flush=True)
        del B, X, C, out, box
    decisions.close()
    h_replay.cache_save(os.path.join(args.out, "%s.cache" % args.workload))
    h_replay.close()
    tag = os.path.join(args.out, "%s_%s" % (args.workload, args.dtype))
    if rows_alpha:
        write_csv(tag + "_guardrail.csv",
                  ["workload", "op", "F", "alpha", "probe_t_baseline_ms", "probe_t_best_ms", "accepted", "ms", "fallback_ms",
                   "speedup_vs_fallback", "cold_call_ms", "choice"], rows_alpha, meta)
    if rows_vec:
        write_csv(tag + "_vector_loads.csv",
                  ["workload", "op", "F", "mapping", "vec_bytes", "ms_vector", "scalar_mapping", "ms_scalar",
                   "speedup_off_over_on"], rows_vec, meta)
    if rows_hub:
        write_csv(tag + "_hub_threshold.csv",
                  ["workload", "op", "F", "hub_t", "hub_rows", "heavy_nnz_fraction", "ms", "fallback_ms",
                   "speedup_vs_fallback"], rows_hub, meta)
    if rows_probe:
        write_csv(tag + "_probe_budget.csv",
                  ["workload", "op", "F", "probe_frac", "probe_cap_ms", "probe_rows", "cold_call_ms", "probe_wall_ms", "steady_ms",
                   "cold_over_steady", "speedup_vs_fallback", "choice"], rows_probe, meta)
    h.close()


if __name__ == "__main__":
    main()
