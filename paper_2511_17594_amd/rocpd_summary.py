"""Short text summaries of rocprofv3 output databases (rocpd SQLite files), as kept under profiles/.

    python -m paper_2511_17594_amd.rocpd_summary kernels  <kernel-trace .db>
    python -m paper_2511_17594_amd.rocpd_summary counters <FETCH_SIZE .db> <WRITE_SIZE .db> [--traffic-out FILE]
    python -m paper_2511_17594_amd.rocpd_summary fetch    <FETCH_SIZE .db>
    python -m paper_2511_17594_amd.rocpd_summary issue    <SQ counters .db> [--match REGEX]

`kernels` prints calls / total / average duration per kernel from the profiler's per-dispatch begin and
end times, and the average over the last `--last` dispatches of each kernel: the selector's cold calls
launch the same kernels on row samples, so only the trailing dispatches are the timed steps.
`counters` scales the two HBM counters by what they read for the plain 1 GiB device copies that
`bench.py --copy-calibration` issues (1 GiB read and 1 GiB written per copy), prints the HBM bytes per
launch of every kernel (mean over its last `--last` dispatches, the full-input ones), and with
`--traffic-out` writes the "stage bytes" lines that `bench.py` reports as `roofline.traffic`.
`fetch` is the read half alone (one profiler run), with the rate each kernel fetched at.
`issue` reads a run with SQ_WAVES, SQ_INSTS_VALU, SQ_INSTS_SALU, SQ_INSTS_LDS and SQ_INSTS_VMEM_RD and prints the
instructions per wavefront of every kernel and the share of the kernel's duration that issuing its vector-ALU
instructions alone takes (4 cycles each on one of the 4 x 256 SIMDs at 2.4 GHz): how far a kernel is from being
bound by instruction issue rather than by memory.
Reads only; runs on the CPU.
"""
from __future__ import annotations

import argparse
import re
import sqlite3

STAGE_OF = [  # kernel-name pattern -> stage name used by the library's per-stage telemetry
    (r"spmm_rows_kernel<bf16_t.*true>", "attn_spmm_rows"),
    (r"spmm_hub_partial_kernel<bf16_t.*true>", "attn_spmm_hub"),
    (r"sddmm_rows_kernel<bf16_t", "attn_sddmm_rows"),
    (r"sddmm_hub_kernel<bf16_t", "attn_sddmm_hub"),
    (r"attn_fused_rows_kernel", "attn_fused_rows"),
    (r"attn_fused_hub_partial_kernel", "attn_fused_hub"),
    (r"spmm_rows_kernel<float", "spmm_rows"),
    (r"spmm_hub_partial_kernel<float", "spmm_hub"),
    (r"sddmm_rows_kernel<float", "sddmm_rows"),
    (r"sddmm_hub_kernel<float", "sddmm_hub"),
    (r"softmax_rows_kernel", "softmax_rows"),
]


def short(name):
    name = re.sub(r"^void ", "", name)
    name = name.replace("autosage::", "").replace("(anonymous namespace)::", "")
    name = re.sub(r"\(.*\)$", "", name)
    return name[:100]


def kernel_table(path, last):
    db = sqlite3.connect(path)
    agg = {}
    for name, dur in db.execute("select name, duration from kernels order by start"):
        agg.setdefault(short(name), []).append(dur)
    total = sum(sum(v) for v in agg.values())
    lines = ["| kernel | calls | total ms | avg ms | avg ms, last %d calls | %% |" % last, "|---|---|---|---|---|---|"]
    for k, v in sorted(agg.items(), key=lambda kv: -sum(kv[1])):
        tail = v[-last:]
        lines.append("| `%s` | %d | %.3f | %.4f | %.4f | %.1f |"
                     % (k, len(v), sum(v) / 1e6, sum(v) / len(v) / 1e6, sum(tail) / len(tail) / 1e6, 100 * sum(v) / total))
    return "\n".join(lines)


def counter_samples(path):
    db = sqlite3.connect(path)
    agg = {}
    for kn, cn, v, dur in db.execute("select kernel_name, counter_name, value, duration from counters_collection order by start"):
        agg.setdefault((short(kn), cn), []).append((v, dur))
    return agg


def bytes_per_unit(agg, gib_per_launch=1.0):
    """Counter units of the three largest copy dispatches (the 1 GiB calibration copies) -> bytes per unit."""
    vals = sorted(v for (k, _), l in agg.items() if "copyBuffer" in k for v, _ in l)[-3:]
    if not vals:
        raise SystemExit("no copy kernel in the database: run bench.py with --copy-calibration")
    return gib_per_launch * (1 << 30) / (sum(vals) / len(vals))


def counter_report(fetch_path, write_path, last):
    fetch, write = counter_samples(fetch_path), counter_samples(write_path)
    bf, bw = bytes_per_unit(fetch), bytes_per_unit(write)
    out = ["bytes per FETCH_SIZE unit (from the 1 GiB copy): %.1f" % bf,
           "bytes per WRITE_SIZE unit (from the 1 GiB copy): %.1f" % bw, "",
           "FETCH_SIZE, WRITE_SIZE and ms are means over the last %d launches of each kernel." % last, "",
           "| kernel | stage | launches | FETCH_SIZE | WRITE_SIZE | HBM read MB | HBM write MB | total MB / launch | ms |",
           "|---|---|---|---|---|---|---|---|---|"]
    rows = []
    for (k, _), l in fetch.items():
        if "plain" in k or "copyBuffer" in k or "at::" in k:
            continue
        n_all = len(l)
        w = write.get((k, "WRITE_SIZE"), [])[-last:]
        l = l[-last:]
        fm = sum(v for v, _ in l) / len(l)
        wm = sum(v for v, _ in w) / max(len(w), 1)
        dm = sum(d for _, d in l) / len(l) / 1e6
        stage = next((s for p, s in STAGE_OF if re.search(p, k)), "")
        rows.append((dm * n_all, k, stage, n_all, fm, wm, fm * bf / 1e6, wm * bw / 1e6, dm))
    rows.sort(reverse=True)
    for _, k, stage, n, fm, wm, rb, wb, dm in rows:
        out.append("| `%s` | %s | %d | %.0f | %.0f | %.1f | %.1f | %.1f | %.4f |" % (k, stage, n, fm, wm, rb, wb, rb + wb, dm))
    traffic, seen = [], set()
    for _, k, stage, n, fm, wm, rb, wb, dm in rows:      # the most-launched variant of a stage is the steady-state one
        if stage and stage not in seen and n >= last:
            seen.add(stage)
            traffic.append("%s %d" % (stage, int((rb + wb) * 1e6)))
    return "\n".join(out), traffic


def fetch_report(fetch_path, last):
    fetch = counter_samples(fetch_path)
    bf = bytes_per_unit(fetch)
    out = ["bytes per FETCH_SIZE unit (from the 1 GiB copy): %.1f" % bf, "",
           "FETCH_SIZE and ms are means over the last %d launches of each kernel." % last, "",
           "| kernel | launches | FETCH_SIZE | HBM read MB | ms | read GB/s |", "|---|---|---|---|---|---|"]
    for (k, _), l in fetch.items():
        if "plain" in k or "copyBuffer" in k or "at::" in k or len(l) < last:
            continue
        tail = l[-last:]
        fm = sum(v for v, _ in tail) / len(tail)
        dm = sum(d for _, d in tail) / len(tail) / 1e6
        out.append("| `%s` | %d | %.0f | %.1f | %.4f | %.0f |" % (k, len(l), fm, fm * bf / 1e6, dm, fm * bf / dm / 1e6))
    return "\n".join(out)


SIMDS, CLOCK_GHZ, VALU_CYCLES = 256 * 4, 2.4, 4


def issue_report(path, last, match):
    agg = counter_samples(path)
    kernels = sorted({k for k, _ in agg})
    out = ["Means over the last %d launches of each kernel; VALU issue = SQ_INSTS_VALU x %d cycles / %d SIMDs / (duration x %.1f GHz)."
           % (last, VALU_CYCLES, SIMDS, CLOCK_GHZ), "",
           "| kernel | launches | ms | wavefronts | VALU / wave | SALU / wave | LDS / wave | VMEM read / wave | VALU issue |",
           "|---|---|---|---|---|---|---|---|---|"]
    for k in kernels:
        if (match and not re.search(match, k)) or (k, "SQ_WAVES") not in agg:
            continue

        def mean(counter):
            tail = agg.get((k, counter), [])[-last:]
            return sum(v for v, _ in tail) / len(tail) if tail else 0.0

        tail = agg[(k, "SQ_WAVES")][-last:]
        dur_ns = sum(d for _, d in tail) / len(tail)
        waves = mean("SQ_WAVES")
        if waves <= 0 or dur_ns <= 0:
            continue
        valu = mean("SQ_INSTS_VALU")
        out.append("| `%s` | %d | %.4f | %.0f | %.0f | %.0f | %.0f | %.1f | %.0f %% |"
                   % (k, len(agg[(k, "SQ_WAVES")]), dur_ns / 1e6, waves, valu / waves, mean("SQ_INSTS_SALU") / waves,
                      mean("SQ_INSTS_LDS") / waves, mean("SQ_INSTS_VMEM_RD") / waves,
                      100.0 * valu * VALU_CYCLES / SIMDS / (dur_ns * CLOCK_GHZ)))
    return "\n".join(out)


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    sub = ap.add_subparsers(dest="cmd", required=True)
    k = sub.add_parser("kernels")
    k.add_argument("db")
    k.add_argument("--last", type=int, default=30, help="dispatches per kernel that belong to the timed steps")
    c = sub.add_parser("counters")
    c.add_argument("fetch_db")
    c.add_argument("write_db")
    c.add_argument("--traffic-out", default=None)
    c.add_argument("--last", type=int, default=5, help="dispatches per kernel that belong to the timed steps")
    f = sub.add_parser("fetch")
    f.add_argument("db")
    f.add_argument("--last", type=int, default=5)
    i = sub.add_parser("issue")
    i.add_argument("db")
    i.add_argument("--last", type=int, default=3)
    i.add_argument("--match", default=None, help="only kernels whose short name matches this regular expression")
    args = ap.parse_args(argv)
    if args.cmd == "issue":
        print(issue_report(args.db, args.last, args.match))
        return
    if args.cmd == "fetch":
        print(fetch_report(args.db, args.last))
        return
    if args.cmd == "kernels":
        print(kernel_table(args.db, args.last))
        return
    text, traffic = counter_report(args.fetch_db, args.write_db, args.last)
    print(text)
    if args.traffic_out:
        with open(args.traffic_out, "w") as f:
            f.write("# stage  HBM bytes per launch (FETCH_SIZE + WRITE_SIZE, scaled by the copy calibration)\n")
            f.write("\n".join(traffic) + "\n")


if __name__ == "__main__":
    main()
