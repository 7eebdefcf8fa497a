"""Turns rocprofv3 output of `bench.py` runs into the short summaries under profiles/ and the traffic table bench.py reads.

    python -m paper_2506_15689_amd.profile_summary --workload C5 --title "C5 gate/up prefill (M=4096, K=8192, N=28672)" \\
        --bench-args "--config C5" --stats DIR --fetch DIR --write DIR [--pmc DIR ...] --out profiles/NAME.md

DIR = the `-d` directory of one rocprofv3 run (CSV output).  The runs this expects, from the repository root after
`cd /tmp && export TMPDIR=/tmp` ($R = repository, $B = the bench arguments; every run puts the program itself after `--`):

    rocprofv3 --kernel-trace --stats --output-format csv -d STATS -- python3 $R/bench.py --no-cpu-baseline --no-other-workloads $B
    rocprofv3 --pmc FETCH_SIZE --kernel-trace --output-format csv -d FETCH -- python3 $R/bench.py --no-cpu-baseline --no-other-workloads --no-ceilings --calibrate-copy --steps 5 --warmup 2 $B
    rocprofv3 --pmc WRITE_SIZE --kernel-trace --output-format csv -d WRITE -- python3 $R/bench.py ... (same)
    rocprofv3 --pmc <up to 8 SQ_ counters> GRBM_GUI_ACTIVE --kernel-trace --output-format csv -d PMCn -- python3 $R/bench.py --no-cpu-baseline --no-other-workloads --no-ceilings --steps 5 --warmup 2 $B

`--calibrate-copy` adds three plain 256 MiB device-to-device copies whose known size scales FETCH_SIZE and WRITE_SIZE
(KiB per dispatch) to bytes.  HBM-side traffic per launch = factor_fetch * FETCH_SIZE + factor_write * WRITE_SIZE.
The table profiles/traffic.json gets one entry per (workload, kernel of the library) and records the command and the
commit it was measured at.  Nothing here touches a GPU.
"""
from __future__ import annotations

import argparse
import collections
import csv
import glob
import json
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
COPY_KIB = 262144.0
LIB_KERNELS = ("gemm_w4a4", "gemv_w4a4", "rotate_quant", "linear_decode", "diag_read", "diag_stream", "diag_mfma", "pack_fp6")
SIMDS = 1024                     # 256 compute units x 4
XCDS = 8


def short(name: str) -> str:
    name = name.replace("basq::(anonymous namespace)::", "").replace("void ", "")
    return name.split("(")[0][:78]


def one(pattern: str) -> str:
    hits = sorted(glob.glob(pattern))
    if not hits:
        raise SystemExit(f"no file matches {pattern}")
    return hits[-1]


def read_stats(d: str):
    rows = []
    for r in csv.DictReader(open(one(os.path.join(d, "*", "*kernel_stats.csv")))):
        rows.append((short(r["Name"]), int(r["Calls"]), float(r["AverageNs"]) / 1e3, float(r["MinNs"]) / 1e3,
                     float(r["MaxNs"]) / 1e3, float(r["Percentage"])))
    return rows


def read_counters(d: str):
    """{kernel: {counter: [values per dispatch]}} plus {kernel: [durations in ns]} from the same run's kernel trace."""
    agg = collections.defaultdict(lambda: collections.defaultdict(list))
    seen = collections.defaultdict(set)
    span = {}
    for r in csv.DictReader(open(one(os.path.join(d, "*", "*counter_collection.csv")))):
        k = short(r["Kernel_Name"])
        agg[k][r["Counter_Name"]].append(float(r["Counter_Value"]))
        if r["Dispatch_Id"] not in seen[k]:
            seen[k].add(r["Dispatch_Id"])
            span.setdefault(k, []).append(int(r["End_Timestamp"]) - int(r["Start_Timestamp"]))
    return agg, span


def mean(v):
    return sum(v) / len(v) if v else 0.0


def main(argv=None):
    p = argparse.ArgumentParser()
    p.add_argument("--workload", required=True, help="key in profiles/traffic.json (C5, C2, C4, C3_M1, ...)")
    p.add_argument("--title", required=True)
    p.add_argument("--bench-args", required=True, help="the bench.py arguments that select the workload")
    p.add_argument("--stats", required=True)
    p.add_argument("--fetch")
    p.add_argument("--write")
    p.add_argument("--pmc", action="append", default=[])
    p.add_argument("--bench-json", help="file holding the JSON line bench.py printed in the --stats run")
    p.add_argument("--out", required=True)
    p.add_argument("--no-traffic-json", action="store_true")
    p.add_argument("--commit", default="", help="commit the runs were made at (default: the current HEAD)")
    a = p.parse_args(argv)

    out = [f"# rocprofv3 summary: W4A4 rotated linear, {a.title}", ""]
    out.append("Commands (one MI355X, from the repository root after `cd /tmp && export TMPDIR=/tmp`; `$R` is the repository):")
    out.append("")
    B = a.bench_args
    out.append(f"    rocprofv3 --kernel-trace --stats --output-format csv -d out_stats -- python3 $R/bench.py --no-cpu-baseline --no-other-workloads {B}")
    if a.fetch:
        for c in ("FETCH_SIZE", "WRITE_SIZE"):
            out.append(f"    rocprofv3 --pmc {c} --kernel-trace --output-format csv -d out_{c.split('_')[0].lower()} -- python3 $R/bench.py "
                       f"--no-cpu-baseline --no-other-workloads --no-ceilings --calibrate-copy --steps 5 --warmup 2 {B}")
    pmc_data = []
    for d in a.pmc:
        agg, span = read_counters(d)
        names = sorted({c for k in agg for c in agg[k]})
        pmc_data.append((names, agg, span))
        out.append(f"    rocprofv3 --pmc {' '.join(names)} --kernel-trace --output-format csv -d out_pmc{len(pmc_data)} -- python3 $R/bench.py "
                   f"--no-cpu-baseline --no-other-workloads --no-ceilings --steps 5 --warmup 2 {B}")
    out.append(f"    python3 -m paper_2506_15689_amd.profile_summary --workload {a.workload} ... --out {os.path.relpath(a.out, ROOT)}")
    out.append("")

    bench = None
    if a.bench_json and os.path.exists(a.bench_json):
        lines = [l for l in open(a.bench_json).read().splitlines() if l.startswith("{")]
        if lines:
            bench = json.loads(lines[-1])
    if bench:
        r, q = bench.get("roofline") or {}, bench.get("roofline_rotate_quant") or {}
        out.append(f"Bench line of the stats run (profiler attached): {bench['value']:.1f} {bench['unit']}, "
                   f"{bench['ms_per_step'] * 1e3:.1f} us per step; {r.get('kernel')} {r.get('avg_kernel_ms', 0) * 1e3:.2f} us and "
                   f"{q.get('kernel')} {q.get('avg_kernel_ms', 0) * 1e3:.2f} us by the bench's own HIP events "
                   "(the profiler serialises dispatches, so its per-kernel averages differ by a few percent either way).")
        out.append("")

    stats = read_stats(a.stats)
    entries = {}
    if a.fetch and a.write:
        fetch, _ = read_counters(a.fetch)
        write, _ = read_counters(a.write)
        copyk = [k for k in fetch if "copyBuffer" in k]
        if not copyk:
            raise SystemExit("no __amd_rocclr_copyBuffer dispatch in the FETCH run: was --calibrate-copy given?")
        cf = [v for v in fetch[copyk[0]]["FETCH_SIZE"]]
        cw = [v for v in write[copyk[0]]["WRITE_SIZE"]]
        cf = [v for v in cf if v >= 0.5 * max(cf)]          # only the 256 MiB calibration copies
        cw = [v for v in cw if v >= 0.5 * max(cw)]
        ff, wf = COPY_KIB / mean(cf), COPY_KIB / mean(cw)
        out.append(f"Calibration: a plain 256 MiB device copy reads and writes {COPY_KIB:.0f} KiB; FETCH_SIZE reports {mean(cf):.0f} KiB "
                   f"(factor {ff:.3f}), WRITE_SIZE {mean(cw):.0f} KiB (factor {wf:.3f}).  HBM-side bytes per launch = "
                   f"1024 * ({ff:.3f} * FETCH_SIZE + {wf:.3f} * WRITE_SIZE).")
        out.append("")
        out.append("HBM-side traffic per launch, kernels of the library:")
        out.append("")
        out.append(f"    {'kernel':78s} {'launches':>8s} {'FETCH KiB':>12s} {'WRITE KiB':>12s} {'bytes/launch':>14s}")
        avg_us = {k: v for k, _, v, _, _, _ in stats}
        for k in sorted(set(fetch) | set(write)):
            if not any(s in k for s in LIB_KERNELS):
                continue
            f, w = mean(fetch[k]["FETCH_SIZE"]), mean(write[k]["WRITE_SIZE"])
            b = 1024.0 * (ff * f + wf * w)
            out.append(f"    {k:78s} {len(fetch[k]['FETCH_SIZE']):8d} {f:12.1f} {w:12.1f} {b:14.0f}")
            entries[f"{a.workload}/{k}"] = {"bytes_per_launch": int(round(b)), "fetch_kib": round(f, 1), "write_kib": round(w, 1),
                                            "factor_fetch": round(ff, 4), "factor_write": round(wf, 4),
                                            "avg_us_kernel_trace": round(avg_us.get(k, 0.0), 2)}
        if bench:
            r, q = bench.get("roofline") or {}, bench.get("roofline_rotate_quant") or {}
            out.append("")
            out.append(f"    algorithmic bytes the bench prices with: {q.get('kernel')} {q.get('algorithmic_bytes')} "
                       f"(this design's own: {q.get('design_bytes')}); {r.get('kernel')} {r.get('algorithmic_bytes')}"
                       + (f" ({int(r['algorithmic_ops'])} operations)" if r.get("algorithmic_ops") else ""))
        out.append("")

    out.append("```")
    out.append("kernel-trace --stats (per kernel)")
    out.append(f"{'kernel':78s} {'calls':>6s} {'avg_us':>10s} {'min_us':>10s} {'max_us':>10s} {'pct':>6s}")
    for k, calls, avg, mn, mx, pct in stats:
        if pct >= 0.05 or any(s in k for s in LIB_KERNELS):
            out.append(f"{k:78s} {calls:6d} {avg:10.2f} {mn:10.2f} {mx:10.2f} {pct:6.2f}")
    out.append("```")

    for i, (names, agg, span) in enumerate(pmc_data):
        out.append("")
        out.append(f"Counters, set {i + 1} (mean per dispatch over the launches of the run; SQ_ counters are summed over the chip, "
                   f"GRBM_GUI_ACTIVE over its {XCDS} XCDs):")
        out.append("")
        out.append("```")
        for k in sorted(agg):
            if not any(s in k for s in LIB_KERNELS) or "diag_read" in k or "diag_stream" in k or "pack_fp6" in k:
                continue
            c = {n: mean(v) for n, v in agg[k].items()}
            n = len(next(iter(agg[k].values())))
            if n < 3:                                    # one-off preparation kernels
                continue
            out.append(f"{k}   (launches {n}, mean duration under the counters {mean(span.get(k, [0])) / 1e3:.1f} us)")
            for name in names:
                if name in c:
                    out.append(f"    {name:28s} {c[name]:16.4g}")
            cyc = c.get("GRBM_GUI_ACTIVE", 0.0) / XCDS                      # cycles of the kernel on one XCD's clock
            d = []
            if cyc > 0:
                ns = mean(span.get(k, [0]))
                if ns > 0 and cyc / ns <= 2.45:
                    d.append(f"shader clock {cyc / ns:.2f} GHz")
                elif ns > 0:
                    # a kernel of a few microseconds: the busy counter also covers the dispatch's ramp, so it does not
                    # give the clock; percentages below are then against the nominal 2.4 GHz over the kernel's duration
                    cyc = 2.4 * ns
                    d.append("cycles taken as 2.4 GHz x duration (the GUI-active counter also covers the ramp of a kernel this short)")
                if "SQ_VALU_MFMA_BUSY_CYCLES" in c:
                    d.append(f"MFMA pipe busy {100 * c['SQ_VALU_MFMA_BUSY_CYCLES'] / (SIMDS * cyc):.1f} % of SIMD cycles")
                if "SQ_ACTIVE_INST_VALU" in c:
                    d.append(f"VALU issuing {100 * c['SQ_ACTIVE_INST_VALU'] / (SIMDS * cyc) * 4:.1f} % of SIMD cycles (x4 cycles per wave instruction)")
                if "SQ_LDS_IDX_ACTIVE" in c:
                    d.append(f"LDS index unit active {100 * c['SQ_LDS_IDX_ACTIVE'] / (SIMDS / 4 * cyc):.1f} % of CU cycles")
                if "SQ_LDS_BANK_CONFLICT" in c and c.get("SQ_LDS_IDX_ACTIVE"):
                    d.append(f"LDS bank-conflict cycles {100 * c['SQ_LDS_BANK_CONFLICT'] / c['SQ_LDS_IDX_ACTIVE']:.1f} % of LDS active cycles")
            if c.get("SQ_WAVE_CYCLES"):
                wc = c["SQ_WAVE_CYCLES"]
                if "SQ_WAIT_INST_ANY" in c:
                    d.append(f"waves waiting in s_waitcnt {100 * c['SQ_WAIT_INST_ANY'] / wc:.1f} % of wave cycles")
                if "SQ_WAIT_INST_LDS" in c:
                    d.append(f"... of which for LDS {100 * c['SQ_WAIT_INST_LDS'] / wc:.1f} %")
                if "SQ_WAIT_ANY" in c:
                    d.append(f"waves waiting for anything {100 * c['SQ_WAIT_ANY'] / wc:.1f} % of wave cycles")
            key = f"{a.workload}/{k}"
            if key in entries:                           # instruction counts per launch, for the issue-rate view of bench.py
                for nm, field in (("SQ_INSTS_VALU", "valu_insts_per_launch"), ("SQ_INSTS_MFMA", "mfma_insts_per_launch"),
                                  ("SQ_WAVES", "waves_per_launch")):
                    if nm in c:
                        entries[key][field] = int(round(c[nm]))
            if c.get("SQ_WAVES"):
                w = c["SQ_WAVES"]
                for nm, label in (("SQ_INSTS_VALU", "VALU"), ("SQ_INSTS_MFMA", "MFMA"), ("SQ_INSTS_LDS", "LDS"), ("SQ_INSTS_VMEM", "VMEM")):
                    if nm in c:
                        d.append(f"{label} instructions per wave {c[nm] / w:.0f}")
            if d:
                out.append("    -> " + "; ".join(d))
        out.append("```")

    os.makedirs(os.path.dirname(os.path.abspath(a.out)), exist_ok=True)
    with open(a.out, "w") as f:
        f.write("\n".join(out) + "\n")
    print("wrote", a.out)

    if entries and not a.no_traffic_json:
        path = os.path.join(ROOT, "profiles", "traffic.json")
        table = {"entries": {}}
        if os.path.exists(path):
            try:
                table = json.load(open(path))
            except ValueError:
                pass
        table.setdefault("entries", {})
        for k in [k for k in table["entries"] if k.startswith(a.workload + "/")]:
            del table["entries"][k]
        commit = a.commit
        if not commit:
            try:
                commit = subprocess.run(["git", "-C", ROOT, "rev-parse", "--short", "HEAD"], stdout=subprocess.PIPE, text=True).stdout.strip()
            except OSError:
                commit = ""
        for k, e in entries.items():
            e["measured_at_commit"] = commit
            e["summary"] = os.path.relpath(a.out, ROOT)
            table["entries"][k] = e
        table["source"] = ("rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of bench.py --calibrate-copy, summarised by "
                           "python -m paper_2506_15689_amd.profile_summary (commands in the profiles/*.md each entry names)")
        with open(path, "w") as f:
            json.dump(table, f, indent=1, sort_keys=True)
            f.write("\n")
        print("updated", path)


def sweep_main(argv):
    """profile_summary sweep --title T --out FILE --kernel NAME --bench-args-common "..." --point "label|bytes|DIR" ...:
    one table of kernel-trace averages over several runs (token-count sweeps of the rotate+quant kernels)."""
    p = argparse.ArgumentParser(prog="profile_summary sweep")
    p.add_argument("--title", required=True)
    p.add_argument("--out", required=True)
    p.add_argument("--kernel", required=True, help="kernel name prefix to report")
    p.add_argument("--bench-args-common", required=True)
    p.add_argument("--point", action="append", default=[], help="'<bench args of the point>|<algorithmic bytes per launch>|<stats dir>'")
    a = p.parse_args(argv)
    out = [f"# rocprofv3 summary: {a.title}", "",
           "One run per row (one MI355X, from the repository root after `cd /tmp && export TMPDIR=/tmp`; `$R` is the repository):", "",
           f"    rocprofv3 --kernel-trace --stats --output-format csv -d out_<row> -- python3 $R/bench.py {a.bench_args_common} <row's arguments>",
           "", "Algorithmic bytes = tokens * (2 K bf16 in + K/2 of codes + 16 of record), i.e. without the fp6 copy of the codes that",
           "this design may write on top; GB/s and the fraction of the 8 TB/s HBM peak are priced on those bytes.", "", "```",
           f"{'arguments':44s} {'kernel':58s} {'calls':>5s} {'avg_us':>9s} {'min_us':>9s} {'alg. MB':>9s} {'GB/s':>8s} {'of 8 TB/s':>9s}"]
    for pt in a.point:
        args_pt, nbytes, d = pt.split("|")
        nbytes = float(nbytes)
        rows = [r for r in read_stats(d) if r[0].startswith(a.kernel)]
        for k, calls, avg, mn, mx, pct in rows:
            if calls < 3:
                continue
            gbs = nbytes / (avg * 1e-6) / 1e9
            out.append(f"{args_pt:44s} {k[:58]:58s} {calls:5d} {avg:9.2f} {mn:9.2f} {nbytes / 1e6:9.2f} {gbs:8.0f} {gbs / 8000.0:9.3f}")
    out.append("```")
    with open(a.out, "w") as f:
        f.write("\n".join(out) + "\n")
    print("wrote", a.out)


if __name__ == "__main__":
    if len(sys.argv) > 1 and sys.argv[1] == "sweep":
        sweep_main(sys.argv[2:])
    else:
        main()
