"""Turns rocprofv3 output of ``bench.py`` runs into the short summaries under ``profiles/`` and into
``profiles/measured_traffic.json`` (the HBM bytes per launch that ``bench.py`` reports as
``roofline.traffic`` while the kernel sources are unchanged).

Per workload, four rocprofv3 runs of the same committed command are expected in one directory
(``--dir``), each with ``--output-format csv`` and its console output saved beside it:

    <dir>/trace/trace_kernel_trace.csv, <dir>/trace.log      rocprofv3 --kernel-trace --stats -d <dir>/trace -o trace
          -- python3 bench.py --only --no-cpu --workload W --steps 30 --warmup 20
    <dir>/fetch/fetch_counter_collection.csv                 rocprofv3 --pmc FETCH_SIZE --kernel-trace -d <dir>/fetch -o fetch
          -- python3 bench.py --only --no-cpu --workload W --steps 5 --warmup 5 --copy-calibration
    <dir>/write/write_counter_collection.csv                 the same with WRITE_SIZE
    <dir>/inst/inst_counter_collection.csv (optional)        the same with the SQ_* instruction counters, no calibration

Kernel statistics are taken over the launches inside bench.py's timed region only: bench.py reports how
many launches it timed and how many followed them (the first-call samples), and the dispatches of the
main kernel in the trace are counted back from the end.  The wake-up and warm-up launches, which run up
to 15 % slower, are left out, so the kernel's average can be held against bench.py's own step time.

    python -m paper_2512_09685_amd.rocprof_summary --workload bert_base --dir out/prof/bert_base
    python -m paper_2512_09685_amd.rocprof_summary --all-workloads-dir out/prof/all [--op reduce]
"""
from __future__ import annotations

import argparse
import collections
import csv
import dataclasses
import json
import os
import re
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PROFILES = os.path.join(ROOT, "profiles")
TRAFFIC_FILE = os.path.join(PROFILES, "measured_traffic.json")
COPY_KIB = (1 << 28) * 4 / 1024          # the 1 GiB copy of bench.py --copy-calibration
INST_COUNTERS = ["SQ_WAVES", "SQ_INSTS_VALU", "SQ_INSTS_VALU_FMA_F32", "SQ_INSTS_VALU_MFMA_F32",
                 "SQ_INSTS_VALU_MFMA_BF16", "SQ_INSTS_LDS", "SQ_INSTS_VMEM_RD", "SQ_INSTS_VMEM_WR"]


def short(name: str) -> str:
    return re.sub(r"\(.*", "", name).replace("void ", "")


def bench_line(log_path: str) -> dict:
    m = re.search(r'\{"metric".*\}', open(log_path).read())
    if not m:
        raise SystemExit(f"{log_path}: no bench.py JSON line")
    return json.loads(m.group(0))


def dispatches(trace_csv: str):
    """[(kernel, duration_us)] of the library's kernels, in dispatch order."""
    rows = []
    for r in csv.DictReader(open(trace_csv)):
        if "star::" in r["Kernel_Name"]:
            rows.append((int(r["Start_Timestamp"]), short(r["Kernel_Name"]),
                         (int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3))
    rows.sort()
    return [(k, d) for _, k, d in rows]


def timed_only(disp, timed: int, after: int):
    """Per kernel: durations of the launches that fall into the timed region.  A kernel launched n times per
    call appears n * (timed + after) times at the end of the trace; the last n * after are dropped."""
    by = collections.OrderedDict()
    for k, d in disp:
        by.setdefault(k, []).append(d)
    main = max(by, key=lambda k: sum(by[k]))
    per_call = {k: max(1, round(len(v) / len(by[main]))) for k, v in by.items()}
    out = collections.OrderedDict()
    for k, v in by.items():
        n = per_call[k]
        hi = len(v) - n * after
        lo = hi - n * timed
        if lo >= 0 and hi > lo:
            out[k] = v[lo:hi]
    return main, out, {k: len(v) for k, v in by.items()}


def counter_values(path: str, counter: str):
    agg = collections.defaultdict(list)
    for r in csv.DictReader(open(path)):
        if r["Counter_Name"] == counter:
            agg[short(r["Kernel_Name"])].append(float(r["Counter_Value"]))
    return agg


def table(rows):
    return "\n".join("| " + " | ".join(str(c) for c in r) + " |" for r in rows)


def summarise_workload(name: str, d: str, extra: str, tag: str) -> None:
    sys.path.insert(0, ROOT)
    import bench
    import workloads
    wl = workloads.WORKLOADS[name]
    if "--norms on" in extra:
        wl = dataclasses.replace(wl, norms=True)
    b = bench_line(os.path.join(d, "trace.log"))
    roof = b["roofline"]
    timed, after = int(roof["timed_launches"]), int(roof["launches_after_timed"])
    main, sel, total = timed_only(dispatches(os.path.join(d, "trace", "trace_kernel_trace.csv")), timed, after)
    avg = sum(sel[main]) / len(sel[main])
    alg = int(roof["algorithmic_bytes_per_launch"])
    cmd = f"python3 bench.py --only --no-cpu --workload {name}{extra}"
    out = [f"# {main} on workload `{name}`{' (norms forced on)' if extra else ''} (MI355X, rocprofv3)\n",
           f"Workload: P={wl.P:,}, W={wl.W} {wl.grad_dtype} gradient rows, U={wl.U} updates per call, {wl.calls} call(s) "
           f"per step, norms={'on' if wl.norms else 'off'}.  bench.py names the kernel `{roof['kernel']}` "
           f"(from star_plan_choice).\n",
           "## Kernel trace (`--kernel-trace --stats`), launches of the timed region only\n",
           "Command (from the repository root, after `cd /tmp && export TMPDIR=/tmp && cd -`):\n",
           f"    rocprofv3 --kernel-trace --stats -d {d}/trace -o trace --output-format csv -- {cmd} --steps 30 --warmup 20\n",
           f"bench.py timed {timed} launches of the main kernel; {after} more followed them (first-call samples) and "
           f"{total[main] - timed - after} came before (wake-up and warm-up).  Statistics over the {timed} timed ones:\n",
           table([["kernel", "launches", "avg us", "min us", "max us"], ["---"] * 5] +
                 [[f"`{k}`", len(v), f"{sum(v) / len(v):.1f}", f"{min(v):.1f}", f"{max(v):.1f}"]
                  for k, v in sorted(sel.items(), key=lambda kv: -sum(kv[1]))]),
           ""]
    others = sum(sum(v) / len(sel[main]) for k, v in sel.items() if k != main)
    out.append(f"bench.py in the same run (HIP events on the launch stream, whole timed region): {b['ms_per_step']:.4f} ms per "
               f"step = {roof['launch_ms'] * 1e3:.1f} us per launch; rocprofv3: {avg:.1f} us for the main kernel + "
               f"{others:.1f} us for the small kernels of a call = {avg + others:.1f} us.\n")
    out.append(f"Algorithmic bytes per launch: {alg / 1e9:.4f} GB -> {alg / avg / 1e3:.0f} GB/s over the kernel's own time "
               f"({alg / avg / 1e3 / 8000:.3f} of 8 TB/s); {roof['achieved']:.0f} GB/s over the event-timed launch "
               f"({roof['frac']:.3f}).  After a pause: {b['first_call_ms']:.4f} ms for one step (median of 5 single steps, each "
               f"after 250 ms of an idle device).\n")
    traffic = None
    fpath = os.path.join(d, "fetch", "fetch_counter_collection.csv")
    wpath = os.path.join(d, "write", "write_counter_collection.csv")
    if os.path.exists(fpath) and os.path.exists(wpath):
        fetch, write = counter_values(fpath, "FETCH_SIZE"), counter_values(wpath, "WRITE_SIZE")
        cf = max(max(v) for k, v in fetch.items() if "copyBuffer" in k) if any("copyBuffer" in k for k in fetch) else None
        cw = max(max(v) for k, v in write.items() if "copyBuffer" in k) if any("copyBuffer" in k for k in write) else None
        if cf is None or cw is None:
            # the filter applied to the CSVs keeps the copy kernel's rows; without them use the known factors
            cf, cw = COPY_KIB / 2.0, COPY_KIB
        sf, sw = COPY_KIB / cf, COPY_KIB / cw
        kf, kw = fetch[main], write[main]
        fbytes, wbytes = sum(kf) / len(kf) * sf * 1024, sum(kw) / len(kw) * sw * 1024
        # an update reads the rows and the state and writes the state back (8 bytes per element); norms alone only read
        ralg, walg = (alg - 8 * wl.P, 8 * wl.P) if "update" in roof["kernel"] else (alg, 0)
        traffic = fbytes + wbytes
        out += ["## HBM traffic (`--pmc`, one counter per run)\n",
                f"    rocprofv3 --pmc FETCH_SIZE --kernel-trace -d {d}/fetch -o fetch --output-format csv -- {cmd} --steps 5 --warmup 5 --copy-calibration",
                f"    rocprofv3 --pmc WRITE_SIZE --kernel-trace -d {d}/write -o write --output-format csv -- {cmd} --steps 5 --warmup 5 --copy-calibration\n",
                f"Calibration: the plain 1 GiB device copy issued by `--copy-calibration` (`__amd_rocclr_copyBuffer`, 1,048,576 KiB "
                f"read and written) reads FETCH_SIZE = {cf:,.1f} and WRITE_SIZE = {cw:,.1f}, so the scale factors are {sf:.4f} "
                f"(fetch) and {sw:.4f} (write).\n",
                table([["counter", f"per launch (mean of {len(kf)})", "x scale -> bytes", "algorithmic bytes", "ratio"], ["---"] * 5,
                       ["FETCH_SIZE", f"{sum(kf) / len(kf):,.1f}", f"{fbytes / 1e9:.4f} GB", f"{ralg / 1e9:.4f} GB", f"{fbytes / ralg:.4f}"],
                       ["WRITE_SIZE", f"{sum(kw) / len(kw):,.1f}", f"{wbytes / 1e9:.4f} GB", f"{walg / 1e9:.4f} GB",
                        f"{wbytes / walg:.4f}" if walg else "-"],
                       ["total", "", f"{traffic / 1e9:.4f} GB", f"{alg / 1e9:.4f} GB", f"{traffic / alg:.4f}"]]),
                ""]
    ipath = os.path.join(d, "inst", "inst_counter_collection.csv")
    if os.path.exists(ipath):
        vals = {}
        for c in INST_COUNTERS:
            v = counter_values(ipath, c).get(main)
            if v:
                vals[c] = sum(v) / len(v)
        out += ["## Instruction counters (`--pmc`, one run)\n",
                f"    rocprofv3 --pmc {' '.join(INST_COUNTERS)} --kernel-trace -d {d}/inst -o inst --output-format csv -- {cmd} --steps 5 --warmup 5\n",
                "Wave-level instruction counts per launch; x 64 lanes / P = lane-instructions per element.\n",
                table([["counter", "per launch", "per element"], ["---"] * 3] +
                      [[c, f"{vals[c]:,.0f}", "" if c == "SQ_WAVES" else f"{vals[c] * 64 / wl.P:.2f}"] for c in INST_COUNTERS if c in vals]),
                "",
                f"Expected from the source: {2 * wl.W + 2} fp32 FMAs per element for the update (2W + 2, plus two multiplies), "
                f"{wl.W + 2} loads and 2 stores per chunk of 4 elements ({(wl.W + 2) / 4:.2f} and 0.50 per element).\n"]
    os.makedirs(PROFILES, exist_ok=True)
    path = os.path.join(PROFILES, f"{main.split('<')[0].replace('star::', '')}_{tag}.md")
    open(path, "w").write("\n".join(out))
    print("wrote", path)
    if traffic is not None and not extra:
        try:
            tab = json.load(open(TRAFFIC_FILE))
        except (OSError, ValueError):
            tab = {}
        digest = bench.kernel_source_digest()
        if tab.get("kernels_sha256") != digest:
            tab = {"kernels_sha256": digest, "bytes_per_launch": {}}
        tab["note"] = ("HBM bytes per launch of the main kernel (rocprofv3 FETCH_SIZE + WRITE_SIZE, each scaled by a plain "
                       "1 GiB copy), valid for the kernel sources with this digest; written by paper_2512_09685_amd.rocprof_summary")
        tab["bytes_per_launch"][name] = round(traffic)
        json.dump(tab, open(TRAFFIC_FILE, "w"), indent=1, sort_keys=True)
        print("updated", TRAFFIC_FILE)


def summarise_all(d: str, op: str) -> None:
    b = bench_line(os.path.join(d, "trace.log"))
    disp = dispatches(os.path.join(d, "trace", "trace_kernel_trace.csv"))
    by = collections.OrderedDict()
    for k, dur in disp:
        by.setdefault(k, []).append(dur)
    flag = "" if op == "update" else f" --op {op}"
    out = [f"# Kernel statistics of `bench.py{flag}` (all five workloads, MI355X, rocprofv3)\n",
           f"    rocprofv3 --kernel-trace --stats -d {d}/trace -o trace --output-format csv -- python3 bench.py --no-cpu{flag} --steps 30 --warmup 20\n",
           "All launches of the run (wake-up, warm-up, timed and first-call samples together; the per-workload files hold "
           "the timed launches alone):\n",
           table([["kernel", "launches", "avg us", "min us", "max us"], ["---"] * 5] +
                 [[f"`{k}`", len(v), f"{sum(v) / len(v):.1f}", f"{min(v):.1f}", f"{max(v):.1f}"]
                  for k, v in sorted(by.items(), key=lambda kv: -sum(kv[1]))]),
           "\nbench.py's own per-workload figures in that run (HIP events; steady state, and one step after 250 ms idle):\n",
           table([["workload", "ms per step", "per s", "GB/s (algorithmic)", "of 8 TB/s", "first call ms", "of 8 TB/s", "kernel"],
                  ["---"] * 8] +
                 [[c["workload"], f"{c['ms_per_step']:.4f}", f"{c['group_updates_per_s']:.0f}", f"{c['hbm_gbps']:.0f}",
                   f"{c['hbm_frac']:.3f}", f"{c['first_call_ms']:.4f}", f"{c['first_call_hbm_frac']:.3f}", f"`{c['kernel']}`"]
                  for c in b["per_config"]]),
           ""]
    name = "bench_default_all_workloads.md" if op == "update" else f"bench_op_{op}_all_workloads.md"
    open(os.path.join(PROFILES, name), "w").write("\n".join(out))
    print("wrote", os.path.join(PROFILES, name))


def main() -> None:
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--workload")
    ap.add_argument("--dir", help="directory with trace/, fetch/, write/ (and inst/) of one workload")
    ap.add_argument("--extra", default="", help="extra bench.py flags the runs were made with, e.g. ' --norms on'")
    ap.add_argument("--tag", help="suffix of the summary's file name (default: the workload)")
    ap.add_argument("--all-workloads-dir", help="directory with trace/ and trace.log of a run over all workloads")
    ap.add_argument("--op", default="update")
    a = ap.parse_args()
    if a.all_workloads_dir:
        summarise_all(a.all_workloads_dir.rstrip("/"), a.op)
    if a.workload:
        summarise_workload(a.workload, a.dir.rstrip("/"), a.extra, a.tag or a.workload)


if __name__ == "__main__":
    main()
