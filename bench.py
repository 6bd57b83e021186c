#!/usr/bin/env python3
"""Benchmark of the group-synchronous parameter update on one MI355X.

A step is one pass of the whole path over one batch of synthetic input: all
calls of the workload (one star_group_update with U updates; four back-to-back
calls for the streamed BERT-large workload), gradient norms included where the
workload asks for them.  Inputs are resident in HBM before the timed region.
Before the W warm-up steps the same calls run untimed for 80 ms ("wake-up": the
device's step times settle only after 25-50 ms of sustained work); then exactly
K steps are timed.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--only]
"""
import argparse
import json
import os
import sys
import time

HBM_PEAK_GBPS = 8000.0   # MI355X HBM3E, published peak
WAKEUP_SECONDS = 0.08    # untimed work before the warm-up steps, see measure()
FIRST_CALL_IDLE = 0.25   # seconds the device idles before each "first call" sample
FIRST_CALL_REPS = 5

# HBM bytes per launch of the dominant kernel, from rocprofv3 FETCH_SIZE / WRITE_SIZE runs (each scaled by what
# the same counter reads for a plain 1 GiB copy).  profiles/measured_traffic.json holds them together with a digest
# of the kernel sources they were taken with (star_kernels.hip, star_mfma_kernels.hip and star_device.h, hashed
# without comments and white space); it is written by `python -m paper_2512_09685_amd.rocprof_summary`.
TRAFFIC_FILE = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", "measured_traffic.json")


def kernel_source_digest():
    """sha256 of the kernel sources with comments and white space removed: it changes when the code does."""
    import hashlib
    import re
    csrc = os.path.join(os.path.dirname(os.path.abspath(__file__)), "paper_2512_09685_amd", "csrc")
    h = hashlib.sha256()
    for name in ("star_kernels.hip", "star_mfma_kernels.hip", "star_reduce_kernels.hip", "star_device.h", "star_kernels.h"):
        text = open(os.path.join(csrc, name), "r").read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        text = re.sub(r"//[^\n]*", "", text)
        h.update(re.sub(r"\s+", "", text).encode())
    return h.hexdigest()


def measured_traffic(workload):
    try:
        table = json.load(open(TRAFFIC_FILE))
        digest = kernel_source_digest()
    except (OSError, ValueError):
        return None
    if digest != table.get("kernels_sha256"):
        return None            # the kernels changed since the counters were taken
    return table.get("bytes_per_launch", {}).get(workload)


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=20,
                    help="untimed steps first; the step time keeps falling for the first 25-50 ms of sustained work "
                         "(bert_base: 1.64 ms for the first step after a pause, 1.46 ms from about the 12th on)")
    ap.add_argument("--workload", default="bert_base",
                    help="headline workload: tiny | resnet50 | bert_base | vgg16 | bert_large")
    ap.add_argument("--only", action="store_true", help="measure the headline workload only (no per-config table)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--kernel", default="auto", choices=["auto", "seq", "affine", "affine_mfma"])
    ap.add_argument("--norms", default="workload", choices=["workload", "on", "off"],
                    help="per-group gradient norms: as the workload defines them (default), or forced on / off")
    ap.add_argument("--op", default="update", choices=["update", "publish", "reduce", "norms"],
                    help="update: star_group_update (the headline path); publish: the same with a bf16 copy of the "
                         "new params written in the pass; reduce: star_group_reduce, one full-group aggregation per "
                         "call; norms: star_group_norms alone (the rows are read, nothing is written)")
    ap.add_argument("--updates", type=int, default=0,
                    help="updates per call instead of the workload's (1 = every gradient report applied on arrival)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="before the timed region, run three plain device copies of 1 GiB (a known-size kernel to "
                         "scale rocprofv3's FETCH_SIZE / WRITE_SIZE counters against)")
    return ap.parse_args()


KERNEL_OPTION = None      # star_options.kernel of every call (None: the library chooses)
KERNEL_NAMES = {1: "seq_kernel", 2: "aff_kernel", 3: "aff_mfma_kernel"}


def kernel_label(star, wl, us, op):
    """Name of the main kernel of a call, from the library's own account of what it launches."""
    c = star.star_plan_choice(wl.P, wl.W, wl.grad_dtype, us, lr=wl.lr, momentum_coef=wl.momentum,
                              weight_decay=wl.weight_decay, wmode=wl.wmode, update=op != "norms",
                              want_norms=wl.norms or op == "norms", kernel=KERNEL_OPTION)
    row = "RowF32" if c["grad_dtype"] == 0 else "RowBf16x4"
    what = "norms only" if op == "norms" else ("update+norms" if wl.norms else "update")
    order = "queue order" if c["queue_order"] else "fixed assignment"
    return f"{KERNEL_NAMES[c['kernel']]}<{c['rows_padded']}, {row}> {what}, {order}", c


def measure(wl, steps, warmup, torch, star, workloads, op="update"):
    """Times `steps` steps of workload `wl`; returns a dict of results."""
    import numpy as np
    dev = "cuda"
    stream = torch.cuda.Stream()
    p = workloads.make_params(wl, 0, dev)
    v = workloads.make_momentum(wl, dev)
    nsets = wl.calls if wl.fresh_grads_per_call else 1
    # the rows' pointers are marshalled once, as a server does that receives its reports in fixed buffers
    sets = [star.GradRows(workloads.make_grad_rows(wl, 0, c, dev)) for c in range(nsets)]
    streams = []
    for c in range(wl.calls):
        s = workloads.make_update_stream(wl, 0, c)
        streams.append(star.UpdateStream(s["offsets"], s["members"], s["staleness"]))
    norms = ([torch.zeros(wl.U, device=dev) for _ in range(wl.calls)] if wl.norms or op == "norms"
             else [None] * wl.calls)
    hp = dict(lr=wl.lr, momentum_coef=wl.momentum, weight_decay=wl.weight_decay, wmode=wl.wmode)
    extra_bytes = 0
    if op == "publish":
        pub = torch.empty(wl.P, dtype=torch.bfloat16, device=dev)
        extra_bytes = 2 * wl.P
    if op == "reduce":
        # one aggregation of all W rows per call (a parent adding its children's gradients to its own),
        # output in the gradients' dtype
        full = star.UpdateStream(np.array([0, wl.W], np.int32), np.arange(wl.W, dtype=np.int32))
        out = [torch.empty(wl.P, dtype=sets[0][0].dtype, device=dev)]
    torch.cuda.synchronize()

    def step():
        for c in range(wl.calls):
            if op == "update":
                star.star_group_update(p, v, sets[c % nsets], streams[c], norms_out=norms[c], stream=stream,
                                       kernel=KERNEL_OPTION, **hp)
            elif op == "publish":
                star.star_group_update_publish(p, v, sets[c % nsets], streams[c], pub, norms_out=norms[c],
                                               stream=stream, kernel=KERNEL_OPTION, **hp)
            elif op == "norms":
                star.star_group_norms(sets[c % nsets], streams[c], norms[c], wmode=wl.wmode, stream=stream,
                                      kernel=KERNEL_OPTION)
            else:
                star.star_group_reduce(out, sets[c % nsets], full, norms_out=None if norms[c] is None else norms[c][:1],
                                       stream=stream, kernel=KERNEL_OPTION)

    # Wake-up: after a pause the device needs 25-50 ms of sustained work before step times settle (the first
    # steps run 10-30 % slower), whatever --warmup says; untimed, like the warm-up steps that follow.
    t_wake, n_wake = time.perf_counter(), 0
    while time.perf_counter() - t_wake < WAKEUP_SECONDS:
        step()
        stream.synchronize()
        n_wake += 1
    for _ in range(warmup):
        step()
    stream.synchronize()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps)]
    e0.record(stream)
    for i in range(steps):
        step()
        marks[i].record(stream)       # per-step times for the median / minimum; the headline is the whole region
    e1.record(stream)
    stream.synchronize()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    ev_ms = e0.elapsed_time(e1)
    ms_per_step = ev_ms / steps
    per_step = sorted(a.elapsed_time(b) for a, b in zip([e0] + marks[:-1], marks))
    assert bool(torch.isfinite(p[:: max(1, wl.P // 4096)]).all()), "non-finite parameters after the timed steps"

    # A step after a pause: the paper's server is called once per training iteration, 100-800 ms apart
    # (Section 5.1, overhead of STAR), not back to back.  One step after FIRST_CALL_IDLE seconds of an idle
    # device, five times; the median is reported beside the steady-state figure.
    first = []
    for _ in range(FIRST_CALL_REPS):
        torch.cuda.synchronize()
        time.sleep(FIRST_CALL_IDLE)
        a0, a1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a0.record(stream)
        step()
        a1.record(stream)
        stream.synchronize()
        first.append(a0.elapsed_time(a1))
    first.sort()
    first_call_ms = first[len(first) // 2]

    # rows referenced per call (each call reads only the rows its own groups name), averaged over the calls
    used = [set(int(x) for x in us.members) for us in streams]
    n_used = sum(len(u) for u in used) / len(used)
    bytes_per_call = int(sum(wl.algorithmic_bytes_per_call(len(u)) for u in used) / len(used)) + extra_bytes
    n_updates = wl.U
    label, choice = kernel_label(star, wl, streams[0], op)
    fs, fa = choice["fma_seq"], choice["fma_affine"]
    if op == "reduce":
        bytes_per_call = wl.P * (wl.W * wl.grad_bytes + wl.grad_bytes)      # W rows read, one output row written
        n_updates = 1
        label = f"reduce_rows_kernel<{wl.W}, {'RowF32' if wl.grad_dtype == 'f32' else 'RowBf16x4'}>"
        fs, fa = float(wl.W + (1 if wl.norms else 0)), None
    if op == "norms":
        bytes_per_call = int(wl.P * n_used * wl.grad_bytes)                 # the referenced rows, read once
    bytes_per_step = bytes_per_call * wl.calls
    gbps = bytes_per_step / (ms_per_step * 1e-3) / 1e9
    res = {
        "workload": wl.name, "op": op, "P": wl.P, "W": wl.W, "U_per_call": wl.U, "calls_per_step": wl.calls,
        "grad_dtype": wl.grad_dtype, "norms": wl.norms,
        "group_updates_per_s": n_updates * wl.calls / (ms_per_step * 1e-3),
        "ms_per_step": ms_per_step, "wall_ms_per_step": wall_ms / steps,
        "ms_per_step_median": per_step[len(per_step) // 2], "ms_per_step_min": per_step[0],
        "wakeup_steps": n_wake, "first_call_ms": first_call_ms,
        "first_call_hbm_frac": bytes_per_call * wl.calls / (first_call_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
        "timed_launches": steps * wl.calls,
        "algorithmic_bytes_per_step": bytes_per_step, "bytes_per_element": bytes_per_call / wl.P,
        "hbm_gbps": gbps, "hbm_frac": gbps / HBM_PEAK_GBPS, "kernel": label,
        "fma_per_element_seq": fs, "fma_per_element_affine": fa,
        "launch_ms": ms_per_step / wl.calls, "bytes_per_launch": bytes_per_call,
    }
    del p, v, sets, norms
    if op == "publish":
        del pub
    if op == "reduce":
        del out
    torch.cuda.empty_cache()
    return res


def device_copy_gbps(torch):
    """Bandwidth of a plain device-to-device copy of 1 GiB (read + written bytes over time), for context: what
    the memory system gives the simplest mixed read / write stream."""
    src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
    dst = torch.empty_like(src)
    t0 = time.perf_counter()
    while time.perf_counter() - t0 < WAKEUP_SECONDS:
        dst.copy_(src)
        torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(10):
        dst.copy_(src)
    e1.record()
    torch.cuda.synchronize()
    gbps = 10 * 2 * src.numel() * 4 / (e0.elapsed_time(e1) * 1e-3) / 1e9
    del src, dst
    torch.cuda.empty_cache()
    return gbps


def cpu_baseline(wl, torch, workloads):
    """The CPU oracle, one thread pinned to one core, on a contiguous slice of the same workload; elements are
    independent, so the full-shard rate is the slice's rate scaled by the slice fraction.  Two timings of about
    8 s each: the exact mode (fp64 arithmetic, the parity reference; this is `value`) and the stepwise-fp32 mode
    (what a literal fp32 parameter server computes: add the gradient copies, then update, Section 2)."""
    import numpy as np
    from oracle import star_oracle as so

    def run(P, mode):
        w = wl.scaled(P)
        rows = workloads.rows_to_numpy(workloads.make_grad_rows(w, 0, 0, "cpu"))
        p0 = workloads.make_params(w, 0, "cpu").numpy()
        s = workloads.make_update_stream(w, 0, 0)
        t = time.perf_counter()
        so.group_update(p0, np.zeros_like(p0), rows, s["offsets"], s["members"], staleness=s["staleness"],
                        lr=w.lr, momentum_coef=w.momentum, weight_decay=w.weight_decay, wmode=w.wmode,
                        want_norms=w.norms, mode=mode)
        return time.perf_counter() - t

    nproc = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else os.cpu_count()
    try:
        os.sched_setaffinity(0, {sorted(os.sched_getaffinity(0))[0]})
    except (AttributeError, OSError):
        pass
    cpu_model = "unknown"
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                cpu_model = line.split(":", 1)[1].strip()
                break
    except OSError:
        pass
    out = {}
    for mode in ("exact", "f32step"):
        probe_P = 20000
        t_probe = max(run(probe_P, mode), 1e-4)
        P = int(min(wl.P, max(probe_P, probe_P * 8.0 / t_probe)))
        t = run(P, mode)
        full_call_s = t * wl.P / P
        out[mode] = (wl.U / full_call_s, wl.algorithmic_bytes_per_call() / full_call_s / 1e9, P, t)
    v, g, P, t = out["exact"]
    v32, g32, P32, t32 = out["f32step"]
    return {
        "value": v, "unit": "group-updates/s", "cores": 1, "kind": "oracle",
        "sample": f"exact-mode (fp64) oracle, one call of U={wl.U} updates on a contiguous slice of {P} of "
                  f"{wl.P} elements in {t:.2f} s, scaled by {wl.P / P:.1f}x (elements are independent)",
        "gbps": g,
        "f32step_value": v32, "f32step_gbps": g32,
        "f32step_sample": f"stepwise-fp32 oracle (state rounded to fp32 after every update), slice of {P32} elements "
                          f"in {t32:.2f} s, scaled by {wl.P / P32:.1f}x",
        "build": "gcc " + " ".join(so.BUILD_FLAGS), "cpu_model": cpu_model, "host_cpus": nproc,
    }


def main():
    a = parse()
    if a.gpus != 1:
        sys.stderr.write("bench.py: this build runs on one GPU; --gpus must be 1 "
                         "(the update shards by element across parameter-server GPUs, no multi-GPU path here)\n")
        sys.exit(2)
    import torch
    import paper_2512_09685_amd as star
    import workloads

    if not torch.cuda.is_available():
        sys.stderr.write("bench.py: no GPU visible\n")
        sys.exit(1)
    star.load_library()
    global KERNEL_OPTION
    KERNEL_OPTION = {"auto": None, "seq": star.KERNEL_SEQ, "affine": star.KERNEL_AFFINE,
                     "affine_mfma": star.KERNEL_AFFINE_MFMA}[a.kernel]
    import dataclasses
    wl_of = {n: (w if a.norms == "workload" else dataclasses.replace(w, norms=a.norms == "on"))
             for n, w in workloads.WORKLOADS.items()}
    if a.updates > 0:
        wl_of = {n: dataclasses.replace(w, U=a.updates) for n, w in wl_of.items()}
    head_wl = wl_of[a.workload]
    if a.copy_calibration:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
        torch.cuda.empty_cache()
    copy_gbps = device_copy_gbps(torch)
    head = measure(head_wl, a.steps, a.warmup, torch, star, workloads, a.op)
    per_config = []
    if not a.only:
        for name in workloads.ORDER:
            if name == a.workload:
                per_config.append(head)
            else:
                per_config.append(measure(wl_of[name], a.steps, a.warmup, torch, star, workloads, a.op))
    out = {
        "metric": "group_updates_per_s" if a.op != "reduce" else "group_aggregations_per_s",
        "value": head["group_updates_per_s"],
        "unit": "group-updates/s",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": head["ms_per_step"],
        "ms_per_step_median": head["ms_per_step_median"], "ms_per_step_min": head["ms_per_step_min"],
        "first_call_ms": head["first_call_ms"],
        "regime": "value, ms_per_step and roofline are steady state (calls back to back after 80 ms of wake-up work "
                  "and the warm-up steps); first_call_ms is one step after 250 ms of an idle device, median of 5",
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": a.workload, "op": a.op, "P": head_wl.P, "W": head_wl.W, "U": head_wl.U * head_wl.calls,
                   "grad_dtype": head_wl.grad_dtype, "norms": head_wl.norms, "kernel_choice": a.kernel},
        "hbm_gbps": head["hbm_gbps"],
        "roofline": {
            "bound": "hbm", "achieved": head["bytes_per_launch"] / (head["launch_ms"] * 1e-3) / 1e9,
            "peak": HBM_PEAK_GBPS, "unit": "GB/s",
            "frac": head["bytes_per_launch"] / (head["launch_ms"] * 1e-3) / 1e9 / HBM_PEAK_GBPS,
            "traffic": (measured_traffic(a.workload)
                        if a.op == "update" and a.norms == "workload" and a.kernel == "auto" and a.updates == 0
                        else None),
            "kernel": head["kernel"],
            "algorithmic_bytes_per_launch": head["bytes_per_launch"], "launch_ms": head["launch_ms"],
            "timed_launches": head["timed_launches"],
            "launches_after_timed": FIRST_CALL_REPS * head["calls_per_step"],
            "device_copy_gbps": copy_gbps,
            "frac_of_device_copy": head["bytes_per_launch"] / (head["launch_ms"] * 1e-3) / 1e9 / copy_gbps,
            "note": "launch duration = HIP-event time of the timed region / launches; it includes the two small "
                    "norm-finishing kernels that follow each update kernel",
        },
    }
    if not a.no_cpu:
        out["cpu_baseline"] = cpu_baseline(head_wl, torch, workloads)
    if per_config:
        out["per_config"] = per_config
    print(json.dumps(out))


if __name__ == "__main__":
    main()
