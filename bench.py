#!/usr/bin/env python3
"""Benchmark of the Two-Pass softmax hot path on one MI355X.

A step is one call of softmax2p_f32 (every pass of Algorithm 3) on the headline
workload, with the input already resident in HBM.  Prints ONE JSON line:

  value / unit     whole-job algorithmic bandwidth of the Two-Pass call in GB/s,
                   counting 3 N s bytes (Table 2: two reads and one write per element)
  roofline         the dominant kernel (pass 2: read x, write y = 2 N s bytes) timed
                   per launch with events on the launch stream, against 8 TB/s HBM
  cpu_baseline     the long-double oracle on the same input, on the host cores
  long_run         the headline call repeated for at least a second and 25 calls, every
                   call timed on its own: median and minimum (the protocol of Section 6.2)
  variants         Three-Pass baselines on the same input (4 N s and 5 N s bytes)
  parity           every variant's output on the headline input against the oracle
  calibration      read / fill / copy / scale streams at 1 GiB (the STREAM comparison of
                   Section 6.4)
  other_workloads  the remaining configurations, each with all variants

Every (workload, variant) entry says what its numbers mean: `algorithmic_bytes` (Table 2),
`hbm_bytes_measured` (rocprofv3 counters recorded in profiles/counters.json, or null),
`cache_assisted` (the memory side saw fewer bytes than the algorithm moves: a re-read was
served on chip), `frac_of_hbm_peak` (on the measured bytes when cache-assisted, else on the
algorithmic ones) and `frac_of_stream_copy` (the same byte rate over that of the library's plain
copy of an array of the same size, timed in the same run on the same buffers).

Usage: python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg4] [--quick]
       python bench.py --workload cfg5 --calls-only softmax2p,copy     (profiler target)
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
# algorithmic bytes per element in units of the element size (Table 2); the on-chip variants
# read x from memory once and are therefore counted with 2, not 3
BYTES_PER_ELEM = {"softmax2p": 3, "softmax3p_recompute": 4, "softmax3p_reload": 5,
                  "softmax2p_onchip": 2, "softmax3p_onchip": 2}
# 256 compute units x 4 SIMDs x 16 lanes x 2.4 GHz, one fp32 operation per lane and clock
# (packed fp32 arithmetic is not used)
VALU_PEAK_TOPS = 256 * 4 * 16 * 2.4e9 / 1e12
WAKEUP_S = 0.25
LONG_RUN_MIN_S = 1.0
LONG_RUN_MIN_CALLS = 25
COUNTERS_JSON = os.path.join(ROOT, "profiles", "counters.json")


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def _events(torch, k):
    return [torch.cuda.Event(enable_timing=True) for _ in range(k)]


def time_calls(torch, fn, steps, warmup, sets):
    """Wall-clock and event time of `steps` calls of fn(set_index), rotating over buffer sets."""
    for i in range(warmup):
        fn(i % sets)
    torch.cuda.synchronize()
    e0, e1 = _events(torch, 2)
    t0 = time.perf_counter()
    e0.record()
    for i in range(steps):
        fn(i % sets)
    e1.record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    return (t1 - t0) * 1e3 / steps, e0.elapsed_time(e1) / steps


def wake_up(torch, fn, sets):
    """Untimed: keeps the GPU busy for WAKEUP_S seconds before the first measurement.  The
    host spends seconds generating the input while the device idles and drops its clocks; the
    few warm-up steps of a sub-millisecond call do not bring them back up."""
    t0 = time.perf_counter()
    i = 0
    while time.perf_counter() - t0 < WAKEUP_S:
        for _ in range(20):
            fn(i % sets)
            i += 1
        torch.cuda.synchronize()


def per_launch_ms(torch, fn, steps, sets, group=1):
    """Average duration of one launch of fn.  `group` consecutive launches are bracketed by one pair of
    events recorded on the stream the kernels run on (torch's current stream); with group = 1 every
    launch has its own pair and the figure includes the few microseconds an event pair costs."""
    groups = max(steps // group, 3)
    evs = [_events(torch, 2) for _ in range(groups)]
    torch.cuda.synchronize()
    k = 0
    for g in range(groups):
        evs[g][0].record()
        for _ in range(group):
            fn(k % sets)
            k += 1
        evs[g][1].record()
    torch.cuda.synchronize()
    ts = sorted(a.elapsed_time(b) / group for a, b in evs)
    return sum(ts) / len(ts), ts[len(ts) // 2], ts[0]


def long_run(torch, fn, sets):
    """Section 6.2 repeats a measurement until it is stable and reports the median.  Here: the
    call is repeated, every call between its own pair of events, in batches of 25 until at least
    LONG_RUN_MIN_S seconds of wall time and LONG_RUN_MIN_CALLS calls have gone by."""
    times = []
    t0 = time.perf_counter()
    k = 0
    while time.perf_counter() - t0 < LONG_RUN_MIN_S or len(times) < LONG_RUN_MIN_CALLS:
        evs = [_events(torch, 2) for _ in range(25)]
        for a, b in evs:
            a.record()
            fn(k % sets)
            b.record()
            k += 1
        torch.cuda.synchronize()
        times += [a.elapsed_time(b) for a, b in evs]
    wall = time.perf_counter() - t0
    ts = sorted(times)
    return {"calls": len(ts), "wall_s": wall, "ms_median": ts[len(ts) // 2], "ms_min": ts[0],
            "ms_mean": sum(ts) / len(ts), "ms_p90": ts[int(len(ts) * 0.9)],
            "timing": "one event pair per call on the launch stream"}


def load_counters():
    """Counter figures recorded from rocprofv3 runs of this file (profiles/counters.json, written
    by paper_2001_04438_amd/prof_summary.py), or {} if none has been recorded."""
    try:
        with open(COUNTERS_JSON) as f:
            return json.load(f)
    except (OSError, ValueError):
        return {}


def traffic_of(counters, workload, variant):
    return counters.get("workloads", {}).get(workload, {}).get(variant)


def describe_variant(entry, alg_bytes, wall_ms, copy_ms, copy_bytes, rec):
    """Adds the fields that say what a variant's byte rate means (see the module docstring)."""
    measured = rec.get("hbm_bytes") if rec else None
    assisted = None if measured is None else bool(measured < 0.95 * alg_bytes)
    effective = measured if assisted else alg_bytes
    rate = effective / wall_ms / 1e6
    entry["algorithmic_bytes"] = alg_bytes
    entry["GBps_algorithmic"] = alg_bytes / wall_ms / 1e6
    entry["hbm_bytes_measured"] = measured
    entry["cache_assisted"] = assisted
    entry["GBps_effective"] = rate
    if rate <= HBM_PEAK_GBS:
        entry["frac_of_hbm_peak"] = rate / HBM_PEAK_GBS
    else:  # only possible when no counter record exists for a variant whose re-reads stay on chip
        entry["frac_of_hbm_peak"] = None
        entry["frac_of_hbm_peak_note"] = ("algorithmic bytes over time exceed the HBM peak: part of them "
                                          "never left the chip and no counter record says how many")
    entry["frac_of_stream_copy"] = rate / (copy_bytes / copy_ms / 1e6)
    return entry


def run_workload(torch, B, W, name, steps, warmup, full, counters):
    import numpy as np

    # "<cfg>_f16": the same values stored as IEEE binary16 instead of the workload's own format
    base, f16 = (name[:-4], True) if name.endswith("_f16") else (name, False)
    rows, n = W.SHAPES[base]
    bf16 = W.DTYPES[base] == "bf16" and not f16
    fmt = "f16" if f16 else "bf16" if bf16 else "f32"
    s = 4 if fmt == "f32" else 2
    t0 = time.perf_counter()
    x_host = W.make(base)
    if f16:
        vals = W.bf16_bits_to_f32(x_host) if W.DTYPES[base] == "bf16" else x_host
        x_host = W.f32_to_f16_bits(vals).reshape(rows, n)
    log(f"[bench] {name}: generated {rows}x{n} {fmt} in {time.perf_counter() - t0:.1f}s")
    flat = x_host.reshape(-1)
    host_t = torch.from_numpy(flat.view(np.int16) if s == 2 else flat)
    footprint = 2 * flat.size * s
    sets = 1 if footprint >= (1 << 30) else int(min(8, -(-(1 << 30) // footprint)))
    xs = [host_t.cuda() for _ in range(sets)]
    ys = [torch.empty_like(xs[0]) for _ in range(sets)]
    elems = rows * n
    plan = B.softmax_tp_plan(rows, n, s, True)
    out = {"rows": rows, "n": n, "dtype": fmt, "buffer_sets": sets,
           "plan": plan.as_dict(), "variants": {}}

    suffix = {"f32": "_f32", "bf16": "_bf16io", "f16": "_f16io"}[fmt]
    variants = [("softmax2p", getattr(B, "softmax2p" + suffix)),
                ("softmax3p_recompute", getattr(B, "softmax3p_recompute" + suffix)),
                ("softmax3p_reload", getattr(B, "softmax3p_reload" + suffix))]
    if n <= 32768:  # short rows: also the variants that keep the row in registers
        variants += [("softmax2p_onchip", getattr(B, "softmax2p_onchip" + suffix)),
                     ("softmax3p_onchip", getattr(B, "softmax3p_onchip" + suffix))]
    wake_up(torch, lambda i: variants[0][1](xs[i], ys[i], rows, n), sets)
    # the plain copy of an array of this size, same buffers, same rotation: the ceiling every
    # variant's byte rate is set against (the paper compares with STREAM the same way, Section 6.4)
    words = elems * s // 4
    copy = lambda i: B.softmax_tp_stream_copy_f32(xs[i].data_ptr(), ys[i].data_ptr(), words)
    copy_ms, _ = time_calls(torch, copy, steps, warmup, sets)
    copy_bytes = 2 * words * 4
    out["stream_copy_same_size"] = {"ms_per_step": copy_ms, "bytes": copy_bytes,
                                    "GBps": copy_bytes / copy_ms / 1e6,
                                    "frac_of_hbm_peak": copy_bytes / copy_ms / 1e6 / HBM_PEAK_GBS}
    log(f"[bench] {name} stream copy of the same size: {copy_ms:.4f} ms/step, {copy_bytes / copy_ms / 1e6:.0f} GB/s")
    for vname, fn in variants:
        call = lambda i, fn=fn: fn(xs[i], ys[i], rows, n)
        wall_ms, ev_ms = time_calls(torch, call, steps, warmup, sets)
        # the protocol of Section 6.2 reports a median over repetitions: per-call event times,
        # cold (rotating buffer sets) and warm (the same buffers every call)
        _, med_ms, min_ms = per_launch_ms(torch, call, max(steps, 25), sets)
        _, warm_med_ms, _ = per_launch_ms(torch, lambda i, fn=fn: fn(xs[0], ys[0], rows, n),
                                          max(steps, 25), 1)
        alg_bytes = BYTES_PER_ELEM[vname] * elems * s
        entry = {"ms_per_step": wall_ms, "ms_per_step_events": ev_ms,
                 "ms_per_call_median": med_ms, "ms_per_call_min": min_ms,
                 "ms_per_call_median_warm": warm_med_ms,
                 "elements_per_s": elems / wall_ms * 1e3}
        out["variants"][vname] = describe_variant(entry, alg_bytes, wall_ms, copy_ms, copy_bytes,
                                                  traffic_of(counters, name, vname))
        log(f"[bench] {name} {vname}: {wall_ms:.4f} ms/step, {alg_bytes / wall_ms / 1e6:.0f} GB/s algorithmic, "
            f"{entry['frac_of_stream_copy']:.3f} of the same-size copy")

    # dominant kernel, one launch at a time
    if plan.path == 2 and fmt == "f32":
        pairs = torch.empty(2 * rows, dtype=torch.float32, device="cuda")
        B.softmax2p_f32_pass1(xs[0], pairs, rows, n)
        # eight launches per event pair: the cost of the pair itself is spread thin, so the figure
        # is the kernel's duration plus the gap between two launches
        p1 = per_launch_ms(torch, lambda i: B.softmax2p_f32_pass1(xs[i], pairs, rows, n), steps, sets, 8)
        p2 = per_launch_ms(torch, lambda i: B.softmax2p_f32_pass2(xs[i], pairs, ys[i], rows, n),
                           steps, sets, 8)
        out["pass1_ms"] = {"avg": p1[0], "median": p1[1], "min": p1[2], "bytes": elems * s}
        out["pass2_ms"] = {"avg": p2[0], "median": p2[1], "min": p2[2], "bytes": 2 * elems * s}
        dom_name, dom_ms, dom_bytes = "chunk_2p_pass2", p2[0], 2 * elems * s
    else:
        fn = variants[0][1]
        k = per_launch_ms(torch, lambda i: fn(xs[i], ys[i], rows, n), steps, sets)
        out["kernel_ms"] = {"avg": k[0], "median": k[1], "min": k[2]}
        dom_name, dom_ms, dom_bytes = "rows_2p", k[0], 3 * elems * s
    rec = traffic_of(counters, name, "softmax2p") or {}
    krec = rec.get("kernels", {}).get(dom_name, {})
    out["dominant"] = {"kernel": dom_name, "avg_ms": dom_ms, "algorithmic_bytes": dom_bytes,
                       "GBps": dom_bytes / dom_ms / 1e6, "traffic_bytes": krec.get("hbm_bytes")}
    if s == 2 and plan.path == 1 and krec.get("valu_lane_ops_per_element"):
        # rows of 16-bit elements are bound by vector arithmetic, not by memory
        per_elem = krec["valu_lane_ops_per_element"]
        ops = per_elem * elems
        out["alu_roofline"] = {"bound": "alu", "kernel": dom_name, "lane_ops_per_element": per_elem,
                               "lane_ops_source": "SQ_INSTS_VALU x 64 / elements, recorded in profiles/counters.json",
                               "achieved": ops / dom_ms / 1e9, "peak": VALU_PEAK_TOPS,
                               "unit": "T lane-operations/s", "frac": ops / dom_ms / 1e9 / VALU_PEAK_TOPS}
    torch.cuda.synchronize()
    y_hosts = {}
    if full:
        for vname, fn in variants:
            fn(xs[0], ys[0], rows, n)
            torch.cuda.synchronize()
            y = ys[0].cpu().numpy()
            if s == 2:
                y = y.view(np.uint16)
            y_hosts[vname] = y.reshape(rows, n).copy()
        out["long_run"] = long_run(torch, lambda i: variants[0][1](xs[i], ys[i], rows, n), sets)
        log(f"[bench] {name} softmax2p long run: {out['long_run']['calls']} calls, median "
            f"{out['long_run']['ms_median']:.4f} ms, min {out['long_run']['ms_min']:.4f} ms")
    del xs, ys
    torch.cuda.empty_cache()
    return out, x_host, y_hosts


def calls_only(torch, B, W, name, variants, steps, warmup):
    """Profiler target: nothing but the named calls on the named workload.  A
    one-workgroup ExtExp launch goes before each variant's calls so that a counter file can be cut
    into variants by that kernel's name."""
    import numpy as np
    base, f16 = (name[:-4], True) if name.endswith("_f16") else (name, False)
    rows, n = W.SHAPES[base]
    x_host = W.make(base)
    if f16:
        vals = W.bf16_bits_to_f32(x_host) if W.DTYPES[base] == "bf16" else x_host
        x_host = W.f32_to_f16_bits(vals).reshape(rows, n)
    fmt = "f16" if f16 else W.DTYPES[base]
    flat = x_host.reshape(-1)
    host_t = torch.from_numpy(flat.view(np.int16) if fmt != "f32" else flat)
    es = 4 if fmt == "f32" else 2
    footprint = 2 * flat.size * es
    # as in the timed runs: rotate over enough buffer sets to exceed 1 GiB, so no call finds its
    # input in the 256 MB memory-side cache
    sets = 1 if footprint >= (1 << 30) else int(min(8, -(-(1 << 30) // footprint)))
    xs = [host_t.cuda() for _ in range(sets)]
    ys = [torch.empty_like(xs[0]) for _ in range(sets)]
    words = rows * n * es // 4
    mark = torch.zeros(3 * 64, dtype=torch.float32, device="cuda")
    sink = torch.zeros(1, dtype=torch.float32, device="cuda")
    suffix = {"f32": "_f32", "bf16": "_bf16io", "f16": "_f16io"}[fmt]
    out = {}
    torch.cuda.synchronize()
    for v in variants:
        if v == "copy":     # the same bytes as fp32 words
            fn = lambda i: B.softmax_tp_stream_copy_f32(xs[i].data_ptr(), ys[i].data_ptr(), words)
        elif v == "read":
            fn = lambda i: B.softmax_tp_stream_read_f32(xs[i].data_ptr(), sink, words)
        else:
            fn = lambda i, f=getattr(B, v + suffix): f(xs[i], ys[i], rows, n)
        B.softmax_tp_extexp_f32(mark[:64], mark[64:128], mark[128:], 64)
        for k in range(warmup):
            fn(k % sets)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for k in range(steps):
            fn((warmup + k) % sets)
        torch.cuda.synchronize()
        out[v] = (time.perf_counter() - t0) * 1e3 / steps
        log(f"[bench] {name} {v}: {out[v]:.4f} ms per call ({steps} calls, {sets} buffer sets)")
    B.softmax_tp_release()
    print(json.dumps({"workload": name, "rows": rows, "n": n, "dtype": fmt, "calls": steps + warmup,
                      "variants": variants, "ms_per_call": out}))


def calibration(torch, B, steps, warmup):
    n = 1 << 28
    x = torch.rand(n, dtype=torch.float32, device="cuda")
    y = torch.empty_like(x)
    sink = torch.zeros(1, dtype=torch.float32, device="cuda")
    res = {}
    for name, fn, nbytes in (
            ("read", lambda i: B.softmax_tp_stream_read_f32(x, sink, n), 4 * n),
            ("fill", lambda i: B.softmax_tp_stream_fill_f32(y, 0.5, n), 4 * n),
            ("copy", lambda i: B.softmax_tp_stream_copy_f32(x, y, n), 8 * n),
            ("scale", lambda i: B.softmax_tp_stream_scale_f32(x, y, 0.5, n), 8 * n)):
        for i in range(warmup):
            fn(0)
        avg, med, mn = per_launch_ms(torch, fn, steps, 1, 8)
        res[name] = {"ms": avg, "GBps": nbytes / avg / 1e6, "frac_of_hbm_peak": nbytes / avg / 1e6 / HBM_PEAK_GBS}
        log(f"[bench] stream_{name} 1 GiB: {avg:.4f} ms, {nbytes / avg / 1e6:.0f} GB/s")
    return res


def cpu_model():
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(x_host, y_hosts, fmt, tol):
    """Times the oracle as it stands on the host cores and checks every variant's GPU output with it."""
    import oracle
    kw = {"bf16": fmt == "bf16", "f16": fmt == "f16"}
    cores = oracle.threads_available()
    t0 = time.perf_counter()
    oracle.stats(x_host, **kw)
    t_stats = time.perf_counter() - t0
    # softmax = statistics pass + one exp and one division per element: the comparator does
    # exactly that work (plus the comparison), so its time stands for a full oracle softmax.
    t0 = time.perf_counter()
    cmp_ = oracle.compare(x_host, y_hosts["softmax2p"], tol, **kw)  # recomputes mu, S, then every p_i
    t_cmp = time.perf_counter() - t0
    parity = {}
    for vname, y in y_hosts.items():
        three = vname.startswith("softmax3p") and fmt == "f32"
        # Three-Pass on fp32: fl32(x - mu) alone costs up to 2^-24 |x - mu|, hence the per-element bound
        slope = oracle.THREE_PASS_SLOPE if three else 0.0
        c = cmp_ if vname == "softmax2p" else oracle.compare(x_host, y, tol, slope=slope, **kw)
        parity[vname] = {"max_rel_err": c.max_rel_err, "ok": bool(c.ok()),
                         "bound": f"{tol:g} + 2^-24 |x_i - mu|" if three else f"{tol:g}",
                         "max_err_over_bound": c.max_bound_ratio, "max_row_sum_dev": c.max_row_sum_dev,
                         "results_in_normal_range": c.n_normal}
    # Single-thread figure on a prefix of the same data (2^22 elements of the first row).
    rows, n = x_host.shape
    m1 = min(n, 1 << 22)
    xs, ys = x_host[:1, :m1], y_hosts["softmax2p"][:1, :m1]
    t0 = time.perf_counter()
    oracle.compare(xs, ys, 1.0, threads=1, **kw)
    t_one = time.perf_counter() - t0
    return cores, t_stats, t_cmp, parity, m1 / t_one


VARIANT_KEYS = ("ms_per_step", "ms_per_call_median", "ms_per_call_min", "ms_per_call_median_warm",
                "elements_per_s", "algorithmic_bytes", "GBps_algorithmic", "hbm_bytes_measured",
                "cache_assisted", "GBps_effective", "frac_of_hbm_peak", "frac_of_hbm_peak_note",
                "frac_of_stream_copy")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="cfg4", choices=["cfg2", "cfg3", "cfg4", "cfg5", "cfg5_f16"])
    ap.add_argument("--quick", action="store_true", help="headline workload only")
    ap.add_argument("--calls-only", default="", metavar="VARIANT[,VARIANT...]",
                    help="for profiler runs: generate the workload, make --warmup + --steps calls of each "
                         "named variant (softmax2p, softmax3p_recompute, softmax3p_reload, softmax2p_onchip, "
                         "softmax3p_onchip, copy, read) and exit; no oracle, no other workload")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)")

    import torch
    from paper_2001_04438_amd import binding as B
    from paper_2001_04438_amd import workloads as W

    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    B.lib()  # fails loudly if the HIP library is not built
    torch.cuda.set_device(0)
    props = torch.cuda.get_device_properties(0)
    log(f"[bench] device: {props.name}, {props.multi_processor_count} CUs")

    if args.calls_only:
        calls_only(torch, B, W, args.workload, args.calls_only.split(","), args.steps, args.warmup)
        return

    counters = load_counters()
    head, x_host, y_hosts = run_workload(torch, B, W, args.workload, args.steps, args.warmup, True, counters)
    fmt = head["dtype"]
    tol = {"f32": 4e-6, "bf16": 1e-2, "f16": 5e-4}[fmt]
    cores, t_stats, t_cmp, parity, one_thread_eps = cpu_baseline(x_host, y_hosts, fmt, tol)
    log(f"[bench] oracle on {cores} threads: stats {t_stats:.2f}s, softmax+compare {t_cmp:.2f}s; "
        + "; ".join(f"{k} max_rel_err={v['max_rel_err']:.3e} ok={v['ok']}" for k, v in parity.items()))
    del x_host, y_hosts

    two = head["variants"]["softmax2p"]
    s = 4 if fmt == "f32" else 2
    elems = head["rows"] * head["n"]
    dom = head["dominant"]
    meta = counters.get("_meta", {})
    result = {
        "metric": "softmax GB/s and elements/s per MI355X; % of HBM peak; 2-pass vs 3-pass",
        "value": two["GBps_algorithmic"],
        "unit": "GB/s (Two-Pass softmax, algorithmic bytes 3*N*s per call)",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": two["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32" if fmt == "f32" else f"f32 ({fmt} storage)",
        "data": "synthetic",
        "config": {"workload": f"{args.workload}: {head['rows']} x {head['n']} {head['dtype']}",
                   "plan": head["plan"], "buffer_sets": head["buffer_sets"],
                   "device_wakeup_s_before_warmup": WAKEUP_S},
        "elements_per_s": two["elements_per_s"],
        "frac_of_hbm_peak": two["frac_of_hbm_peak"],
        "cache_assisted": two["cache_assisted"],
        "frac_of_stream_copy": two["frac_of_stream_copy"],
        "roofline": {
            "bound": "hbm", "kernel": dom["kernel"],
            "achieved": dom["GBps"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": dom["GBps"] / HBM_PEAK_GBS,
            "algorithmic_bytes_per_launch": dom["algorithmic_bytes"],
            "avg_launch_ms": dom["avg_ms"],
            "traffic": dom["traffic_bytes"],
            "traffic_source": ("not measured in this run: recorded in profiles/counters.json from rocprofv3 "
                               "--pmc runs of this file" + (f" at commit {meta['commit']}" if meta.get("commit") else "")
                               + "; bytes = 128 x TCC_EA0_RDREQ_128B + 64 x 64-byte + 32 x 32-byte read requests "
                                 "+ WRITE_SIZE, see profiles/"),
        },
        "cpu_baseline": {
            "value": 3 * elems * s / t_cmp / 1e9, "unit": "GB/s (same 3*N*s byte count)",
            "elements_per_s": elems / t_cmp, "seconds": t_cmp, "cores": cores, "kind": "oracle",
            "cpu": cpu_model(), "single_thread_elements_per_s": one_thread_eps,
            "sample": f"the whole {args.workload} input, one oracle softmax fused with the comparison "
                      f"of the GPU output (statistics pass alone: {t_stats:.2f}s)",
        },
        "parity": parity,
        "long_run": head["long_run"],
        "stream_copy_same_size": head["stream_copy_same_size"],
        "variants": {k: {kk: v[kk] for kk in VARIANT_KEYS if kk in v} for k, v in head["variants"].items()},
        "passes": {k: head[k] for k in ("pass1_ms", "pass2_ms", "kernel_ms") if k in head},
    }
    if "alu_roofline" in head:
        result["alu_roofline"] = head["alu_roofline"]
    if "softmax3p_recompute" in head["variants"]:
        result["two_pass_speedup"] = {
            "vs_recompute": head["variants"]["softmax3p_recompute"]["ms_per_step"] / two["ms_per_step"],
            "vs_reload": head["variants"]["softmax3p_reload"]["ms_per_step"] / two["ms_per_step"]}
    if not args.quick:
        cal = calibration(torch, B, args.steps, args.warmup)
        result["calibration"] = cal
        if "pass2_ms" in head and elems * s == 1 << 30:
            # each pass next to the plain stream of its kind at the same size (1 GiB), as the paper
            # sets its passes next to STREAM Copy / Scale (Section 6.4)
            result["vs_calibration"] = {
                "pass1_over_stream_read": cal["read"]["ms"] / head["pass1_ms"]["avg"],
                "pass2_over_stream_copy": cal["copy"]["ms"] / head["pass2_ms"]["avg"],
                # reads and writes do not overlap in the memory system: a copy takes as long as the
                # read-only and the write-only stream of its size one after the other
                "copy_over_read_plus_fill": cal["copy"]["ms"] / (cal["read"]["ms"] + cal["fill"]["ms"]),
                "call_over_read_plus_copy": (cal["read"]["ms"] + cal["copy"]["ms"]) / two["ms_per_step"]}
        others = {}
        for name in ("cfg2", "cfg3", "cfg4", "cfg5", "cfg5_f16"):
            if name == args.workload:
                continue
            # these calls take 50 to 200 us: at least 100 timed steps each, whatever --steps says
            o, _, _ = run_workload(torch, B, W, name, max(args.steps, 100), max(args.warmup, 10), False,
                                   counters)
            others[name] = {
                "shape": f"{o['rows']} x {o['n']} {o['dtype']}", "path": o["plan"]["path"],
                "buffer_sets": o["buffer_sets"],
                "stream_copy_same_size": o["stream_copy_same_size"],
                "variants": {k: {kk: v[kk] for kk in VARIANT_KEYS if kk in v}
                             for k, v in o["variants"].items()},
                "dominant": o["dominant"]}
            if "alu_roofline" in o:
                others[name]["alu_roofline"] = o["alu_roofline"]
        result["other_workloads"] = others
    B.softmax_tp_release()
    print(json.dumps(result))


if __name__ == "__main__":
    main()
