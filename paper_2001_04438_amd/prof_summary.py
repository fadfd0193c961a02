"""Turns rocprofv3 output of `bench.py --calls-only` runs into the summaries under profiles/.

Each profiled run is `rocprofv3 <options> --output-format csv -d DIR/<workload>.<set> --
python3 bench.py --workload <workload> --calls-only <variants> --steps S --warmup W`, its standard
output saved as DIR/<workload>.<set>.json.  The sets this script knows:

  trace  --kernel-trace --stats                         kernel durations
  rd     --pmc TCC_EA0_RDREQ_sum TCC_EA0_RDREQ_32B_sum TCC_EA0_RDREQ_64B_sum TCC_EA0_RDREQ_128B_sum
         read requests L2 -> memory fabric by size: bytes read = 32 a + 64 b + 128 c
  wr     --pmc WRITE_SIZE                               KiB written L2 -> memory fabric
  sq     --pmc SQ_INSTS_VALU SQ_WAVES SQ_BUSY_CYCLES SQ_WAVE_CYCLES SQ_ACTIVE_INST_VALU
         SQ_INSTS_VMEM_RD SQ_INSTS_VMEM_WR GRBM_GUI_ACTIVE
  m1..m4 memory-side counters (headline workload only), named in MEMORY_SETS below

`bench.py --calls-only` launches a one-workgroup ExtExp kernel before the calls of each variant;
the dispatch list is cut into variants at those markers, so kernels that several variants share
(chunk_max, the merges) are attributed correctly.  Writes

  profiles/counters.json                   what bench.py reads: HBM-side bytes per call and per
                                           kernel launch, VALU lane-operations per element
  profiles/kernels_all_workloads.md        durations, bytes, VALU counts of every kernel
  profiles/chunk_2p_pass2_cfg4.md          the dominant kernel of the headline workload
  profiles/memory_side_cfg4.md             the memory-side counters of the 1 GiB streams
  profiles/bench_kernel_trace.md           kernel durations of the default bench.py run (if DIR/bench.trace,
                                           made by `rocprofv3 --kernel-trace --stats ... -- python3 bench.py
                                           --steps 20 --warmup 5 > DIR/bench.trace.json`, is there)

    python -m paper_2001_04438_amd.prof_summary DIR [--commit HASH]
"""
from __future__ import annotations

import argparse
import collections
import csv
import glob
import json
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PROFILES = os.path.join(ROOT, "profiles")
MARKER = "extexp_kernel"
WORKLOADS = ("cfg2", "cfg3", "cfg4", "cfg5", "cfg5_f16")
ELEM_BYTES = {"f32": 4, "bf16": 2, "f16": 2}
BYTES_PER_ELEM = {"softmax2p": 3, "softmax3p_recompute": 4, "softmax3p_reload": 5,
                  "softmax2p_onchip": 2, "softmax3p_onchip": 2, "copy": 2, "read": 1}
SQ_SET = ("SQ_INSTS_VALU SQ_WAVES SQ_BUSY_CYCLES SQ_WAVE_CYCLES SQ_ACTIVE_INST_VALU "
          "SQ_INSTS_VMEM_RD SQ_INSTS_VMEM_WR GRBM_GUI_ACTIVE")
RD_SET = "TCC_EA0_RDREQ_sum TCC_EA0_RDREQ_32B_sum TCC_EA0_RDREQ_64B_sum TCC_EA0_RDREQ_128B_sum"
MEMORY_SETS = {
    "m1": "TCC_EA0_RDREQ_sum TCC_EA0_RDREQ_LEVEL_sum TCC_EA0_WRREQ_sum TCC_EA0_WRREQ_LEVEL_sum",
    "m2": "TCC_EA0_RDREQ_DRAM_CREDIT_STALL_sum TCC_EA0_WRREQ_DRAM_CREDIT_STALL_sum TCC_EA0_WRREQ_STALL_sum "
          "TCC_TOO_MANY_EA_WRREQS_STALL_sum",
    "m3": "TCC_BUSY_sum TCC_CYCLE_sum TCC_TAG_STALL_sum TCC_REQ_sum",
    "m4": "TCP_PENDING_STALL_CYCLES_sum TCP_TCR_TCP_STALL_CYCLES_sum TCP_TCC_READ_REQ_LATENCY_sum "
          "TCP_TCC_READ_REQ_sum",
}


def short(name: str) -> str:
    """tp::chunk_2p_pass2<tp::F32x4, 128, 1>(...) -> chunk_2p_pass2<F32x4, 128, 1>"""
    name = name.replace("void ", "").replace("tp::", "")
    depth = 0
    for i, ch in enumerate(name):
        depth += ch == "<"
        depth -= ch == ">"
        if ch == "(" and depth == 0:
            return name[:i]
    return name


def base(name: str) -> str:
    return short(name).split("<")[0]


def newest(pattern):
    """Files matching the pattern, most recently written first (a directory that several profiler
    runs wrote into holds one file per run, named after the process)."""
    return sorted(glob.glob(pattern, recursive=True), key=os.path.getmtime, reverse=True)


def read_run(root, workload, kind):
    """-> (info from the run's JSON line, dispatch list in launch order).  A dispatch is
    {"kernel", "grid", "block", "us", counters...}; None if the run is missing."""
    d = os.path.join(root, f"{workload}.{kind}")
    meta = os.path.join(root, f"{workload}.{kind}.json")
    if not os.path.isdir(d) or not os.path.exists(meta):
        return None
    info = None
    for line in open(meta):
        line = line.strip()
        if line.startswith("{"):
            info = json.loads(line)
    if info is None:
        return None
    files = newest(os.path.join(d, "**", "*_counter_collection.csv")) or \
        newest(os.path.join(d, "**", "*_kernel_trace.csv"))
    if not files:
        return None
    disp = collections.OrderedDict()
    for r in csv.DictReader(open(files[0])):
        key = int(r.get("Dispatch_Id") or r["Correlation_Id"])
        e = disp.setdefault(key, {"kernel": r["Kernel_Name"]})
        e["us"] = (int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3
        if "Counter_Name" in r:
            e["grid"] = int(r["Grid_Size"])
            e["block"] = int(r["Workgroup_Size"])
            e[r["Counter_Name"]] = e.get(r["Counter_Name"], 0.0) + float(r["Counter_Value"])
        else:
            e["grid"] = int(r["Grid_Size_X"])
            e["block"] = int(r["Workgroup_Size_X"])
    return info, [disp[k] for k in sorted(disp)]


def by_variant(info, dispatches):
    """Cuts the dispatch list at the marker kernel: -> {variant: [dispatch, ...]} (library kernels only)."""
    out, cur, names = {}, None, list(info["variants"])
    for d in dispatches:
        if MARKER in d["kernel"]:
            cur = names.pop(0) if names else None
            out[cur] = []
        elif cur is not None and "tp::" in d["kernel"]:
            out[cur].append(d)
    return out


def per_kernel(dispatches, calls, fields):
    """Groups one variant's dispatches by kernel: launches per call, averages per launch."""
    groups = collections.OrderedDict()
    for d in dispatches:
        groups.setdefault(short(d["kernel"]), []).append(d)
    res = collections.OrderedDict()
    for k, ds in groups.items():
        us = sorted(d["us"] for d in ds)
        e = {"launches_per_call": len(ds) / calls, "grid_threads": ds[0]["grid"], "block": ds[0]["block"],
             "us_avg": sum(us) / len(us), "us_med": us[len(us) // 2], "us_min": us[0], "us_max": us[-1],
             "dispatches": len(ds)}
        for f in fields:
            vals = [d[f] for d in ds if f in d]
            if vals:
                e[f] = sum(vals) / len(vals)
        res[k] = e
    return res


def collect(root):
    data = {}
    for w in WORKLOADS:
        wl = {}
        for kind, fields in (("trace", ()), ("rd", RD_SET.split()), ("wr", ("WRITE_SIZE",)),
                             ("sq", SQ_SET.split())) + tuple((m, c.split()) for m, c in MEMORY_SETS.items()):
            run = read_run(root, w, kind)
            if run is None:
                continue
            info, disp = run
            wl.setdefault("info", info)
            for variant, ds in by_variant(info, disp).items():
                wl.setdefault("variants", collections.OrderedDict()).setdefault(variant, {})[kind] = \
                    per_kernel(ds, info["calls"], fields)
        if wl:
            data[w] = wl
    return data


def read_bytes(k):
    return 32 * k.get("TCC_EA0_RDREQ_32B_sum", 0) + 64 * k.get("TCC_EA0_RDREQ_64B_sum", 0) + \
        128 * k.get("TCC_EA0_RDREQ_128B_sum", 0)


def build_counters(data, commit, root):
    out = {"_meta": {
        "commit": commit,
        "made_by": "python -m paper_2001_04438_amd.prof_summary " + os.path.relpath(root, ROOT),
        "source": "rocprofv3 --pmc runs of `bench.py --workload W --calls-only ...`; commands in "
                  "profiles/kernels_all_workloads.md",
        "read_bytes": "32 x TCC_EA0_RDREQ_32B + 64 x TCC_EA0_RDREQ_64B + 128 x TCC_EA0_RDREQ_128B (requests "
                      "from L2 to the memory fabric, summed over channels); no calibration factor",
        "write_bytes": "WRITE_SIZE x 1024",
        "note": "bytes are what left the L2 caches: hits in the 256 MB memory-side cache are not visible here",
    }, "workloads": {}}
    for w, wl in data.items():
        info = wl["info"]
        elems = info["rows"] * info["n"]
        ow = out["workloads"].setdefault(w, {})
        for variant, kinds in wl.get("variants", {}).items():
            if variant in ("copy", "read"):
                name = "stream_" + variant
            else:
                name = variant
            kernels = collections.OrderedDict()
            tot_r = tot_w = 0.0
            have = "rd" in kinds and "wr" in kinds
            for kname in (kinds.get("rd") or kinds.get("sq") or kinds.get("trace") or {}):
                e = {}
                if have and kname in kinds["wr"]:
                    rb = read_bytes(kinds["rd"][kname])
                    wb = kinds["wr"][kname].get("WRITE_SIZE", 0) * 1024
                    lp = kinds["rd"][kname]["launches_per_call"]
                    e.update(fetch_bytes=round(rb), write_bytes=round(wb), hbm_bytes=round(rb + wb),
                             launches_per_call=lp)
                    tot_r += rb * lp
                    tot_w += wb * lp
                if "sq" in kinds and kname in kinds["sq"]:
                    v = kinds["sq"][kname].get("SQ_INSTS_VALU")
                    if v is not None:
                        e["valu_wave_instructions"] = round(v)
                        # every launch of these kernels covers all rows * n elements once
                        e["valu_lane_ops_per_element"] = round(v * 64 / elems, 2)
                if "trace" in kinds and kname in kinds["trace"]:
                    e["us_avg_kernel_trace"] = round(kinds["trace"][kname]["us_avg"], 2)
                b = base(kname)
                if b in kernels:   # two instantiations of one kernel in a call: keep both under full names
                    kernels[kname] = e
                else:
                    kernels[b] = dict(e, instantiation=kname)
            rec = {"kernels": kernels}
            if have:
                rec.update(fetch_bytes=round(tot_r), write_bytes=round(tot_w), hbm_bytes=round(tot_r + tot_w))
            ow[name] = rec
    return out


def fmt_int(v):
    return f"{v:,.0f}"


def write_kernels_md(data, counters, root, path):
    L = []
    L.append("# rocprofv3 summary: every kernel of every softmax variant, all workloads (MI355X, gfx950)\n")
    L.append("Made by `python -m paper_2001_04438_amd.prof_summary` from these runs (from `/tmp` with "
             "`TMPDIR=/tmp`; `$R` is the repository root, `$W` one of cfg2, cfg3, cfg4, cfg5, cfg5_f16, `$V` the "
             "variants of that workload: `softmax2p,softmax3p_recompute,softmax3p_reload,copy,read`, on the "
             "workloads with short rows also `softmax2p_onchip,softmax3p_onchip`):\n")
    L.append("```")
    L.append("rocprofv3 --kernel-trace --stats --output-format csv -d $D/$W.trace -- python3 $R/bench.py --workload $W --calls-only $V --steps 300 --warmup 100 > $D/$W.trace.json")
    L.append(f"rocprofv3 --pmc {RD_SET} --output-format csv -d $D/$W.rd -- python3 $R/bench.py --workload $W --calls-only $V --steps 5 --warmup 2 > $D/$W.rd.json")
    L.append("rocprofv3 --pmc WRITE_SIZE --output-format csv -d $D/$W.wr -- python3 $R/bench.py --workload $W --calls-only $V --steps 5 --warmup 2 > $D/$W.wr.json")
    L.append(f"rocprofv3 --pmc {SQ_SET} --output-format csv -d $D/$W.sq -- python3 $R/bench.py --workload $W --calls-only $V --steps 5 --warmup 2 > $D/$W.sq.json")
    L.append("```\n")
    L.append("`--calls-only` makes nothing but the named calls (a one-workgroup marker kernel before each variant "
             "lets the dispatch list be cut into variants).  Bytes are requests between the L2 caches and the memory "
             "fabric: read = 32 x `TCC_EA0_RDREQ_32B` + 64 x `TCC_EA0_RDREQ_64B` + 128 x `TCC_EA0_RDREQ_128B`, "
             "written = `WRITE_SIZE` x 1024.  Hits in the 256 MB memory-side cache are behind that point and not "
             "visible.  VALU = `SQ_INSTS_VALU` (wave instructions) x 64 lanes / elements of the workload.  "
             "Durations are from the kernel trace (not from the counter runs, which serialise dispatches); the "
             "first few dozen launches after the host has kept the device idle run at a reduced shader clock "
             "(1.5 to 2.0 instead of 2.4 GHz, which slows the passes with arithmetic in them by up to a quarter), "
             "hence 400 calls per variant and the median next to the average.  The last two columns are the "
             "per-pass bandwidth picture (the analogue of the paper's per-pass charts against STREAM, Section "
             "6.4): the bytes this kernel moved between L2 and the fabric over its median duration, and that "
             "rate over the rate of the calibration kernel of the same workload with the same kind of traffic "
             "(`chunk_read` for a pass that only reads, `chunk_copy` for one that also writes).\n")
    for w, wl in data.items():
        info = wl["info"]
        s = ELEM_BYTES[info["dtype"]]
        elems = info["rows"] * info["n"]
        L.append(f"## {w}: {info['rows']} x {info['n']} {info['dtype']} ({elems * s / 2**20:,.1f} MiB in, the same out)\n")
        L.append("| variant | kernel | launches per call | grid x block | avg us | median | min | max | MiB read | "
                 "MiB written | VALU lane-ops per element | GB/s on those bytes (median) | of the calibration kernel |")
        L.append("|---|---|---|---|---|---|---|---|---|---|---|---|---|")

        def moved(variant, kname):
            """(bytes between L2 and fabric, median us) of one kernel, or None."""
            kinds = wl.get("variants", {}).get(variant, {})
            rd, wr, tr = (kinds.get(k, {}).get(kname) for k in ("rd", "wr", "trace"))
            if not (rd and wr and tr):
                return None
            return read_bytes(rd) + wr.get("WRITE_SIZE", 0) * 1024, tr["us_med"], wr.get("WRITE_SIZE", 0) * 1024

        # the calibration kernels of the same workload: a pass that only reads is set against the
        # read kernel, one that reads and writes against the copy kernel (Section 6.4 does the same
        # with STREAM)
        calib = {}
        for cv in ("read", "copy"):
            for kname in wl.get("variants", {}).get(cv, {}).get("trace", {}):
                if base(kname) in ("chunk_read", "chunk_copy"):
                    m = moved(cv, kname)
                    if m:
                        calib[cv] = m[0] / m[1]
        for variant, kinds in wl.get("variants", {}).items():
            ref = kinds.get("trace") or kinds.get("rd") or kinds.get("sq") or {}
            for kname, t in ref.items():
                rd = kinds.get("rd", {}).get(kname)
                wr = kinds.get("wr", {}).get(kname)
                sq = kinds.get("sq", {}).get(kname)
                tr = kinds.get("trace", {}).get(kname)
                m = moved(variant, kname)
                rate = against = "-"
                if m and m[0] > 2**20:
                    rate = f"{m[0] / m[1] / 1e3:,.0f}"
                    kind = "copy" if m[2] > 2**20 else "read"
                    if kind in calib:
                        against = f"{m[0] / m[1] / calib[kind]:.2f} of {kind}"
                L.append("| {} | `{}` | {:g} | {} x {} | {} | {} | {} | {} | {} | {} | {} | {} | {} |".format(
                    variant, kname, t["launches_per_call"], t["grid_threads"] // max(t["block"], 1), t["block"],
                    f"{tr['us_avg']:.1f}" if tr else "-", f"{tr['us_med']:.1f}" if tr else "-",
                    f"{tr['us_min']:.1f}" if tr else "-", f"{tr['us_max']:.1f}" if tr else "-",
                    f"{read_bytes(rd) / 2**20:,.2f}" if rd else "-",
                    f"{wr.get('WRITE_SIZE', 0) / 1024:,.2f}" if wr else "-",
                    f"{sq['SQ_INSTS_VALU'] * 64 / elems:.1f}" if sq and "SQ_INSTS_VALU" in sq else "-",
                    rate, against))
        L.append("")
        L.append("| variant | algorithmic MiB per call (Table 2) | measured MiB per call | measured / algorithmic | |")
        L.append("|---|---|---|---|---|")
        for variant in wl.get("variants", {}):
            name = "stream_" + variant if variant in ("copy", "read") else variant
            rec = counters["workloads"][w].get(name, {})
            alg = BYTES_PER_ELEM[variant] * elems * s
            if "hbm_bytes" in rec:
                ratio = rec["hbm_bytes"] / alg
                label = "cache-assisted: a re-read is served on chip" if ratio < 0.95 else ""
                L.append(f"| {variant} | {alg / 2**20:,.1f} | {rec['hbm_bytes'] / 2**20:,.1f} | {ratio:.3f} | {label} |")
        L.append("")
    L.append("## SQ counters per launch\n")
    L.append("| workload | kernel | SQ_WAVES | SQ_INSTS_VALU | SQ_ACTIVE_INST_VALU | SQ_BUSY_CYCLES | SQ_WAVE_CYCLES | "
             "SQ_INSTS_VMEM_RD | SQ_INSTS_VMEM_WR | VALU time at 4 cycles per wave instruction over 1024 SIMDs, 2.4 GHz (us) |")
    L.append("|---|---|---|---|---|---|---|---|---|---|")
    for w, wl in data.items():
        seen = set()
        for variant, kinds in wl.get("variants", {}).items():
            for kname, q in kinds.get("sq", {}).items():
                if kname in seen or "SQ_INSTS_VALU" not in q:
                    continue
                seen.add(kname)
                L.append("| {} | `{}` | {} | {} | {} | {} | {} | {} | {} | {:.1f} |".format(
                    w, kname, *(fmt_int(q.get(c, 0)) for c in ("SQ_WAVES", "SQ_INSTS_VALU", "SQ_ACTIVE_INST_VALU",
                                                               "SQ_BUSY_CYCLES", "SQ_WAVE_CYCLES", "SQ_INSTS_VMEM_RD",
                                                               "SQ_INSTS_VMEM_WR")),
                    q["SQ_INSTS_VALU"] * 4 / 1024 / 2.4e3))
    L.append("")
    open(path, "w").write("\n".join(L))


def write_memory_md(data, path):
    wl = data.get("cfg4")
    if not wl:
        return
    rows = []
    for variant, kinds in wl["variants"].items():
        names = collections.OrderedDict()
        for m in MEMORY_SETS:
            for kname in kinds.get(m, {}):
                names[kname] = None
        for kname in names:
            row = {"variant": variant, "kernel": kname}
            for m in MEMORY_SETS:
                row.update({c: v for c, v in kinds.get(m, {}).get(kname, {}).items() if c.startswith("TC")})
            tr = kinds.get("trace", {}).get(kname)
            if tr:
                row["us"] = tr["us_avg"]
            rows.append(row)
    L = ["# Memory-side counters of the 1 GiB streams (cfg4: 1 x 2^28 fp32), per launch\n",
         "Why a pass that reads 1 GiB and writes 1 GiB stops at about 6.6 TB/s when a read-only pass reaches 7.2: "
         "what the L2 caches (TCC) and the vector L1 (TCP) report for the plain copy, the plain read and the two "
         "Two-Pass kernels.  Commands (as in `kernels_all_workloads.md`, one counter set per run):\n", "```"]
    for m, c in MEMORY_SETS.items():
        L.append(f"rocprofv3 --pmc {c} --output-format csv -d $D/cfg4.{m} -- python3 $R/bench.py --workload cfg4 "
                 f"--calls-only softmax2p,copy,read --steps 5 --warmup 2 > $D/cfg4.{m}.json")
    L += ["```\n", "All `_sum` counters are summed over the 16 channels of each of the 8 L2 caches.  `LEVEL / REQ` is the "
          "average number of cycles a request to the memory fabric was outstanding.\n"]
    cols = []
    for c in " ".join(MEMORY_SETS.values()).split():
        if c not in cols:
            cols.append(c)
    L.append("| kernel | avg us (kernel trace) | " + " | ".join(c.replace("_sum", "") for c in cols) + " |")
    L.append("|---|---|" + "---|" * len(cols))
    for r in rows:
        L.append(f"| `{r['kernel']}` ({r['variant']}) | " + (f"{r['us']:.1f}" if "us" in r else "-") + " | " +
                 " | ".join(fmt_int(r[c]) if c in r else "-" for c in cols) + " |")
    L.append("")
    L.append("| kernel | read latency at the fabric (RDREQ_LEVEL / RDREQ, cycles) | write latency (WRREQ_LEVEL / WRREQ) | "
             "write requests stalled (WRREQ_STALL / WRREQ) | DRAM credit stalls per request, read | ... write | "
             "L1 read latency (TCP_TCC_READ_REQ_LATENCY / TCP_TCC_READ_REQ) |")
    L.append("|---|---|---|---|---|---|---|")

    def ratio(r, a, b):
        return f"{r[a] / r[b]:.2f}" if a in r and r.get(b) else "-"
    for r in rows:
        L.append(f"| `{r['kernel']}` | {ratio(r, 'TCC_EA0_RDREQ_LEVEL_sum', 'TCC_EA0_RDREQ_sum')} | "
                 f"{ratio(r, 'TCC_EA0_WRREQ_LEVEL_sum', 'TCC_EA0_WRREQ_sum')} | "
                 f"{ratio(r, 'TCC_EA0_WRREQ_STALL_sum', 'TCC_EA0_WRREQ_sum')} | "
                 f"{ratio(r, 'TCC_EA0_RDREQ_DRAM_CREDIT_STALL_sum', 'TCC_EA0_RDREQ_sum')} | "
                 f"{ratio(r, 'TCC_EA0_WRREQ_DRAM_CREDIT_STALL_sum', 'TCC_EA0_WRREQ_sum')} | "
                 f"{ratio(r, 'TCP_TCC_READ_REQ_LATENCY_sum', 'TCP_TCC_READ_REQ_sum')} |")
    L.append("")
    open(path, "w").write("\n".join(L))


def write_dominant_md(data, counters, path):
    wl = data.get("cfg4")
    if not wl or "softmax2p" not in wl.get("variants", {}):
        return
    kinds = wl["variants"]["softmax2p"]
    tr = kinds.get("trace", {})
    p2 = next((k for k in tr if k.startswith("chunk_2p_pass2")), None)
    if p2 is None:
        return
    t = tr[p2]
    rec = counters["workloads"]["cfg4"]["softmax2p"]["kernels"].get("chunk_2p_pass2", {})
    alg = 2 * (1 << 28) * 4
    copy = wl["variants"].get("copy", {}).get("trace", {})
    ck = next(iter(copy.values()), None)
    p1 = next((tr[k] for k in tr if k.startswith("chunk_2p_pass1")), None)
    mg = next((tr[k] for k in tr if k.startswith("merge_pairs")), None)
    L = [f"# `{p2}` on cfg4 (1 x 2^28 fp32, 1 GiB in, 1 GiB out): the dominant kernel\n",
         "Commands: as in `kernels_all_workloads.md` with `$W` = cfg4 (`rocprofv3 --kernel-trace --stats ... -- python3 "
         "bench.py --workload cfg4 --calls-only softmax2p,softmax3p_recompute,softmax3p_reload,copy,read --steps 300 "
         "--warmup 100`, and the `rd` / `wr` counter runs of the same command with `--steps 5 --warmup 2`).\n",
         "| figure | value |", "|---|---|",
         f"| launches in the trace | {t['dispatches']} |",
         f"| average duration (kernel trace) | {t['us_avg']:.1f} us (median {t['us_med']:.1f}, min {t['us_min']:.1f}, "
         f"max {t['us_max']:.1f}) |",
         f"| algorithmic bytes per launch | 2 * 2^28 * 4 = {alg:,} B (read x once, write y once) |",
         f"| achieved (algorithmic bytes / average duration) | {alg / t['us_avg'] / 1e6:.2f} TB/s = "
         f"{alg / t['us_avg'] / 1e6 / 8 * 100:.1f} % of the 8 TB/s HBM peak |"]
    if "hbm_bytes" in rec:
        L += [f"| bytes read from the memory fabric per launch (request counters) | {rec['fetch_bytes']:,} |",
              f"| bytes written per launch (WRITE_SIZE) | {rec['write_bytes']:,} |",
              f"| measured traffic per launch | {rec['hbm_bytes']:,} B = {rec['hbm_bytes'] / alg:.5f} x algorithmic |"]
    if ck:
        L.append(f"| plain copy kernel of the same size in the same run (`{next(iter(copy))}`) | {ck['us_avg']:.1f} us "
                 f"(median {ck['us_med']:.1f}) |")
    L.append("")
    if p1 and mg:
        L.append(f"The whole Two-Pass call on this workload: pass 1 {p1['us_avg']:.1f} us "
                 f"({(1 << 30) / p1['us_avg'] / 1e6:.2f} TB/s on 1 GiB read) + `merge_pairs_kernel` {mg['us_avg']:.1f} us + this "
                 f"kernel {t['us_avg']:.1f} us.  Durations vary by a few percent from box to box.")
    L.append("")
    open(path, "w").write("\n".join(L))


def write_bench_trace_md(root, path):
    """Kernel durations of the default `bench.py` run under rocprofv3 --kernel-trace --stats (DIR/bench.trace)."""
    files = newest(os.path.join(root, "bench.trace", "**", "*_kernel_trace.csv"))
    line = os.path.join(root, "bench.trace.json")
    if not files or not os.path.exists(line):
        return False
    bench = None
    for text in open(line):
        if text.startswith("{"):
            bench = json.loads(text)
    groups = collections.OrderedDict()
    for r in csv.DictReader(open(files[0])):
        if "tp::" not in r["Kernel_Name"]:
            continue
        k = (short(r["Kernel_Name"]), int(r["Grid_Size_X"]) // max(int(r["Workgroup_Size_X"]), 1), int(r["Workgroup_Size_X"]))
        groups.setdefault(k, []).append((int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3)
    L = ["# Kernel trace of the default `bench.py` run (MI355X, gfx950)\n",
         "Command (from `/tmp` with `TMPDIR=/tmp`; `$R` is the repository root):\n", "```",
         "rocprofv3 --kernel-trace --stats --output-format csv -d $D/bench.trace -- python3 $R/bench.py --steps 20 --warmup 5 > $D/bench.trace.json",
         "```\n"]
    if bench:
        ro = bench["roofline"]
        # the headline shape is the instantiation of that kernel the run spent the most time in
        dom = sorted((v for k, v in groups.items() if k[0].startswith(ro["kernel"] + "<")), key=sum, reverse=True)
        L.append(f"The same run's JSON line: `value` {bench['value']:.0f} GB/s, `ms_per_step` {bench['ms_per_step']:.4f}, "
                 f"`roofline.avg_launch_ms` {ro['avg_launch_ms']:.4f} for `{ro['kernel']}` (events, eight launches per "
                 f"pair), `roofline.frac` {ro['frac']:.3f}; `long_run` median {bench['long_run']['ms_median']:.4f} ms over "
                 f"{bench['long_run']['calls']} calls.")
        if dom:
            us = sorted(dom[0])
            L.append(f"Kernel trace of that kernel at the headline shape: {len(us)} launches, average "
                     f"{sum(us) / len(us):.1f} us, median {us[len(us) // 2]:.1f}, min {us[0]:.1f}, max {us[-1]:.1f}: "
                     f"{ro['algorithmic_bytes_per_launch'] / (sum(us) / len(us)) / 1e6 / 8 * 100:.1f} % of the 8 TB/s peak "
                     "on its algorithmic bytes.")
        L.append("")
    L += ["| kernel | grid (workgroups x threads) | launches | avg us | median | min | max |", "|---|---|---|---|---|---|---|"]
    for (k, g, b), us in sorted(groups.items(), key=lambda kv: -sum(kv[1])):
        us = sorted(us)
        L.append(f"| `{k}` | {g} x {b} | {len(us)} | {sum(us) / len(us):.1f} | {us[len(us) // 2]:.1f} | {us[0]:.1f} | {us[-1]:.1f} |")
    L.append("")
    open(path, "w").write("\n".join(L))
    return True


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("dir", help="directory holding the <workload>.<set> rocprofv3 outputs")
    ap.add_argument("--commit", default="", help="commit the profiled library was built from")
    args = ap.parse_args()
    data = collect(args.dir)
    if not data:
        raise SystemExit(f"no profiled runs under {args.dir}")
    counters = build_counters(data, args.commit, args.dir)
    os.makedirs(PROFILES, exist_ok=True)
    with open(os.path.join(PROFILES, "counters.json"), "w") as f:
        json.dump(counters, f, indent=1)
        f.write("\n")
    write_kernels_md(data, counters, args.dir, os.path.join(PROFILES, "kernels_all_workloads.md"))
    write_dominant_md(data, counters, os.path.join(PROFILES, "chunk_2p_pass2_cfg4.md"))
    write_memory_md(data, os.path.join(PROFILES, "memory_side_cfg4.md"))
    extra = ", bench_kernel_trace.md" if write_bench_trace_md(args.dir, os.path.join(PROFILES, "bench_kernel_trace.md")) else ""
    print("wrote profiles/counters.json, kernels_all_workloads.md, chunk_2p_pass2_cfg4.md, memory_side_cfg4.md" + extra)


if __name__ == "__main__":
    main()
