"""Size sweep of the three softmax algorithms on one GPU (the analogue of the paper's
Figures 1, 2, 5 and 6, which sweep the array length across the cache levels of a CPU).

Two sweeps, both on synthetic N(0, 4) data already resident in HBM, in fp32 and in bf16
storage (the one regime where the outcome differs: bf16 rows are bound by vector instructions):

  batch   a fixed total of 2^26 elements arranged as rows x N with N = 2^8 ... 2^26: shows
          where the one-workgroup-per-row path (second read served by L2) hands over to the
          chunked path (every read from memory)
  single  one vector of N = 2^10 ... 2^28 elements
  ragged  the same 2^26 elements as rows of lengths that are not powers of two (24 ... 57000
          elements, among them 1.5 x 2^k and class counts like 1000 and 21846), which leave
          the last round of a lane group or a workgroup partly filled

Each point is the median of `--iters` calls, every call bracketed by events on the launch
stream, rotating over enough buffer sets to exceed 1 GiB so that no call finds its input in
a cache.  Output: markdown tables on stdout.

    python -m paper_2001_04438_amd.sweep [--iters 20] [--which batch|single|ragged|all] [--dtype f32|bf16|both]
"""
from __future__ import annotations

import argparse
import sys

VARIANTS = (("2p", "softmax2p", 3), ("3p_recompute", "softmax3p_recompute", 4),
            ("3p_reload", "softmax3p_reload", 5), ("2p_onchip", "softmax2p_onchip", 2))
SUFFIX = {"f32": "_f32", "bf16": "_bf16io"}
ONCHIP_MAX_N = 32768
RAGGED_N = (24, 96, 100, 192, 384, 768, 1000, 1100, 1300, 3000, 5000, 10000, 21846, 28000, 40000, 57000)


def median_ms(torch, fn, iters, sets):
    """Median over `iters` calls of fn(set index), each between its own pair of events, after at
    least 50 ms of untimed calls (which also bring the clocks up)."""
    import time
    t0 = time.perf_counter()
    i = 0
    while i < 3 or time.perf_counter() - t0 < 0.05:
        fn(i % sets)
        i += 1
        if i % 16 == 0:
            torch.cuda.synchronize()
    torch.cuda.synchronize()
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
           for _ in range(iters)]
    for i, (a, b) in enumerate(evs):
        a.record()
        fn(i % sets)
        b.record()
    torch.cuda.synchronize()
    ts = sorted(a.elapsed_time(b) for a, b in evs)
    return ts[len(ts) // 2]


def point(torch, B, rows, n, iters, dtype="f32"):
    """One point of the sweep: {variant: (median ms, GB/s on the variant's algorithmic bytes)} plus
    "path" ("rows" or "chunk").  The on-chip variant is present for rows of at most 32768 elements."""
    total = rows * n
    s = 4 if dtype == "f32" else 2
    sets = max(1, min(8, -(-(1 << 30) // (2 * s * total))))
    if dtype == "f32":
        xs = [torch.randn(total, dtype=torch.float32, device="cuda") * 4 for _ in range(sets)]
    else:
        xs = [(torch.randn(total, dtype=torch.float32, device="cuda") * 4).to(torch.bfloat16).view(torch.int16)
              for _ in range(sets)]
    ys = [torch.empty_like(xs[0]) for _ in range(sets)]
    out = {"path": "rows" if B.softmax_tp_plan(rows, n, s).path == 1 else "chunk"}
    for key, name, k in VARIANTS:
        if key == "2p_onchip" and n > ONCHIP_MAX_N:
            continue
        fn = getattr(B, name + SUFFIX[dtype])
        ms = median_ms(torch, lambda i, fn=fn: fn(xs[i], ys[i], rows, n), iters, sets)
        out[key] = (ms, k * total * s / ms / 1e6)
    del xs, ys
    torch.cuda.empty_cache()
    return out


def table(torch, B, shapes, iters, dtype):
    print("| rows | N | path | 2P ms | 2P GB/s (3N) | 3P-recompute ms | 3P-reload ms | "
          "2P vs recompute | 2P vs reload | on-chip 2P ms |")
    print("|---|---|---|---|---|---|---|---|---|---|")
    for rows, n in shapes:
        p = point(torch, B, rows, n, iters, dtype)
        oc = f"{p['2p_onchip'][0]:.4f}" if "2p_onchip" in p else "-"
        print(f"| {rows} | {n} | {p['path']} | {p['2p'][0]:.4f} | {p['2p'][1]:.0f} | "
              f"{p['3p_recompute'][0]:.4f} | {p['3p_reload'][0]:.4f} | "
              f"{p['3p_recompute'][0] / p['2p'][0]:.2f}x | {p['3p_reload'][0] / p['2p'][0]:.2f}x | {oc} |",
              flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--iters", type=int, default=20)
    ap.add_argument("--which", default="all", choices=["batch", "single", "ragged", "both", "all"])
    ap.add_argument("--dtype", default="both", choices=["f32", "bf16", "both"])
    args = ap.parse_args()
    import torch
    from . import binding as B
    if not torch.cuda.is_available():
        sys.exit("the sweep needs a GPU")
    B.lib()
    for dtype in (("f32", "bf16") if args.dtype == "both" else (args.dtype,)):
        if args.which in ("batch", "both", "all"):
            print(f"## batch, {dtype}: 2^26 elements as rows x N\n")
            table(torch, B, [((1 << 26) >> e, 1 << e) for e in range(8, 27, 2)] +
                  [((1 << 26) >> 15, 1 << 15), ((1 << 26) >> 17, 1 << 17)], args.iters, dtype)
            print()
        if args.which in ("single", "both", "all"):
            print(f"## single vector of N elements, {dtype}\n")
            table(torch, B, [(1, 1 << e) for e in range(10, 29, 2)], args.iters, dtype)
            print()
        if args.which in ("ragged", "all"):
            print(f"## ragged rows, {dtype}: about 2^26 elements as rows x N\n")
            table(torch, B, [((1 << 26) // n, n) for n in RAGGED_N], args.iters, dtype)
            print()
    B.softmax_tp_release()


if __name__ == "__main__":
    main()
