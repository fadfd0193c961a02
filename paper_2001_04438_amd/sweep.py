"""Size sweep of the three softmax algorithms on one GPU (the analogue of the paper's
Figures 1, 2, 5 and 6, which sweep the array length across the cache levels of a CPU).

Two sweeps, both on synthetic N(0, 4) fp32 data already resident in HBM:

  batch   a fixed total of 2^26 elements (256 MiB in, 256 MiB out) arranged as rows x N with
          N = 2^8 ... 2^26: shows where the one-workgroup-per-row path (second read served by
          L2) hands over to the chunked path (every read from memory)
  single  one vector of N = 2^10 ... 2^28 elements

Each point is the median of `--iters` calls, every call bracketed by events on the launch
stream, rotating over enough buffer sets to exceed 1 GiB so that no call finds its input in
a cache.  Output: a markdown table on stdout.

    python -m paper_2001_04438_amd.sweep [--iters 20] [--which batch|single|both]
"""
from __future__ import annotations

import argparse
import sys


def _median_ms(torch, fn, iters, sets):
    import time
    t0 = time.perf_counter()
    i = 0
    while i < 3 or time.perf_counter() - t0 < 0.05:   # untimed: also brings the clocks up
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


def _point(torch, B, rows, n, iters):
    total = rows * n
    sets = max(1, min(8, -(-(1 << 30) // (8 * total))))
    xs = [torch.randn(total, dtype=torch.float32, device="cuda") * 4 for _ in range(sets)]
    ys = [torch.empty_like(xs[0]) for _ in range(sets)]
    out = {}
    variants = [("2p", B.softmax2p_f32, 3), ("3p_recompute", B.softmax3p_recompute_f32, 4),
                ("3p_reload", B.softmax3p_reload_f32, 5)]
    if n <= 32768:
        variants.append(("2p_onchip", B.softmax2p_onchip_f32, 2))
    for name, fn, k in variants:
        ms = _median_ms(torch, lambda i, fn=fn: fn(xs[i], ys[i], rows, n), iters, sets)
        out[name] = (ms, k * total * 4 / ms / 1e6)
    del xs, ys
    torch.cuda.empty_cache()
    return out


def _table(torch, B, shapes, iters):
    print("| rows | N | path | 2P ms | 2P GB/s (3N) | 3P-recompute ms | 3P-reload ms | "
          "2P vs recompute | 2P vs reload | on-chip 2P ms |")
    print("|---|---|---|---|---|---|---|---|---|---|")
    for rows, n in shapes:
        p = _point(torch, B, rows, n, iters)
        path = "rows" if B.softmax_tp_plan(rows, n).path == 1 else "chunk"
        oc = f"{p['2p_onchip'][0]:.4f}" if "2p_onchip" in p else "-"
        print(f"| {rows} | {n} | {path} | {p['2p'][0]:.4f} | {p['2p'][1]:.0f} | "
              f"{p['3p_recompute'][0]:.4f} | {p['3p_reload'][0]:.4f} | "
              f"{p['3p_recompute'][0] / p['2p'][0]:.2f}x | {p['3p_reload'][0] / p['2p'][0]:.2f}x | {oc} |",
              flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--iters", type=int, default=20)
    ap.add_argument("--which", default="both", choices=["batch", "single", "both"])
    args = ap.parse_args()
    import torch
    from . import binding as B
    if not torch.cuda.is_available():
        sys.exit("the sweep needs a GPU")
    B.lib()
    if args.which in ("batch", "both"):
        print("## batch: 2^26 elements as rows x N\n")
        _table(torch, B, [((1 << 26) >> e, 1 << e) for e in range(8, 27, 2)] +
               [((1 << 26) >> 15, 1 << 15), ((1 << 26) >> 17, 1 << 17)], args.iters)
        print()
    if args.which in ("single", "both"):
        print("## single vector of N elements\n")
        _table(torch, B, [(1, 1 << e) for e in range(10, 29, 2)], args.iters)
    B.softmax_tp_release()


if __name__ == "__main__":
    main()
