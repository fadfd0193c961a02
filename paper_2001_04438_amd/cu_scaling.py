"""Scaling of the three softmax algorithms with the number of compute units in use (the
analogue of the paper's multi-threaded weak-scaling study, Section 6.6, Figures 8 and 9).

The single 2^28-element fp32 vector (1 GiB, out of every cache) is processed on streams
created with hipExtStreamCreateWithCUMask so that only the first k compute units take part.
The array stays the same while k grows, as in the paper, where the array is 4 x the last-level
cache for every thread count.  Prints a markdown table.

    python -m paper_2001_04438_amd.cu_scaling [--iters 5]
"""
from __future__ import annotations

import argparse
import ctypes
import sys
import time


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--iters", type=int, default=5)
    args = ap.parse_args()
    import torch
    from . import binding as B
    if not torch.cuda.is_available():
        sys.exit("needs a GPU")
    B.lib()
    hip = ctypes.CDLL("libamdhip64.so")
    hip.hipExtStreamCreateWithCUMask.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.c_uint32,
                                                 ctypes.POINTER(ctypes.c_uint32)]
    hip.hipStreamSynchronize.argtypes = [ctypes.c_void_p]
    hip.hipStreamDestroy.argtypes = [ctypes.c_void_p]
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    n = 1 << 28
    x = torch.rand(n, device="cuda") * 200 - 100
    y = torch.empty_like(x)
    torch.cuda.synchronize()
    words = (cus + 31) // 32
    print("| CUs | 2P ms | 2P GB/s (3N) | 3P-recompute ms | 3P-reload ms | 2P vs recompute | 2P vs reload |")
    print("|---|---|---|---|---|---|---|")
    for k in (8, 16, 32, 64, 96, 128, 192, cus):
        mask = (ctypes.c_uint32 * words)()
        for i in range(k):
            mask[i // 32] |= 1 << (i % 32)
        st = ctypes.c_void_p()
        rc = hip.hipExtStreamCreateWithCUMask(ctypes.byref(st), words, mask)
        if rc != 0:
            sys.exit(f"hipExtStreamCreateWithCUMask failed with {rc}")
        ms = []
        for fn in (B.softmax2p_f32, B.softmax3p_recompute_f32, B.softmax3p_reload_f32):
            w0 = time.perf_counter()
            warm = 0
            while warm < 2 or time.perf_counter() - w0 < 0.05:   # untimed; also brings the clocks up
                fn(x, y, 1, n, stream=st.value)
                hip.hipStreamSynchronize(st)
                warm += 1
            t0 = time.perf_counter()
            for _ in range(args.iters):
                fn(x, y, 1, n, stream=st.value)
            hip.hipStreamSynchronize(st)
            ms.append((time.perf_counter() - t0) / args.iters * 1e3)
        print(f"| {k} | {ms[0]:.3f} | {3 * n * 4 / ms[0] / 1e6:.0f} | {ms[1]:.3f} | {ms[2]:.3f} | "
              f"{ms[1] / ms[0]:.2f}x | {ms[2] / ms[0]:.2f}x |", flush=True)
        hip.hipStreamDestroy(st)
    B.softmax_tp_release()


if __name__ == "__main__":
    main()
