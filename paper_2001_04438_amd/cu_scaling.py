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
import contextlib
import ctypes
import sys
import time

_hip = None


def hip():
    """The HIP runtime, for the three stream calls torch has no binding for."""
    global _hip
    if _hip is None:
        h = ctypes.CDLL("libamdhip64.so")
        h.hipExtStreamCreateWithCUMask.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.c_uint32,
                                                   ctypes.POINTER(ctypes.c_uint32)]
        h.hipStreamSynchronize.argtypes = [ctypes.c_void_p]
        h.hipStreamDestroy.argtypes = [ctypes.c_void_p]
        _hip = h
    return _hip


@contextlib.contextmanager
def masked_stream(k, cus):
    """A HIP stream (default priority) whose kernels run on the first k of the device's `cus`
    compute units only; yields the raw hipStream_t value.  Synchronised and destroyed on exit."""
    if not 1 <= k <= cus:
        raise ValueError(f"k = {k} outside 1..{cus}")
    words = (cus + 31) // 32
    mask = (ctypes.c_uint32 * words)()
    for i in range(k):
        mask[i // 32] |= 1 << (i % 32)
    st = ctypes.c_void_p()
    rc = hip().hipExtStreamCreateWithCUMask(ctypes.byref(st), words, mask)
    if rc != 0:
        raise RuntimeError(f"hipExtStreamCreateWithCUMask failed with {rc}")
    try:
        yield st.value
    finally:
        hip().hipStreamSynchronize(st)
        hip().hipStreamDestroy(st)


def time_on_stream(fn, stream, iters):
    """Host-clock milliseconds per call of fn(stream) over `iters` calls, after at least 50 ms and
    two untimed calls."""
    w0 = time.perf_counter()
    warm = 0
    while warm < 2 or time.perf_counter() - w0 < 0.05:
        fn(stream)
        hip().hipStreamSynchronize(stream)
        warm += 1
    t0 = time.perf_counter()
    for _ in range(iters):
        fn(stream)
    hip().hipStreamSynchronize(stream)
    return (time.perf_counter() - t0) / iters * 1e3


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--iters", type=int, default=5)
    args = ap.parse_args()
    import torch
    from . import binding as B
    if not torch.cuda.is_available():
        sys.exit("needs a GPU")
    B.lib()
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    n = 1 << 28
    x = torch.rand(n, device="cuda") * 200 - 100
    y = torch.empty_like(x)
    torch.cuda.synchronize()
    print("| CUs | 2P ms | 2P GB/s (3N) | 3P-recompute ms | 3P-reload ms | 2P vs recompute | 2P vs reload |")
    print("|---|---|---|---|---|---|---|")
    for k in (8, 16, 32, 64, 96, 128, 192, cus):
        with masked_stream(k, cus) as st:
            ms = [time_on_stream(lambda s, fn=fn: fn(x, y, 1, n, stream=s), st, args.iters)
                  for fn in (B.softmax2p_f32, B.softmax3p_recompute_f32, B.softmax3p_reload_f32)]
        print(f"| {k} | {ms[0]:.3f} | {3 * n * 4 / ms[0] / 1e6:.0f} | {ms[1]:.3f} | {ms[2]:.3f} | "
              f"{ms[1] / ms[0]:.2f}x | {ms[2] / ms[0]:.2f}x |", flush=True)
    B.softmax_tp_release()


if __name__ == "__main__":
    main()
