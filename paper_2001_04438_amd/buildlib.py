"""Compiles the HIP sources for gfx950 into paper_2001_04438_amd/libsoftmax_tp.so."""
from __future__ import annotations

import os
import shutil
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB_PATH = os.path.join(HERE, "libsoftmax_tp.so")
SOURCES = ["softmax_tp.hip"]
HEADERS = ["tp_kernels.h", "tp_device.h", "extexp.h", "expconst.h", os.path.join("..", "..", "include", "softmax_tp.h")]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off",            # every fused multiply-add in the kernels is written out
    "-fno-gpu-rdc", "-fvisibility=hidden",
    # packed-fp32 instructions are kept out of the generated code on the test machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option",
]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found")


def up_to_date() -> bool:
    if not os.path.exists(LIB_PATH):
        return False
    t = os.path.getmtime(LIB_PATH)
    deps = [os.path.join(CSRC, f) for f in SOURCES + HEADERS]
    return all(os.path.getmtime(d) <= t for d in deps)


def build(force: bool = True, extra_flags=(), out: str = LIB_PATH) -> str:
    """Runs hipcc.  With force=False the compile is skipped when the library is newer than its sources."""
    if not force and out == LIB_PATH and up_to_date():
        return out
    cmd = [hipcc(), *HIPCC_FLAGS, *extra_flags, "-o", out] + [os.path.join(CSRC, s) for s in SOURCES]
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = ("packed-fp32-ops", "is not a recognized feature")
    err = "\n".join(l for l in res.stderr.splitlines() if not any(k in l for k in noise))
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if err.strip():
        print(err)
    return out


if __name__ == "__main__":
    print(build())
