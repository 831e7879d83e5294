"""Build the C-ABI library ``libpod_attn.so`` for gfx950 with hipcc (cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libpod_attn.so")
SOURCES = ["pod_kernels.hip", "pod_probe.hip", "pod_planner.cpp", "pod_api.cpp"]
HEADERS = ["pod_common.h", "pod_launch.h", "pod_planner.h", os.path.join("..", "..", "include", "pod_attn.h")]
# Packed-fp32 instructions are switched off for the device pass (the host pass does not know
# the feature and says so; that message is harmless).  The compiler's rewriting of atomics is
# switched off too: every counter update here is already issued by one lane, and the rewrite
# reads the result back at once, which makes a claim issued ahead of its use wait on the spot.
HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
               "-mllvm", "-amdgpu-atomic-optimizer-strategy=None",
               "-Wall", "-Wno-unused-function", "-Wno-inline-asm"]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    built = os.path.getmtime(LIB)
    return any(os.path.getmtime(os.path.join(CSRC, f)) > built for f in SOURCES + HEADERS)


def build(force: bool = True, extra_flags=(), verbose: bool = False) -> str:
    """Compile the library; returns its path.  With force=False only when sources are newer."""
    if not force and not is_stale():
        return LIB
    tmp = LIB + f".tmp{os.getpid()}"
    cmd = [hipcc(), *HIPCC_FLAGS, *extra_flags, *[os.path.join(CSRC, s) for s in SOURCES], "-o", tmp]
    proc = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    log = "\n".join(l for l in (proc.stdout + proc.stderr).splitlines() if noise not in l)
    if proc.returncode != 0:
        if os.path.exists(tmp):
            os.remove(tmp)
        raise RuntimeError("hipcc failed:\n" + log)
    if verbose and log.strip():
        print(log, file=sys.stderr)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(force=True, verbose=True))
