"""Builds librlhf_rollout.so (gfx950) next to this file with hipcc.

    python -m paper_2410_15651_amd.build

hipcc cross-compiles without a GPU.  Packed-fp32 VALU instructions are switched
off for every device translation unit.
"""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "librlhf_rollout.so")
SOURCES = ["error.cpp", "alloc_sim.cpp", "arena.hip", "attention.hip", "logprob_kl.hip", "sampling.hip", "prefill.hip", "probe.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function", "-Wno-unknown-warning-option",
    "-fno-gpu-rdc",
    "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
]


def sources():
    return [os.path.join(CSRC, s) for s in SOURCES]


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, f) for f in os.listdir(CSRC)]
    deps.append(os.path.join(ROOT, "include", "rlhf_rollout.h"))
    deps.append(os.path.join(ROOT, "include", "rlhf_memtrace.h"))
    return any(os.path.getmtime(d) > t for d in deps)


def build(verbose: bool = False) -> str:
    cmd = [HIPCC] + FLAGS + ["-x", "hip"] + sources() + ["-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    # the host pass warns that it does not know the packed-fp32 feature: harmless
    err = "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if verbose and err.strip():
        print(err, file=sys.stderr)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
