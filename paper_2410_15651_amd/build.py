"""Builds librlhf_rollout.so (gfx950) next to this file with hipcc.

    python -m paper_2410_15651_amd.build              the library
    python -m paper_2410_15651_amd.build --sanitize   librlhf_rollout_sanitized.so: the same sources with
                                                      AddressSanitizer and UndefinedBehaviorSanitizer on the
                                                      HOST code only (device code untouched), for the CPU
                                                      tests of the host logic; see sanitizer_env()

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
SANITIZED_LIB = os.path.join(HERE, "librlhf_rollout_sanitized.so")
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


# each -fsanitize goes directly after -Xarch_host: the device passes are compiled as always
SANITIZE_FLAGS = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                  "-Xarch_host", "-fno-omit-frame-pointer", "-Xarch_host", "-fno-sanitize-recover=undefined",
                  "-shared-libsan", "-g"]


def sanitizer_env(env=None) -> dict:
    """Environment for a child process that loads the sanitized library from an
    interpreter that was not built with the sanitizers: the library is named by
    RLHF_ROLLOUT_LIB and the ASan runtime is put in front of whatever LD_PRELOAD
    already holds.  Leak checking is off (the interpreter itself never frees much
    of what it allocates)."""
    env = dict(os.environ if env is None else env)
    rt = subprocess.run([HIPCC, "--print-file-name=libclang_rt.asan-x86_64.so"], capture_output=True,
                        text=True).stdout.strip()
    if not os.path.isabs(rt) or not os.path.exists(rt):
        raise RuntimeError("the ASan runtime of " + HIPCC + " was not found")
    env["RLHF_ROLLOUT_LIB"] = SANITIZED_LIB
    env["LD_PRELOAD"] = rt + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1:verify_asan_link_order=0"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    return env


def build(verbose: bool = False, sanitize: bool = False) -> str:
    out = SANITIZED_LIB if sanitize else LIB
    cmd = [HIPCC] + FLAGS + (SANITIZE_FLAGS if sanitize else []) + ["-x", "hip"] + sources() + ["-o", out]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    # the host pass warns that it does not know the packed-fp32 feature: harmless
    err = "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if verbose and err.strip():
        print(err, file=sys.stderr)
    return out


if __name__ == "__main__":
    print(build(verbose=True, sanitize="--sanitize" in sys.argv[1:]))
