"""The library's host code (arena bookkeeping, allocator simulator, argument
checks of every entry point) under AddressSanitizer and UndefinedBehaviorSanitizer.

`python -m paper_2410_15651_amd.build --sanitize` compiles the same sources with the
sanitizers on the host passes only; the host-side test files are then run in a
child interpreter that loads that build (RLHF_ROLLOUT_LIB) with the ASan runtime
preloaded (build.sanitizer_env).  A report from either sanitizer aborts the child.
"""
import os
import subprocess
import sys

from paper_2410_15651_amd import build as lib_build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HOST_TESTS = ["tests/test_abi_and_host.py", "tests/test_alloc_model.py", "tests/test_memtrace.py"]


def _sanitized_is_stale() -> bool:
    if not os.path.exists(lib_build.SANITIZED_LIB):
        return True
    t = os.path.getmtime(lib_build.SANITIZED_LIB)
    deps = [os.path.join(lib_build.CSRC, f) for f in os.listdir(lib_build.CSRC)]
    deps += [os.path.join(ROOT, "include", f) for f in os.listdir(os.path.join(ROOT, "include"))]
    return any(os.path.getmtime(d) > t for d in deps)


def test_host_side_tests_pass_under_asan_and_ubsan():
    if _sanitized_is_stale():
        lib_build.build(sanitize=True)
    env = lib_build.sanitizer_env()
    res = subprocess.run([sys.executable, "-m", "pytest", *HOST_TESTS, "-q", "-x", "-p", "no:cacheprovider"],
                         cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)
    tail = (res.stdout + res.stderr)[-4000:]
    assert res.returncode == 0, tail
    assert " passed" in res.stdout and "failed" not in res.stdout, tail
    # the child really ran against the sanitized build
    probe = subprocess.run([sys.executable, "-c",
                            "from paper_2410_15651_amd import binding as rb; rb.lib(); print(rb.LIB_PATH); "
                            "print(open('/proc/self/maps').read().count('libclang_rt.asan'))"],
                           cwd=ROOT, env=env, capture_output=True, text=True, timeout=120)
    lines = probe.stdout.split()
    assert probe.returncode == 0 and lines[0] == lib_build.SANITIZED_LIB and int(lines[1]) > 0, probe.stdout + probe.stderr
