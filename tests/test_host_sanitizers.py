"""The host-side C++ (micro-batch scheduler, KV page pool: csrc/gllm_sched.cpp, csrc/gllm_kv.cpp, csrc/page_pool.h)
under AddressSanitizer and UndefinedBehaviorSanitizer: the two sources are built with g++ -fsanitize=address,undefined
into a library of their own, and the exact-parity suites of both run against that library in a child interpreter
that has the sanitizer runtime preloaded.  Any report (out-of-bounds access, use after free, signed overflow,
misaligned access ...) aborts the child, which fails this test.  CPU only."""
import os
import subprocess
import sys

import pytest

from paper_2504_14775_amd import build as hip_build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_scheduler_and_page_pool_parity_suites_under_asan_and_ubsan():
    lib = hip_build.build_host_sanitized()
    runtime = hip_build.sanitizer_runtime()
    if not os.path.isabs(runtime) or not os.path.exists(runtime):
        pytest.skip("no AddressSanitizer runtime next to g++")
    env = dict(os.environ)
    # the sanitizer runtime must come first among the preloaded libraries; whatever is preloaded already stays
    env["LD_PRELOAD"] = runtime + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    # the interpreter itself is not instrumented: its allocations are not this test's subject
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1:halt_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["GLLM_HOST_LIBRARY"] = lib
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
           os.path.join(ROOT, "tests", "test_sched_parity.py"), os.path.join(ROOT, "tests", "test_kv_parity.py")]
    r = subprocess.run(cmd, cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)
    tail = (r.stdout + r.stderr)[-4000:]
    assert r.returncode == 0, tail
    assert "passed" in r.stdout and "failed" not in r.stdout, tail
    assert "ERROR: AddressSanitizer" not in tail and "runtime error" not in tail, tail
