"""The library's host code (packer, plan builders, net layout: index arithmetic that runs
without a GPU) under AddressSanitizer and UndefinedBehaviorSanitizer: the host-side test files
are run once more, in a child process, against `python -m paper_1905_00571_amd.build --asan`."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_host_code_is_clean_under_asan_and_ubsan():
    from paper_1905_00571_amd import build
    if os.environ.get("LD_PRELOAD"):
        pytest.skip("something is preloaded already: the sanitizer runtime could not come first")
    runtime = build.asan_runtime()
    if not runtime:
        pytest.skip("no shared AddressSanitizer runtime beside the compiler")
    lib = build.build_asan(force=False)
    env = dict(os.environ)
    env.update({"LD_PRELOAD": runtime, "CADNN_LIB_PATH": lib,
                # (the interpreter itself is not leak-clean; every other check is on)
                "ASAN_OPTIONS": "detect_leaks=0:halt_on_error=1", "UBSAN_OPTIONS": "print_stacktrace=1:halt_on_error=1"})
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-s", "-p", "no:cacheprovider",
                        os.path.join(ROOT, "tests", "test_host_library.py"),
                        os.path.join(ROOT, "tests", "test_net_layout.py"),
                        os.path.join(ROOT, "tests", "test_host_plans.py")],
                       cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    tail = (r.stdout + r.stderr)[-3000:]
    assert r.returncode == 0, tail
    assert "runtime error" not in tail and "AddressSanitizer" not in tail, tail
