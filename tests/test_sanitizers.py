"""CPU-side sanitizer passes: the C oracle, and the host code of the library (argument validation,
the split and workspace planning, the host scan of the paged cache), rebuilt with AddressSanitizer and
UndefinedBehaviorSanitizer and driven by the existing CPU tests in a child process that preloads the
sanitizer runtime.  Any report aborts the child, which fails the test.  No GPU is involved; the
device code of the library is compiled as usual and never launched here."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run(tests, env_extra, preload):
    env = dict(os.environ)
    env.update(env_extra)
    env["LD_PRELOAD"] = preload + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    # (leak checking off: the interpreter and the runtime libraries it loads are not leak-clean)
    env["ASAN_OPTIONS"] = "detect_leaks=0:halt_on_error=1:abort_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    res = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", *tests],
                         cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    tail = (res.stdout + res.stderr)[-3000:]
    assert res.returncode == 0, tail
    assert "AddressSanitizer" not in tail and "runtime error" not in tail, tail
    assert " passed" in res.stdout, tail


def test_oracle_under_asan_and_ubsan():
    import oracle
    so = oracle.build_sanitized()
    libasan = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    if not os.path.isabs(libasan) or not os.path.exists(libasan):
        pytest.skip("gcc's libasan is not installed")
    _run(["tests/test_oracle_pins.py", "tests/test_oracle_paged_pins.py"], {"DEINFER_ORACLE_SO": so}, libasan)


def test_library_host_code_under_asan_and_ubsan():
    from paper_2604_17709_amd import build as b
    so = b.build_host_sanitized()
    _run(["tests/test_abi.py", "tests/test_kv_plan.py"], {"DEINFER_LIBRARY_PATH": so}, b.asan_runtime())
