"""The CPU oracle under AddressSanitizer + UndefinedBehaviorSanitizer (host code only, no GPU).

A second build of oracle/lowdiff_oracle.cpp (-fsanitize=address,undefined, -O1) is loaded in a
child interpreter that was started with the sanitizer runtime preloaded, and the oracle's own pin
tests run against it there: the hand-worked fixtures, ragged and empty segments, k = 0 / 1 / n,
the combine's edge cases, the replays. Any out-of-bounds access, use after free, signed overflow
or misaligned access inside the oracle aborts the child, which fails this test.
"""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _runtime(name):
    out = subprocess.run(["g++", f"-print-file-name={name}"], capture_output=True, text=True).stdout.strip()
    return out if os.path.isabs(out) and os.path.exists(out) else None


def test_oracle_pins_pass_under_asan_and_ubsan():
    asan = _runtime("libasan.so")
    if asan is None:
        pytest.skip("no AddressSanitizer runtime next to g++")
    env = dict(os.environ)
    env["LOWDIFF_ORACLE_SANITIZE"] = "1"
    # the sanitizer runtime has to come first; whatever was preloaded before stays, after it
    env["LD_PRELOAD"] = ":".join(x for x in (asan, os.environ.get("LD_PRELOAD", "")) if x)
    # python itself is not instrumented: its arenas are not leaks of the oracle; nothing here uses a GPU
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1:verify_asan_link_order=0"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["HIP_VISIBLE_DEVICES"] = ""
    cmd = [sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-x", "-q",
           "-p", "no:cacheprovider", "-m", "not gpu"]
    res = subprocess.run(cmd, cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    tail = (res.stdout + res.stderr)[-4000:]
    assert res.returncode == 0, tail
    assert " passed" in res.stdout and "failed" not in res.stdout, tail
    assert "liblowdiff_oracle_san.so" in _loaded_library(env), "the child did not load the sanitized build"


def _loaded_library(env):
    code = "import oracle; print(oracle._LIB)"
    return subprocess.run([sys.executable, "-c", code], cwd=ROOT, env=env, capture_output=True, text=True).stdout
