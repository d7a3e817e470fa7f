"""The oracle's pins once more with the oracle compiled under AddressSanitizer and
UndefinedBehaviorSanitizer (host code only, on the CPU): an out-of-bounds access, a signed
overflow or a misaligned load that happens to give the right answer would still be caught.

The sanitizer runtime has to be the first library of the process, so the pins run in a child
Python process that has it in front of whatever is preloaded already; the oracle package is
pointed at the instrumented library through the same swap that the planted-mistake tests use.
"""
import os
import subprocess
import sys

import pytest

import oracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(os.path.dirname(oracle.__file__), "surel_oracle.c")

CHILD = r"""
import ctypes, os, sys
sys.path.insert(0, os.path.join({root!r}, "tests"))
sys.path.insert(0, {root!r})
import oracle
import test_oracle_mutants as runner
real = oracle._load()
inst = ctypes.CDLL({lib!r})
for fn in ("oracle_philox4x32_10", "oracle_sample_walks", "oracle_build_rpe", "oracle_join_queries",
           "oracle_query_rpe_ids", "oracle_prune_rpe", "oracle_bfs_batch"):
    getattr(inst, fn).argtypes = getattr(real, fn).argtypes
    getattr(inst, fn).restype = getattr(real, fn).restype
oracle._lib = inst
failed = runner._run_pins(os.path.join({root!r}, "tests", "golden"))
print("PINS_RUN", len(runner.PIN_TESTS) + len(runner.PARAM_PIN_TESTS), "FAILED", failed)
sys.exit(1 if failed else 0)
"""


def test_pins_pass_with_the_oracle_under_asan_and_ubsan(tmp_path):
    asan = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True,
                          text=True).stdout.strip()
    if not os.path.isabs(asan) or not os.path.exists(asan):
        pytest.skip("gcc has no AddressSanitizer runtime here")
    lib = tmp_path / "liboracle_san.so"
    subprocess.run(["gcc", "-O1", "-g", "-std=c99", "-Wall", "-Wextra", "-fPIC", "-shared",
                    "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
                    "-fno-omit-frame-pointer", "-o", str(lib), SRC], check=True)
    env = dict(os.environ)
    env["LD_PRELOAD"] = asan + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    # the interpreter's own allocations are not the subject; a report from the oracle aborts
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    res = subprocess.run([sys.executable, "-c", CHILD.format(root=ROOT, lib=str(lib))], env=env,
                         capture_output=True, text=True, timeout=900)
    assert res.returncode == 0, f"stdout:\n{res.stdout[-2000:]}\nstderr:\n{res.stderr[-4000:]}"
    assert "PINS_RUN" in res.stdout and "FAILED []" in res.stdout
    assert "ERROR: AddressSanitizer" not in res.stderr and "runtime error" not in res.stderr
