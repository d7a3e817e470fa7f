"""Builds libsurel.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree.

``python -m paper_2202_13538_amd.build`` compiles every source under ``csrc/`` and links
``paper_2202_13538_amd/libsurel.so``, then the memory-system micro-benchmarks of
``membench/`` into ``libsurel_membench.so`` (benchmark tooling that ``bench.py --membench``
loads; the hot path does not).  hipcc cross-compiles for gfx950, so no GPU is needed to build.
"""
from __future__ import annotations

import concurrent.futures
import os
import subprocess
import sys

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG_DIR, "csrc")
LIB_PATH = os.path.join(PKG_DIR, "libsurel.so")
MEMBENCH_SRC = os.path.join(PKG_DIR, "membench", "membench.hip")
MEMBENCH_LIB_PATH = os.path.join(PKG_DIR, "libsurel_membench.so")
BUILD_DIR = os.path.join(PKG_DIR, "_build")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
ARCH = "gfx950"
# Packed FP32 instructions are switched off for all device code of this library.
HIP_FLAGS = ["--offload-arch=" + ARCH, "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wextra",
             "-Wno-unused-parameter", "-Xclang", "-target-feature", "-Xclang",
             "-packed-fp32-ops"]


def sources() -> list[str]:
    return sorted(os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".hip"))


def _compile(src: str, extra: list[str]) -> str:
    obj = os.path.join(BUILD_DIR, os.path.basename(src) + ".o")
    cmd = [HIPCC, *HIP_FLAGS, *extra, "-c", src, "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    # hipcc's host pass does not know the packed-fp32 feature name; that warning is harmless
    noise = ("is not a recognized feature for this target", "1 warning generated",
             "warning generated when compiling for host")
    err = "\n".join(l for l in res.stderr.splitlines() if not any(n in l for n in noise))
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{res.stderr}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def _link(objs: list[str], lib_path: str) -> None:
    tmp = lib_path + f".tmp{os.getpid()}"
    cmd = [HIPCC, "--offload-arch=" + ARCH, "-shared", "-fPIC", "-o", tmp, *objs]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"link failed:\n{res.stderr}")
    os.replace(tmp, lib_path)


def build(extra_flags: list[str] | None = None, verbose: bool = False) -> str:
    """Compile and link unconditionally.  Returns the path of libsurel.so."""
    os.makedirs(BUILD_DIR, exist_ok=True)
    extra = list(extra_flags or [])
    srcs = sources()
    all_srcs = srcs + [MEMBENCH_SRC]
    wanted = {os.path.basename(s) + ".o" for s in all_srcs}
    for f in os.listdir(BUILD_DIR):           # objects of sources that no longer exist
        if f.endswith(".o") and f not in wanted:
            os.remove(os.path.join(BUILD_DIR, f))
    with concurrent.futures.ThreadPoolExecutor(max_workers=min(8, len(all_srcs))) as pool:
        objs = list(pool.map(lambda s: _compile(s, extra), all_srcs))
    _link(objs[:-1], LIB_PATH)
    _link(objs[-1:], MEMBENCH_LIB_PATH)
    if verbose:
        print(f"built {LIB_PATH} from {len(srcs)} sources, {MEMBENCH_LIB_PATH} from 1")
    return LIB_PATH


if __name__ == "__main__":
    build(verbose=True)
