"""Builds libcoopt_attn.so and the benchmark's libcoopt_probe.so (HIP, gfx950 only) in-tree with hipcc.

    python -m paper_2602_09323_amd.build [--force]

hipcc cross-compiles without a GPU.  Objects go to ``_build/`` next to this file; the shared
library lands beside the Python binding so that it travels with the source tree.
"""
from __future__ import annotations

import concurrent.futures
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
BUILD = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libcoopt_attn.so")
PROBE_LIB = os.path.join(HERE, "libcoopt_probe.so")      # measurement aid, not the product
SOURCES = ["kv_write.hip", "decode.hip", "decode_flat.hip", "prefill.hip", "gather.hip"]
PROBE_SOURCES = ["probe.hip"]
HEADERS = [os.path.join(CSRC, h) for h in ("common.hpp", "attn_tile.hpp", "kv_quant.hpp",
                                          "decode_internal.hpp")] + [
    os.path.join(ROOT, "include", "coopt_attn.h"), os.path.join(ROOT, "include", "coopt_probe.h")]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc",
         "-I" + os.path.join(ROOT, "include"),
         # packed-FP32 VALU forms are kept out of the generated code on purpose
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument"]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    return "hipcc"


def _compile(src: str) -> str:
    obj = os.path.join(BUILD, os.path.splitext(src)[0] + ".o")
    cmd = [_hipcc(), *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    # the host pass does not know the device-only target feature; that warning is expected
    err = "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def needs_build() -> bool:
    if not os.path.exists(LIB) or not os.path.exists(PROBE_LIB):
        return True
    newest = max(os.path.getmtime(p)
                 for p in [os.path.join(CSRC, s) for s in SOURCES + PROBE_SOURCES] + HEADERS)
    return min(os.path.getmtime(LIB), os.path.getmtime(PROBE_LIB)) < newest


def build(force: bool = True) -> str:
    """Compile every HIP source for gfx950 and link the shared library.  Returns its path."""
    if not force and not needs_build():
        return LIB
    os.makedirs(BUILD, exist_ok=True)
    with concurrent.futures.ThreadPoolExecutor(max_workers=6) as pool:
        objs = list(pool.map(_compile, SOURCES + PROBE_SOURCES))
    for lib, n in ((LIB, objs[:len(SOURCES)]), (PROBE_LIB, objs[len(SOURCES):])):
        cmd = [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-fno-gpu-rdc", "-o", lib, *n]
        res = subprocess.run(cmd, capture_output=True, text=True)
        if res.returncode != 0:
            raise RuntimeError("link failed:\n" + res.stderr)
    return LIB


if __name__ == "__main__":
    print(build(force=True))
