"""Builds libadasd.so (HIP, gfx950 only) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
BUILD = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libadasd.so")
SOURCES = ["stats.hip", "stats_fused.hip", "decide.hip", "sample.hip", "draft.hip", "shard.hip", "diag.hip", "api.hip"]
HEADERS = [os.path.join(CSRC, h) for h in ("device_common.h", "internal.h", "decide_device.h",
                                             "sample_device.h", "stats_device.h")] + [
           os.path.join(os.path.dirname(HERE), "include", "adasd.h")]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall",
         # fused multiply-adds only where the source says fmaf: the same expression must round the
         # same way in every inlined copy (a recomputed partial result has to be bit-identical)
         "-ffp-contract=off",
         # packed-FP32 instructions are kept out of every kernel of this library
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _compile(src: str) -> str:
    obj = os.path.join(BUILD, src.replace(".hip", ".o"))
    cmd = [HIPCC, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = ("packed-fp32-ops", "warning generated", "warnings generated")
    msgs = [l for l in res.stderr.splitlines() if l.strip() and not any(n in l for n in noise)]
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{res.stderr}")
    if msgs:
        print("\n".join(msgs))
    return obj


def build(force: bool = True, jobs: int = 4) -> str:
    """Compile every HIP source and link the shared library.  With force=False the build is
    skipped when the library is newer than every source and header."""
    os.makedirs(BUILD, exist_ok=True)
    deps = [os.path.join(CSRC, s) for s in SOURCES] + HEADERS
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= max(map(os.path.getmtime, deps)):
        return LIB
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(_compile, SOURCES))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"link failed:\n{res.stderr}")
    return LIB


if __name__ == "__main__":
    print(build())
