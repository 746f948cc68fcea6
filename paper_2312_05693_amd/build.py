"""Builds libagq.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libagq.so")
SOURCES = ["agq_api.cpp", "agq_quant.hip", "agq_gemm_decode.hip", "agq_gemm_tiled.hip", "agq_attn.hip", "agq_trip.hip", "agq_attn_qk.hip",
           "agq_block.hip", "agq_block_api.cpp", "agq_static.hip", "agq_gemm_chain.hip"]
PROBE_LIB = os.path.join(HERE, "libagq_probe.so")     # bench.py's measurement aid, a library of its own
PROBE_SOURCE = "agq_probe.hip"
HEADERS = ["agq_device.h", "agq_internal.h", os.path.join("..", "..", "include", "agq.h")]
FLAGS = ["-O3", "--offload-arch=gfx950", "-fPIC", "-std=c++17", "-x", "hip",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _newest(paths):
    return max(os.path.getmtime(p) for p in paths)


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, os.path.splitext(src)[0] + ".o")
    cmd = ["hipcc", *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s" % (src, r.stderr))
    return obj


def build(force: bool = True, jobs: int = 4) -> str:
    """Compiles every source and links the shared library.  With force=False an
    up-to-date library is kept."""
    deps = [os.path.join(CSRC, s) for s in SOURCES + [PROBE_SOURCE]] + [os.path.join(CSRC, h) for h in HEADERS]
    if not force and os.path.exists(LIB) and os.path.exists(PROBE_LIB) and \
            min(os.path.getmtime(LIB), os.path.getmtime(PROBE_LIB)) >= _newest(deps):
        return LIB
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(_compile, SOURCES + [PROBE_SOURCE]))
    probe_obj = objs.pop()
    r = subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", PROBE_LIB, probe_obj],
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link of the probe library failed:\n%s" % r.stderr)
    r = subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs],
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n%s" % r.stderr)
    return LIB


if __name__ == "__main__":
    print(build())
