"""Build libsprnn.so (HIP, gfx950) in-tree with hipcc.  Run as ``python -m paper_1804_10223_amd.build``."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libsprnn.so")
PROBE_LIB = os.path.join(HERE, "libsprnn_probe.so")
SOURCES = ["sprnn_pack.cpp", "sprnn_kernels.hip", "sprnn_kernels_bwd.hip", "sprnn_kernels_gated_bwd.hip",
           "sprnn_kernels_timeline.hip", "sprnn_kernels_overlap.hip", "sprnn_kernels_short.hip", "sprnn_kernels_pool.hip", "sprnn_kernels_pool_bwd.hip", "sprnn_kernels_pool_bwd_grad.hip", "sprnn_project.hip", "sprnn_api.hip"]
PROBE_SOURCES = ["sprnn_probe.hip"]
FLAGS = ["-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950", "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument"]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


def _filter(stderr: str) -> str:
    keep = [ln for ln in stderr.splitlines() if "packed-fp32-ops" not in ln and "is not a recognized feature" not in ln]
    return "\n".join(keep)


def build_library(verbose: bool = False) -> str:
    """Compile every source for gfx950 and link libsprnn.so and libsprnn_probe.so next to this file."""
    hipcc = _hipcc()
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)

    def compile_one(src: str) -> str:
        obj = os.path.join(objdir, src + ".o")
        cmd = [hipcc, *FLAGS, "-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj]
        r = subprocess.run(cmd, capture_output=True, text=True)
        msg = _filter(r.stderr)
        if r.returncode != 0:
            raise RuntimeError("hipcc failed for %s:\n%s" % (src, msg))
        if verbose and msg.strip():
            print(msg, file=sys.stderr)
        return obj

    with ThreadPoolExecutor(max_workers=len(SOURCES) + len(PROBE_SOURCES)) as ex:
        objs = list(ex.map(compile_one, SOURCES + PROBE_SOURCES))
    for lib, part in ((LIB, objs[:len(SOURCES)]), (PROBE_LIB, objs[len(SOURCES):])):
        r = subprocess.run([hipcc, "-shared", "-fPIC", "--offload-arch=gfx950", *part, "-o", lib], capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("link failed:\n" + _filter(r.stderr))
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
