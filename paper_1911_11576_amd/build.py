"""Builds the HIP library for gfx950:  python -m paper_1911_11576_amd.build

Every source under csrc/ is compiled with hipcc (device code for gfx950 only) and linked
into libfusionstitch.so next to this file, together with the HIP run-time compiler that
the kernel generator of the elementwise schedule uses.  hipcc cross-compiles without a GPU.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.environ.get("FS_OBJ_DIR", os.path.join(HERE, "_build"))
LIB = os.environ.get("FS_LIB_OUT", os.path.join(HERE, "libfusionstitch.so"))

SOURCES = ["api.cpp", "graph.cpp", "match.cpp", "row_stitch.hip", "row_stitch_f32.hip", "row_stitch_f16.hip", "row_stitch_bf16.hip", "row_team.hip", "row_block.hip", "lnbwd_stitch.hip",
           "attn_stitch.hip", "attn_stitch_f16.hip", "attn_stitch_bf16.hip", "per_op.hip", "ew_stitch.hip", "ew_codegen.cpp", "row_codegen.cpp", "shared_plan.cpp", "fusion_plan.cpp", "util.hip", "launch_static.hip"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-mllvm", "-amdgpu-mfma-vgpr-form",      # MFMA results in ordinary registers: no copies to and from the accumulation file
         "-Wall", "-Wno-unused-function", "-Wno-unknown-attributes"]


def _compile(src):
    obj = os.path.join(OBJ, src.rsplit(".", 1)[0] + ".o")
    extra = os.environ.get("FS_EXTRA_FLAGS", "").split()
    cmd = [HIPCC, *FLAGS, *extra, "-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    # the host pass does not know the device-only target feature; that message is harmless
    log = "\n".join(l for l in (r.stdout + r.stderr).splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{log}")
    return obj, log


def build(verbose=False, jobs=None):
    os.makedirs(OBJ, exist_ok=True)
    jobs = jobs or min(8, os.cpu_count() or 1)
    with ThreadPoolExecutor(jobs) as ex:
        results = list(ex.map(_compile, SOURCES))
    for (obj, log), src in zip(results, SOURCES):
        if verbose and log.strip():
            print(f"--- {src}\n{log}")
    cmd = [HIPCC, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB, *[o for o, _ in results], "-lhiprtc"]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stdout + r.stderr)
    return LIB


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
