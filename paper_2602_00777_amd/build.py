"""Builds ``libhylra.so`` (HIP, gfx950) in-tree with hipcc.

``python -m paper_2602_00777_amd.build`` compiles every translation unit under
``csrc/`` for gfx950 and links them into ``paper_2602_00777_amd/libhylra.so``.
hipcc cross-compiles, so no GPU is needed to build.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
BUILD = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libhylra.so")
SOURCES = ["api.hip", "full_attn_d64.hip", "full_attn_d128.hip", "reuse_attn_d64.hip",
           "reuse_attn_d128.hip", "finalize.hip", "topk.hip", "reuse_mfma.hip", "reuse_mfma2.hip", "full_mfma.hip", "full_mfma2.hip", "policy.hip", "ragged_plan.hip", "offload.hip"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
# packed-FP32 code generation is switched off on purpose (device pass only)
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _compile(src: str) -> str:
    obj = os.path.join(BUILD, src.replace(".hip", ".o"))
    cmd = [HIPCC] + FLAGS + ["-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "not a recognized feature" not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s" % (src, err))
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(jobs: int = 8) -> str:
    """Compile and link.  HYLRA_EXTRA_FLAGS adds compiler flags and HYLRA_LIB_OUT redirects
    the output (both only for tuning builds; the product build uses neither)."""
    global BUILD, LIB
    extra = os.environ.get("HYLRA_EXTRA_FLAGS", "").split()
    if extra:
        FLAGS.extend(extra)
        LIB = os.environ.get("HYLRA_LIB_OUT", LIB)
        BUILD = BUILD + "_extra"
    os.makedirs(BUILD, exist_ok=True)
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(_compile, SOURCES))
    tmp = LIB + ".tmp%d" % os.getpid()
    link_extra = [f for f in extra if f.startswith("-fgpu-rdc")]
    r = subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC"] + link_extra + ["-o", tmp] + objs,
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build())
