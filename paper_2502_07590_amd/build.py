"""Builds libdsv.so (hand-written HIP for gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
OBJ = os.path.join(PKG, "_build")
LIB = os.path.join(PKG, "libdsv.so")
SOURCES = ("api.hip", "stage1.hip", "stage1_emit.hip", "stage1_window.hip", "stage2.hip", "stage2_split.hip", "validate.hip", "grouped.hip", "measure.hip", "predictor.hip", "profiler.hip")

# packed-fp32 instructions are disabled for device code (a requirement of the test machines).
HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
               "-munsafe-fp-atomics",                  # LDS float adds as one instruction (the profiler's mass histograms)
               "-mllvm", "-amdgpu-mfma-vgpr-form=1",   # MFMA results straight into VGPRs (no AccVGPR copies)
               "-Wall", "-Wno-unused-function", "-Wno-unknown-attributes",
               "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


def build_library(verbose: bool = False, extra_flags=(), out: str = LIB) -> str:
    """Compile every source for gfx950 and link libdsv.so.  Always recompiles.

    extra_flags / out: for tuning builds (e.g. ("-DDSV_LPR_DQ=8",) into another file name); the
    environment variable DSV_HIPCC_FLAGS adds flags as well."""
    os.makedirs(OBJ, exist_ok=True)
    hipcc = _hipcc()
    extra = list(extra_flags) + os.environ.get("DSV_HIPCC_FLAGS", "").split()

    def compile_one(src: str) -> str:
        obj = os.path.join(OBJ, src.replace(".hip", ".o"))
        cmd = [hipcc, *HIPCC_FLAGS, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
        res = subprocess.run(cmd, capture_output=True, text=True)
        noise = "is not a recognized feature for this target"
        err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
        if res.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{err}")
        if verbose and err.strip():
            print(err)
        return obj

    with ThreadPoolExecutor(max_workers=len(SOURCES)) as ex:
        objs = list(ex.map(compile_one, SOURCES))
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", out, *objs]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"link failed:\n{res.stderr}")
    return out


if __name__ == "__main__":
    print(build_library(verbose=True))
