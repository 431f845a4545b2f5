"""Build the HIP library in-tree: hipcc for gfx950, one object per source, one shared
object ``libba_hip.so`` next to this file."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libba_hip.so")
SOURCES = ["ba_api.hip", "ba_api_prompts.hip", "ba_api_cached.hip", "ba_probe.hip", "ba_plan.cpp", "reencode.hip", "rope_prepass.hip", "attention.hip", "attention_short.hip", "attention_bwd.hip", "head_pad.hip", "diag.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-fPIC", "-std=c++17",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         # MFMA results the softmax reads go to ordinary VGPRs; the allocator moves the
         # long-lived accumulators to AccVGPRs by itself.  Without this the attention core spills.
         "-mllvm", "-amdgpu-mfma-vgpr-form=1",
         "-Wno-unused-command-line-argument"]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    return "hipcc"


def _filter(stderr: str) -> str:
    # the host pass does not know the packed-fp32 feature and says so; harmless
    return "\n".join(l for l in stderr.splitlines() if "packed-fp32-ops" not in l)


def build(verbose: bool = False) -> str:
    os.makedirs(os.path.join(HERE, "_build"), exist_ok=True)
    objs = []

    def compile_one(src: str) -> str:
        obj = os.path.join(HERE, "_build", os.path.splitext(src)[0] + ".o")
        if src.endswith(".cpp"):
            # the host-side planner holds no device code: the host compiler takes it as it is
            cmd = [os.environ.get("CXX", "g++"), "-std=c++17", "-O2", "-fPIC", "-Wall", "-Wextra", "-Werror",
                   "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include", "-c", os.path.join(CSRC, src), "-o", obj]
        else:
            cmd = [_hipcc(), *FLAGS, *os.environ.get("BA_HIPCC_FLAGS", "").split(), "-c", os.path.join(CSRC, src), "-o", obj]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{_filter(r.stderr)}")
        if verbose and _filter(r.stderr).strip():
            print(_filter(r.stderr), file=sys.stderr)
        return obj

    with ThreadPoolExecutor(max_workers=len(SOURCES)) as ex:
        objs = list(ex.map(compile_one, SOURCES))
    cmd = [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{_filter(r.stderr)}")
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
