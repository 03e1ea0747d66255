"""Compiles libea.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree.

    python -m paper_2510_00636_amd.build
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libea.so")
SOURCES = ["ea_host.cpp", "ea_api.hip", "ea_stats.hip", "ea_score.hip", "ea_score_d64.hip", "ea_score_d128.hip", "ea_score_d128b.hip",
           "ea_score_d256.hip", "ea_score_fp8.hip", "ea_score_fp8b.hip", "ea_score_hw.hip", "ea_select.hip",
           "ea_compact.hip", "ea_baselines.hip", "ea_frontend.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
# packed-fp32 instructions are switched off for the device pass (the host pass warns that it
# does not know the feature; harmless)
# The wave-aggregation of atomics is switched off as well: it rewrites "lane 0 draws a ticket" into
# code that reads the returned value at once, i.e. waits for the atomic where it is issued.
# Matrix-core results are kept in ordinary vector registers where they fit (the dot products that
# follow read them there directly: otherwise every accumulator value takes a copy out of the
# accumulation registers first; score pass at d=256: 255 -> 240 us per layer).
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-mllvm", "-amdgpu-atomic-optimizer-strategy=None",
         "-mllvm", "-amdgpu-mfma-vgpr-form"]


def _compile(src):
    obj = os.path.join(OBJ, src + ".o")
    cmd = [HIPCC, *FLAGS, "-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed on %s:\n%s\n%s" % (src, r.stdout, r.stderr))
    warn = [l for l in r.stderr.splitlines() if "warning" in l and "packed-fp32-ops" not in l]
    return obj, warn


def build_lib(verbose=True):
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 2)) as ex:
        res = list(ex.map(_compile, SOURCES))
    objs = [o for o, _ in res]
    if verbose:
        for _, w in res:
            for line in w:
                print(line, file=sys.stderr)
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n%s\n%s" % (r.stdout, r.stderr))
    return LIB


if __name__ == "__main__":
    print(build_lib())
