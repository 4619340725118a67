"""Builds libiolbconv.so (the C-ABI library) for gfx950 with hipcc, in-tree."""
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libiolbconv.so")
OBJ_DIR = os.path.join(ROOT, "_build")

SOURCES = ["api.hip", "direct_fma.hip", "direct_thin.hip", "direct_mfma.hip", "direct_mfma_hwc.hip", "pointwise_mfma.hip", "wino.hip", "wino_fused.hip", "wino_fused_mfma.hip", "wino_fused_rows.hip", "probe.hip", "tune.cpp"]
# packed fp32 VALU forms are disabled on purpose: plain v_fma_f32 only
DEVICE_FLAGS = ["--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
COMMON = ["-O3", "-std=c++17", "-fPIC", "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
          "-Wno-unused-command-line-argument"]


def _compile(src):
    obj = os.path.join(OBJ_DIR, src + ".o")
    cmd = ["hipcc"] + COMMON + (DEVICE_FLAGS if src.endswith(".hip") else ["-x", "c++"]) + \
          ["-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed on %s:\n%s" % (src, r.stdout))
    return obj


def build_library(jobs=6):
    """Compile every source and link the shared library; always recompiles."""
    os.makedirs(OBJ_DIR, exist_ok=True)
    with ThreadPoolExecutor(max_workers=jobs) as pool:
        objs = list(pool.map(_compile, SOURCES))
    cmd = ["hipcc", "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB] + objs
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stdout)
    return LIB


if __name__ == "__main__":
    print(build_library())
