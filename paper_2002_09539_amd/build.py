"""Builds libols.so (the HIP kernels and the C boundary) for gfx950 with hipcc, in-tree.

Usage: python -m paper_2002_09539_amd.build   (cross-compiles without a GPU)
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.environ.get("OLS_BUILD_DIR", os.path.join(HERE, "_build"))
LIB = os.environ.get("OLS_BUILD_OUTPUT", os.path.join(HERE, "libols.so"))   # override: an alternative build

SOURCES = [
    "ols_api.hip",
    "kernels_update.hip",
    "kernels_mean.hip",
    "kernels_mix.hip",
    "kernels_lsq.hip",
    "kernels_mlp_head.hip",
    "kernels_gemm_f32.hip",
    "kernels_gemm_bf16.hip",
    "kernels_conv.hip",
    "kernels_bn.hip",
    "kernels_conv_bf16.hip",
]

# packed-fp32 VALU forms stay disabled for every device translation unit
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option",
    "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
]


def _hipcc():
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    raise RuntimeError("hipcc not found")


def _compile(src):
    obj = os.path.join(OBJ, src.replace(".hip", ".o"))
    extra = os.environ.get("OLS_EXTRA_FLAGS", "").split()   # e.g. -DOLS_TUNING_VARIANTS for a measurement build
    cmd = [_hipcc(), *FLAGS, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s\n%s" % (src, res.stdout, res.stderr))
    noise = "unknown target feature"  # hipcc's host pass does not know the packed-fp32 switch; harmless
    warn = "\n".join(l for l in res.stderr.splitlines() if l.strip() and noise not in l and "-packed-fp32-ops" not in l)
    return obj, warn


def build_library(verbose=True, jobs=8):
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=jobs) as pool:
        results = list(pool.map(_compile, SOURCES))
    objs = [o for o, _ in results]
    if verbose:
        for _, w in results:
            if w:
                print(w, file=sys.stderr)
    cmd = [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("link failed:\n%s\n%s" % (res.stdout, res.stderr))
    return LIB


if __name__ == "__main__":
    print(build_library())
