"""Build libaemodel.so (the HIP library behind the C boundary) in-tree with hipcc for gfx950.

Usage: python -m paper_2602_17681_amd.build [--force]
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libaemodel.so")
SOURCES = ["ae_plan.cpp", "ae_elem.hip", "ae_noise.hip", "ae_conv_direct.hip", "ae_conv_mfma.hip", "ae_conv_thin.hip", "ae_conv_thin_mfma.hip", "ae_calib.hip", "ae_mx.hip", "ae_affine.hip", "ae_fold.hip", "ae_fused_small.hip", "ae_api.hip"]
HEADERS = [os.path.join(CSRC, "ae_internal.h"), os.path.join(CSRC, "ae_device.h"), os.path.join(CSRC, "ae_philox.h"), os.path.join(ROOT, "include", "aemodel.h")]
FLAGS = ["-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950", "-x", "hip",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-ffp-contract=off", "-fhip-fp32-correctly-rounded-divide-sqrt", "-Wall", "-Wno-unused-function",
         "-I" + os.path.join(ROOT, "include"), "-I" + CSRC]


def _compile(src, force):
    obj = os.path.join(OBJ, src + ".o")
    path = os.path.join(CSRC, src)
    deps = [path] + HEADERS
    if not force and os.path.exists(obj) and all(os.path.getmtime(obj) >= os.path.getmtime(d) for d in deps):
        return obj
    subprocess.run(["hipcc"] + FLAGS + ["-c", path, "-o", obj], check=True)
    return obj


def build(force=False, jobs=6):
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(lambda s: _compile(s, force), SOURCES))
    if force or not os.path.exists(LIB) or any(os.path.getmtime(o) > os.path.getmtime(LIB) for o in objs):
        subprocess.run(["hipcc", "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB] + objs, check=True)
    return LIB


if __name__ == "__main__":
    print(build(force="--force" in sys.argv))
