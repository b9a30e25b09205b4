"""Builds the HIP library in-tree for gfx950: one object per translation unit, in parallel."""
from __future__ import annotations

import glob
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OUT = os.path.join(HERE, "libd2mhe.so")
OBJ = os.path.join(HERE, "_build")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def _compile(src):
    obj = os.path.join(OBJ, os.path.basename(src) + ".o")
    subprocess.check_call(["hipcc", *FLAGS, "-c", src, "-o", obj], stderr=subprocess.STDOUT)
    return obj


def build_library(jobs: int = 8) -> str:
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=jobs) as pool:
        objs = list(pool.map(_compile, sources()))
    subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", OUT, *objs])
    return OUT


DEVICE_CHECK_SRC = os.path.join(os.path.dirname(HERE), "tests", "arith_device_check.hip")
DEVICE_CHECK_EXE = os.path.join(os.path.dirname(HERE), "tests", "_build", "arith_device_check")


def build_device_check() -> str:
    """The GPU-side check of the arithmetic policies (tests/arith_device_check.hip): a stand-alone program."""
    os.makedirs(os.path.dirname(DEVICE_CHECK_EXE), exist_ok=True)
    subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-O2", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
                           "-packed-fp32-ops", "-o", DEVICE_CHECK_EXE, DEVICE_CHECK_SRC], stderr=subprocess.STDOUT)
    return DEVICE_CHECK_EXE
