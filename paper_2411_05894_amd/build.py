"""Build libsssd_verify.so (hand-written HIP for gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libsssd_verify.so")
DRIVER = os.path.join(HERE, "step_driver")
SOURCES = ["api.hip", "attention.hip", "elementwise.hip", "stream_gemm.hip", "sampling.hip", "drafter.cpp"]
import shlex
FLAGS = shlex.split(os.environ.get("SSSD_EXTRA_HIPCC_FLAGS", "")) + ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wextra",
         # packed-fp32 VALU forms are kept off on the test machines
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _compile(src: str) -> str:
    obj = os.path.join(HERE, "_build", os.path.splitext(src)[0] + ".o")
    os.makedirs(os.path.dirname(obj), exist_ok=True)
    if src.endswith(".cpp"):   # host-only code (the drafter)
        subprocess.run(["g++", "-O2", "-std=c++17", "-fPIC", "-Wall", "-Wextra", "-c", os.path.join(CSRC, src), "-o", obj],
                       check=True)
    else:
        subprocess.run(["hipcc", *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj], check=True)
    return obj


def build(jobs: int = 4) -> str:
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(_compile, SOURCES))
    subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs], check=True)
    # native driver of the C ABI for profiler runs (plain executable, no Python in the process)
    subprocess.run(["hipcc", *FLAGS, os.path.join(HERE, "tools", "step_driver.hip"), "-o", DRIVER, "-L" + HERE,
                    "-lsssd_verify", "-Wl,-rpath,$ORIGIN"], check=True)
    return LIB


if __name__ == "__main__":
    print(build())
