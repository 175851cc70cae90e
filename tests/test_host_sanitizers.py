"""Everything of the build that runs on the host -- the sizing and launch planning behind the C ABI, the
drafter, the C oracle -- compiled with AddressSanitizer and UndefinedBehaviorSanitizer (host code only;
device code is compiled as usual and never runs here) and driven by tests/sanitize/host_san.cpp."""
import os
import shutil
import subprocess
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2411_05894_amd", "csrc")
OUT = os.path.join(ROOT, "paper_2411_05894_amd", "_build", "host_san")
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-g", "-O1"]
HIP = ["hipcc", "--offload-arch=gfx950", "-std=c++17", "-fno-gpu-sanitize", "-Xclang", "-target-feature", "-Xclang",
       "-packed-fp32-ops", *SAN]


def _compile(job):
    cmd, obj = job
    subprocess.run(cmd + ["-o", obj], check=True, stdout=subprocess.PIPE, stderr=subprocess.STDOUT)
    return obj


@pytest.mark.timeout(900)
def test_host_code_is_clean_under_asan_and_ubsan():
    if shutil.which("hipcc") is None:
        pytest.skip("hipcc not on PATH")
    os.makedirs(OUT, exist_ok=True)
    jobs = []
    for src in ("api.hip", "attention.hip", "elementwise.hip", "stream_gemm.hip", "sampling.hip"):
        jobs.append((HIP + ["-c", os.path.join(CSRC, src)], os.path.join(OUT, src + ".o")))
    jobs.append((HIP + ["-c", "-x", "c++", os.path.join(CSRC, "drafter.cpp")], os.path.join(OUT, "drafter.o")))
    jobs.append((HIP + ["-c", "-x", "c++", os.path.join(ROOT, "tests", "sanitize", "host_san.cpp")], os.path.join(OUT, "host_san.o")))
    jobs.append((["gcc", "-std=c11", *SAN, "-c", os.path.join(ROOT, "oracle", "sssd_oracle.c")], os.path.join(OUT, "oracle.o")))
    with ThreadPoolExecutor(max_workers=4) as ex:
        objs = list(ex.map(_compile, jobs))
    exe = os.path.join(OUT, "host_san")
    subprocess.run(["hipcc", "--offload-arch=gfx950", "-fno-gpu-sanitize", *SAN, *objs, "-lm", "-o", exe], check=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe], env=env, stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True, timeout=600)
    print(run.stdout)
    print(run.stderr[-4000:])
    assert run.returncode == 0, run.stderr[-4000:]
    assert "ERROR: AddressSanitizer" not in run.stderr and "runtime error:" not in run.stderr
    assert "host self-test passed" in run.stdout
