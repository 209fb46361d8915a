"""Build libpolydl.so: every HIP source under csrc/ compiled for gfx950 and linked in-tree."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libpolydl.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         # matrix-core results stay in ordinary vector registers: without this the compiler keeps
         # the accumulators in the accumulation registers inside the reduction loop and copies all
         # of them out and back in every stage
         "-mllvm", "-amdgpu-mfma-vgpr-form"]


HOST_FLAGS = ["-O2", "-std=c++17", "-fPIC", "-Wall", "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include"]


def sources():
    """.hip files hold kernels and their launchers; .cpp files are host-only code."""
    return sorted(f for f in os.listdir(CSRC) if f.endswith(".hip") or f.endswith(".cpp"))


def _compile(src):
    obj = os.path.join(OBJ, src[:-4] + ".o")
    if src.endswith(".cpp"):
        cmd = ["g++"] + HOST_FLAGS
    else:
        cmd = [HIPCC] + FLAGS
    r = subprocess.run(cmd + ["-c", os.path.join(CSRC, src), "-o", obj], capture_output=True, text=True)
    # the host pass does not know the device-only target feature and says so on every file
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError("compiler failed on %s:\n%s" % (src, err))
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(jobs=None):
    os.makedirs(OBJ, exist_ok=True)
    jobs = jobs or min(8, os.cpu_count() or 1)
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(_compile, sources()))
    subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs, check=True)
    return LIB


if __name__ == "__main__":
    print(build())
