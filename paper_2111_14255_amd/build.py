"""Builds libmtsched.so (gfx950 only) in-tree with hipcc.  No fallback: a missing compiler is an error."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libmtsched.so")

DEVICE_SOURCES = ["kernels_direct.hip", "kernels_igemm.hip"]
HOST_SOURCES = ["sched_core.cpp", "runtime.cpp"]
COMMON = ["-O3", "-fPIC", "-std=c++20", "-Wall", "-Wno-unused-function"]
# packed-fp32 code generation is switched off for all device code
DEVICE_FLAGS = ["--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _hipcc():
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    raise RuntimeError("hipcc not found")


def _compile(src, extra):
    out = os.path.join(OBJ, os.path.basename(src) + ".o")
    cmd = [_hipcc(), "-c", os.path.join(CSRC, src), "-o", out] + COMMON + extra + os.environ.get("MT_EXTRA_DEFS", "").split()
    r = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in r.stderr.splitlines() if noise not in l)
    if r.returncode != 0:
        raise RuntimeError("compile failed: %s\n%s" % (" ".join(cmd), err))
    if err.strip():
        sys.stderr.write(err + "\n")
    return out


def build(verbose=False, lib=None):
    global LIB
    if lib:
        LIB = lib
    os.makedirs(OBJ, exist_ok=True)
    jobs = [(s, DEVICE_FLAGS) for s in DEVICE_SOURCES] + [(s, ["-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include"]) for s in HOST_SOURCES]
    with ThreadPoolExecutor(max_workers=4) as ex:
        objs = list(ex.map(lambda j: _compile(*j), jobs))
    cmd = [_hipcc(), "-shared", "-fPIC", "-o", LIB] + objs + ["--offload-arch=gfx950"]
    subprocess.check_call(cmd)
    if verbose:
        print("built", LIB)
    return LIB


def lib_path():
    return LIB


if __name__ == "__main__":
    build(verbose=True)
