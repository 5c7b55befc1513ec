"""Builds libmtsched.so (gfx950 only) in-tree with hipcc.  No fallback: a missing compiler is an error."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libmtsched.so")

DEVICE_SOURCES = ["kernels_direct.hip", "kernels_igemm.hip", "kernels_stem.hip", "kernels_rowb.hip", "kernels_patch.hip"]
HOST_SOURCES = ["sched_core.cpp", "runtime.cpp"]
COMMON = ["-O3", "-fPIC", "-std=c++20", "-Wall", "-Wno-unused-function"]
# packed-fp32 code generation is switched off for all device code
DEVICE_FLAGS = ["--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _hipcc():
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    raise RuntimeError("hipcc not found")


def _compile(src, extra, obj_dir=None):
    out = os.path.join(obj_dir or OBJ, os.path.basename(src) + ".o")
    cmd = [_hipcc(), "-c", os.path.join(CSRC, src), "-o", out] + COMMON + extra
    r = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in r.stderr.splitlines() if noise not in l)
    if r.returncode != 0:
        raise RuntimeError("compile failed: %s\n%s" % (" ".join(cmd), err))
    if err.strip():
        sys.stderr.write(err + "\n")
    return out


# host-side sanitizers (address + undefined behaviour) for the two host sources; device code is never instrumented
SANITIZE_HOST = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-omit-frame-pointer", "-g"]


def build(verbose=False, lib=None, sanitize=False):
    """sanitize=True builds the host objects with AddressSanitizer and UBSan into `lib` (give another path than the
    product library's): the CPU-only tests can then run against it with the sanitizer runtime preloaded, e.g.
    MTSCHED_LIB=<lib> LD_PRELOAD="$LD_PRELOAD:$(clang -print-file-name=libclang_rt.asan-x86_64.so)" pytest -m "not gpu"."""
    global LIB
    out = lib or LIB
    if not sanitize and lib:
        LIB = lib
    obj_dir = OBJ + ("_asan" if sanitize else "")
    os.makedirs(obj_dir, exist_ok=True)
    host_extra = ["-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include"] + (SANITIZE_HOST if sanitize else [])
    jobs = [(s, DEVICE_FLAGS, obj_dir) for s in DEVICE_SOURCES] + [(s, host_extra, obj_dir) for s in HOST_SOURCES]
    with ThreadPoolExecutor(max_workers=4) as ex:
        objs = list(ex.map(lambda j: _compile(*j), jobs))
    cmd = [_hipcc(), "-shared", "-fPIC", "-o", out] + objs + ["--offload-arch=gfx950"]
    if sanitize:
        cmd += ["-fsanitize=address", "-fsanitize=undefined", "-fno-gpu-sanitize", "-shared-libsan"]
    subprocess.check_call(cmd)
    if sanitize:
        return out
    if verbose:
        print("built", LIB)
    return LIB


def lib_path():
    return LIB


if __name__ == "__main__":
    if "--sanitize" in sys.argv:
        print("built", build(lib=os.path.join(HERE, "libmtsched_asan.so"), sanitize=True))
    else:
        build(verbose=True)
