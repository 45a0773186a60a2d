"""Build libl2kv.so (HIP, gfx950 only) in-tree with hipcc.

    python -m paper_2406_11430_amd.build          # compile every source, link

The library is never built implicitly by the binding on import of a compute
call: callers load what is there and fail loudly if nothing is.
"""
from __future__ import annotations

import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB_PATH = os.path.join(HERE, "libl2kv.so")
OBJ_DIR = os.path.join(HERE, "_build")
SOURCES = ["decode_attn_bf16_128.hip", "decode_attn_bf16_256.hip", "decode_attn_bf16_64.hip",
           "decode_attn_f32_128.hip", "decode_attn_f32_64.hip", "api.hip", "norms.hip", "select.hip", "compact.hip", "decode_attn.hip",
           "stream.hip", "alr.hip"]
ARCH = "gfx950"

# -packed-fp32-ops is switched off on purpose: the compiler must not form
# v_pk_*_f32 from the scalar fp32 code of these kernels.
HIPCC_FLAGS = [
    "--offload-arch=" + ARCH, "-O3", "-std=c++17", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wextra", "-Wno-unused-command-line-argument",
]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found (set HIPCC or install ROCm)")


def _compile(src: str, extra, obj_dir: str = OBJ_DIR) -> str:
    obj = os.path.join(obj_dir, os.path.splitext(src)[0] + ".o")
    cmd = [hipcc(), *HIPCC_FLAGS, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    # the host pass warns that it does not know the packed-fp32 feature: harmless
    err = "\n".join(l for l in res.stderr.splitlines()
                    if "packed-fp32-ops" not in l and "is not a recognized feature" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s" % (src, err))
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build_library(extra_flags=(), jobs: int = 8, out: str = LIB_PATH, obj_dir: str = OBJ_DIR) -> str:
    """Compile every kernel source for gfx950 and link the shared library
    (libl2kv.so in the package unless `out` names another file)."""
    os.makedirs(obj_dir, exist_ok=True)
    with ThreadPoolExecutor(max_workers=max(1, jobs)) as pool:
        objs = list(pool.map(lambda s: _compile(s, list(extra_flags), obj_dir), SOURCES))
    tmp = out + ".tmp.%d" % os.getpid()
    cmd = [hipcc(), "--offload-arch=" + ARCH, "-shared", "-fPIC", *objs, "-o", tmp]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("link failed:\n" + res.stderr)
    os.replace(tmp, out)
    return out


C_DRIVER_SRC = os.path.join(os.path.dirname(HERE), "tests", "abi_c", "l2kv_c_driver.c")
C_DRIVER_BIN = os.path.join(os.path.dirname(HERE), "tests", "abi_c", "l2kv_c_driver")


def build_c_driver() -> str:
    """Compile the plain-C program that drives the library with hipMalloc memory (gcc, C99) and
    link it against libl2kv.so and the HIP runtime.  Needs the library built first."""
    rocm = os.path.dirname(os.path.dirname(hipcc()))
    cmd = ["gcc", "-std=c99", "-O1", "-Wall", "-D__HIP_PLATFORM_AMD__", "-I" + os.path.join(rocm, "include"),
           "-I" + os.path.join(os.path.dirname(HERE), "include"), C_DRIVER_SRC, "-o", C_DRIVER_BIN,
           "-L" + HERE, "-ll2kv", "-L" + os.path.join(rocm, "lib"), "-lamdhip64",
           "-Wl,-rpath,$ORIGIN/../../paper_2406_11430_amd", "-Wl,-rpath," + os.path.join(rocm, "lib")]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("gcc failed for the C driver:\n" + res.stderr)
    return C_DRIVER_BIN


if __name__ == "__main__":
    print(build_library(sys.argv[1:]))
    print(build_c_driver())
