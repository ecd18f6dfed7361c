"""Builds libicecache.so (HIP kernels + C ABI, gfx950 only) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libicecache.so")
OBJ_DIR = os.path.join(ROOT, "_build")
SOURCES = ["ice_api.hip", "ice_build.hip", "ice_decode.hip", "ice_hier.hip", "ice_peaks.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
         # packed-fp32 instruction selection is switched off for all device code
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         # the first 16 dwords of a kernel's arguments are handed over in scalar registers at wave start
         "-mllvm", "-amdgpu-kernarg-preload-count=16",
         "-Wall", "-Wno-unused-result", "-Wno-inline-asm"]


def build_library(verbose: bool = False, extra_flags=(), lib_path: str = LIB, obj_dir: str = OBJ_DIR) -> str:
    """Compile every source (always, also when a library is already there) and link.  extra_flags,
    lib_path and obj_dir are for variants that must not replace the product library (the build with
    in-kernel time stamps of phase_stamps.py)."""
    os.makedirs(obj_dir, exist_ok=True)

    def compile_one(src: str) -> str:
        obj = os.path.join(obj_dir, src.replace(".hip", ".o"))
        cmd = [HIPCC, *FLAGS, *extra_flags, "-c", os.path.join(CSRC, src), "-o", obj]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("hipcc failed for %s:\n%s" % (src, r.stderr))
        if verbose:
            print(r.stderr)
        return obj

    with ThreadPoolExecutor(max_workers=len(SOURCES)) as ex:
        objs = list(ex.map(compile_one, SOURCES))
    r = subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib_path, *objs],
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    return lib_path


if __name__ == "__main__":
    print(build_library(verbose=True))
