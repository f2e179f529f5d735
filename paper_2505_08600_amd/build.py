"""Builds libsd.so (the HIP library) in-tree with hipcc for gfx950."""
from __future__ import annotations

import glob
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libsd.so")
OBJ = os.path.join(HERE, "_build")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
# Keeps MFMA operands and results in the architectural registers where they fit: without it the row-blocked GEMM's
# main loop carries ~50 AGPR <-> VGPR moves per 96 MFMAs, and vector instructions next to MFMAs are not free on this
# part (batch-32 verify and prefill 1-1.5 % faster with it).  An option of the compiler's AMDGPU backend, not of the
# driver: a compiler that does not know it gets the same sources without it.
OPTIONAL_FLAGS = ["-mllvm", "-amdgpu-mfma-vgpr-form=1"]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def build_lib(verbose: bool = False) -> str:
    os.makedirs(OBJ, exist_ok=True)
    srcs = sources()
    hdrs = glob.glob(os.path.join(CSRC, "*.h")) + glob.glob(os.path.join(HERE, "..", "include", "*.h"))
    newest_hdr = max(os.path.getmtime(h) for h in hdrs)

    def compile_one(src):
        obj = os.path.join(OBJ, os.path.splitext(os.path.basename(src))[0] + ".o")
        if os.path.exists(obj) and os.path.getmtime(obj) > max(os.path.getmtime(src), newest_hdr):
            return obj
        cmd = [HIPCC] + FLAGS + OPTIONAL_FLAGS + ["-c", src, "-o", obj]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0 and "amdgpu-mfma-vgpr-form" in r.stderr:
            r = subprocess.run([HIPCC] + FLAGS + ["-c", src, "-o", obj], capture_output=True, text=True)
        err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{err}")
        if verbose and err.strip():
            print(err, file=sys.stderr)
        return obj

    with ThreadPoolExecutor(max_workers=4) as ex:
        objs = list(ex.map(compile_one, srcs))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    return LIB


def clean():
    for f in glob.glob(os.path.join(OBJ, "*.o")):
        os.remove(f)


if __name__ == "__main__":
    if "--clean" in sys.argv:
        clean()
    print(build_lib(verbose=True))
