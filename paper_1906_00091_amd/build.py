"""Builds libdlrm_hot.so (the method) and libdlrm_ceilings.so (measurement kernels a benchmark times;
a library of its own) in-tree with hipcc, for gfx950 only."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
INCLUDE = os.path.join(ROOT, "include")
LIB = os.path.join(PKG, "libdlrm_hot.so")
SOURCES = ["bwd_reduce_sgd.hip", "bwd_reduce_adagrad.hip", "bwd_reduce_sgd_weighted.hip",
           "bwd_reduce_adagrad_weighted.hip", "bwd_tail.hip", "bwd_partition.hip", "bwd_export.hip",
           "emb_bwd.hip", "emb_fwd.hip", "interact.hip", "pooled_interact.hip", "util.hip"]
CEIL_LIB = os.path.join(PKG, "libdlrm_ceilings.so")
CEIL_SOURCES = ["ceilings.hip"]

# -packed-fp32-ops: keep hipcc from forming packed fp32 VALU instructions.
HIPCC_FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-fno-gpu-rdc",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function", "-I", INCLUDE, "-I", CSRC,
]


def _hipcc() -> str:
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.isabs(c) and os.path.exists(c) or not os.path.isabs(c)):
            return c
    raise RuntimeError("hipcc not found")


def _stale() -> bool:
    if not os.path.exists(LIB) or not os.path.exists(CEIL_LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, f) for f in os.listdir(CSRC)] + [os.path.join(INCLUDE, f) for f in os.listdir(INCLUDE)]
    return any(os.path.getmtime(p) > t for p in deps)


def build(force: bool = True, verbose: bool = False) -> str:
    """Compile every HIP translation unit for gfx950 and link the shared library."""
    if not force and not _stale():
        return LIB
    hipcc = _hipcc()
    objdir = os.path.join(PKG, "_build")
    os.makedirs(objdir, exist_ok=True)

    def compile_one(src: str) -> str:
        obj = os.path.join(objdir, src.replace(".hip", ".o"))
        cmd = [hipcc] + HIPCC_FLAGS + ["-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("hipcc failed for %s:\n%s\n%s" % (src, r.stdout, r.stderr))
        # the host pass warns that it does not know -packed-fp32-ops: harmless, not shown
        return obj

    with ThreadPoolExecutor(max_workers=8) as ex:
        objs = list(ex.map(compile_one, SOURCES + CEIL_SOURCES))
    for lib, lib_objs in ((LIB, objs[:len(SOURCES)]), (CEIL_LIB, objs[len(SOURCES):])):
        cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib] + lib_objs
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("link failed:\n%s\n%s" % (r.stdout, r.stderr))
    return LIB


def build_host_sanitized(out_dir: str) -> str:
    """The method's library once more with AddressSanitizer and UndefinedBehaviorSanitizer on the HOST code
    (argument checks, launch geometry, workspace layout); the device code is compiled as usual (-O1 here:
    this build exists to be checked, not timed).  Returns the path of the library under out_dir."""
    hipcc = _hipcc()
    os.makedirs(out_dir, exist_ok=True)
    flags = [f for f in HIPCC_FLAGS if f != "-O3"] + ["-O1", "-g", "-Xarch_host", "-fsanitize=address", "-Xarch_host",
                                                       "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=all"]

    def compile_one(src: str) -> str:
        obj = os.path.join(out_dir, src.replace(".hip", ".o"))
        r = subprocess.run([hipcc] + flags + ["-c", os.path.join(CSRC, src), "-o", obj], capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("hipcc failed for %s:\n%s\n%s" % (src, r.stdout, r.stderr))
        return obj

    with ThreadPoolExecutor(max_workers=8) as ex:
        objs = list(ex.map(compile_one, SOURCES))
    lib = os.path.join(out_dir, "libdlrm_hot_hostsan.so")
    r = subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-fsanitize=address", "-fsanitize=undefined",
                        "-o", lib] + objs, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n%s\n%s" % (r.stdout, r.stderr))
    return lib


if __name__ == "__main__":
    print(build(force=True, verbose="-v" in sys.argv))
