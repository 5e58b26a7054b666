"""Builds libluvc.so (the gfx950 kernels + C ABI) in-tree with hipcc."""
from __future__ import annotations

import glob
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
# LUVC_HOST_SANITIZE=1: the host half of the library (argument checks, planners, ragged batching) is built with
# AddressSanitizer and UndefinedBehaviorSanitizer into a file of its own; device code is unchanged.  The process that
# loads it needs clang's libclang_rt.asan-x86_64.so preloaded, see README.
SANITIZE = os.environ.get("LUVC_HOST_SANITIZE", "") not in ("", "0")
LIB = os.path.join(HERE, "libluvc_san.so" if SANITIZE else "libluvc.so")
OBJ = os.path.join(HERE, "_build_san" if SANITIZE else "_build")
SAN_FLAGS = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-omit-frame-pointer", "-g"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall",
    # packed fp32 VALU forms are kept out of the generated code on purpose
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = sources() + glob.glob(os.path.join(CSRC, "*.hpp")) + [os.path.join(HERE, "..", "include", "luvc.h")]
    return any(os.path.getmtime(p) > t for p in deps)


def build(force: bool = True, verbose: bool = False) -> str:
    if not force and not stale():
        return LIB
    os.makedirs(OBJ, exist_ok=True)
    srcs = sources()

    def compile_one(src):
        obj = os.path.join(OBJ, os.path.basename(src) + ".o")
        cmd = [HIPCC, *FLAGS, *(SAN_FLAGS if SANITIZE else []), *os.environ.get("LUVC_HIPCC_EXTRA", "").split(), "-c", src, "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        r = subprocess.run(cmd, capture_output=True, text=True)
        noise = "is not a recognized feature for this target"
        err = "\n".join(l for l in r.stderr.splitlines() if noise not in l)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{err}")
        if err.strip() and verbose:
            print(err, file=sys.stderr)
        return obj

    with ThreadPoolExecutor(max_workers=min(8, len(srcs))) as ex:
        objs = list(ex.map(compile_one, srcs))
    subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *(["-fsanitize=address", "-fsanitize=undefined", "-shared-libsan"] if SANITIZE else []), *objs, "-o", LIB])
    return LIB


if __name__ == "__main__":
    print(build(force=True, verbose=True))
