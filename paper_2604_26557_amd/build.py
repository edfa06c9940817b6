"""Build the native library in-tree with hipcc for gfx950 (cross-compiles without a GPU)."""
from __future__ import annotations

import glob
import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libkvblade.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950",
    # packed fp32 VALU forms stay off for all device code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.cpp")) + glob.glob(os.path.join(CSRC, "*.hip")))


def build(verbose: bool = True) -> str:
    """Compile every source to an object, then link libkvblade.so.  Always rebuilds."""
    objdir = os.path.join(PKG, "_build")
    os.makedirs(objdir, exist_ok=True)
    procs = []
    for src in sources():
        obj = os.path.join(objdir, os.path.basename(src) + ".o")
        cmd = [HIPCC, *FLAGS, "-c", src, "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((obj, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    objs = []
    for obj, pr in procs:
        out, _ = pr.communicate()
        # the host pass does not know the device-only target feature; that warning is expected
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l and l.strip())
        if pr.returncode != 0:
            raise RuntimeError(f"hipcc failed for {obj}:\n{out}")
        if verbose and out:
            print(out, flush=True)
        objs.append(obj)
    cmd = [HIPCC, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB, *objs, "-lpthread"]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return LIB


def build_sanitized(outdir: str) -> str:
    """The same sources with the HOST code instrumented by AddressSanitizer and UndefinedBehaviorSanitizer
    (device code is compiled as usual and not instrumented): for CPU runs of the planner and the host logic.
    The result links against clang's shared sanitizer runtime, which the process that loads it must preload."""
    os.makedirs(outdir, exist_ok=True)
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-omit-frame-pointer"]
    flags = ["-O1", "-g"] + [f for f in FLAGS if f != "-O3"]
    procs = []
    for src in sources():
        obj = os.path.join(outdir, os.path.basename(src) + ".o")
        procs.append((obj, subprocess.Popen([HIPCC, *flags, *san, "-c", src, "-o", obj],
                                            stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    objs = []
    for obj, pr in procs:
        out, _ = pr.communicate()
        if pr.returncode != 0:
            raise RuntimeError(f"hipcc failed for {obj}:\n{out}")
        objs.append(obj)
    lib = os.path.join(outdir, "libkvblade_san.so")
    subprocess.check_call([HIPCC, "-shared", "-fPIC", "--offload-arch=gfx950", "-Xarch_host", "-fsanitize=address",
                           "-Xarch_host", "-fsanitize=undefined", "-shared-libsan", "-o", lib, *objs, "-lpthread"])
    return lib


def build_if_missing() -> str:
    """For harnesses (tests, smoke, bench): build only when no library has been built.  The binding itself
    never builds and never falls back: it raises when the library is missing."""
    return LIB if os.path.exists(LIB) else build(verbose=False)


if __name__ == "__main__":
    build()
    print(LIB)
    sys.exit(0)
