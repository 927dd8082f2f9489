"""Builds librestkv.so (HIP, gfx950) in-tree with hipcc."""
from __future__ import annotations

import glob
import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "librestkv.so")
LIB_SAN = os.path.join(PKG, "librestkv_san.so")     # host code under AddressSanitizer + UBSan (CPU tests only)
ASAN_RUNTIME_DIR = "/opt/rocm/lib/llvm/lib/clang"

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc",
    # packed FP32 instruction forms are kept out of the generated code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function", "-Wno-unknown-warning-option",
    # the tile copies set m0 in inline asm and say so in their clobber list; the compiler reserves
    # m0, uses it for nothing in these kernels, and warns about the entry at every instantiation
    "-Wno-inline-asm",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


# host-side sanitizers only: each -fsanitize= directly after -Xarch_host, device code untouched
SAN_FLAGS = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
             "-Xarch_host", "-fno-omit-frame-pointer", "-g"]


def asan_runtime() -> str:
    """Path of clang's shared AddressSanitizer runtime (to be preloaded into the Python process
    that loads a sanitized library), or '' if the toolchain has none."""
    hits = sorted(glob.glob(os.path.join(ASAN_RUNTIME_DIR, "*", "lib", "linux", "libclang_rt.asan-x86_64.so")))
    return hits[-1] if hits else ""


def build(verbose: bool = True, jobs: int = 8, sanitize: bool = False) -> str:
    """Compile every .hip source and link the shared library. Always rebuilds.
    sanitize=True builds librestkv_san.so instead: same device code, host code instrumented."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objdir = os.path.join(PKG, "_build_san" if sanitize else "_build")
    flags = FLAGS + (SAN_FLAGS if sanitize else [])
    lib = LIB_SAN if sanitize else LIB
    os.makedirs(objdir, exist_ok=True)
    procs = []
    objs = []
    for src in sources():
        obj = os.path.join(objdir, os.path.basename(src)[:-4] + ".o")
        objs.append(obj)
        cmd = [hipcc, *flags, "-c", src, "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT)))
        while sum(p.poll() is None for _, p in procs) >= jobs:
            procs[0][1].wait()
    bad = False
    for src, p in procs:
        out, _ = p.communicate()
        text = out.decode(errors="replace")
        text = "\n".join(l for l in text.splitlines()
                         if "packed-fp32-ops" not in l or "error" in l)
        if p.returncode != 0:
            bad = True
            print(f"FAILED: {src}\n{text}", file=sys.stderr)
        elif verbose and text.strip():
            print(text)
    if bad:
        raise RuntimeError("hipcc failed")
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib, *objs]
    if sanitize:
        cmd += ["-fsanitize=address", "-fsanitize=undefined", "-shared-libsan", "-fno-gpu-sanitize"]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return lib


if __name__ == "__main__":
    build()
