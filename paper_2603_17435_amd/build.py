"""Builds libzipserv_hip.so (host packer + gfx950 kernels) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libzipserv_hip.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

COMMON = ["-O3", "-fPIC", "-std=c++17", "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-Wall", "-Wextra"]
# -amdgpu-atomic-optimizer-strategy=None: the kernels' LDS atomics are issued by one lane on
# purpose; the optimizer's wave-reduction wrapper would cost ~15 instructions around each.
DEVICE = ["--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
          "-mllvm", "-amdgpu-atomic-optimizer-strategy=None",
          "-Wno-unused-command-line-argument", "-Wno-int-to-pointer-cast",
          # the LDS-direct staging code names m0 as clobbered (it writes it); clang warns that m0
          # is a reserved register, which is exactly why the compiler must be told
          "-Wno-inline-asm"]


def sources() -> list[str]:
    return [os.path.join(CSRC, f) for f in sorted(os.listdir(CSRC)) if f.endswith((".hip", ".cpp"))]


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, f) for f in os.listdir(CSRC)] + [os.path.join(ROOT, "include", "zipserv.h")]
    return any(os.path.getmtime(p) > t for p in deps)


def build(verbose: bool = False, extra: list[str] | None = None) -> str:
    """Compiles every source for gfx950 and links the shared library.  Always rebuilds."""
    objs = []
    build_dir = os.path.join(PKG, "_build")
    os.makedirs(build_dir, exist_ok=True)
    for src in sources():
        obj = os.path.join(build_dir, os.path.basename(src) + ".o")
        cmd = [HIPCC, "-c", src, "-o", obj] + COMMON + (extra or [])
        if src.endswith(".hip"):
            cmd += DEVICE
        else:
            cmd = [HIPCC, "-x", "c++", "-c", src, "-o", obj, "-pthread", "-D__HIP_PLATFORM_AMD__",
                   "-I", "/opt/rocm/include"] + COMMON
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True)
        objs.append(obj)
    tmp = LIB + ".tmp.%d" % os.getpid()
    cmd = [HIPCC, "-shared", "-o", tmp] + objs + ["--offload-arch=gfx950", "-pthread", "-L/opt/rocm/lib", "-lhipblaslt",
                                                  "-Wl,-rpath,/opt/rocm/lib"]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
