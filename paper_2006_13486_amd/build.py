"""Build the C-ABI library (librbgp.so) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
LIB = os.path.join(_HERE, "librbgp.so")
SOURCES = ["rbgp_mfma_reg_bf16_wide.hip", "rbgp_mfma_reg_bf16.hip", "rbgp_mfma_reg_bf16_lean.hip", "rbgp_mfma_reg.hip", "rbgp_host.cpp",
           "rbgp_device.hip", "rbgp_mfma_reg_dual.hip", "rbgp_sddmm.hip", "rbgp_mfma_tile.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=default",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument"]


def build(verbose: bool = False, extra: list[str] | None = None) -> str:
    """Compile every source and link librbgp.so (always recompiles).  extra: more hipcc flags."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objs = []
    procs = []
    for src in SOURCES:
        obj = os.path.join(CSRC, os.path.splitext(src)[0] + ".o")
        cmd = [hipcc, *FLAGS, *(extra or []), "-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((cmd, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    for cmd, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if p.returncode:
            raise RuntimeError("hipcc failed:\n" + " ".join(cmd) + "\n" + out)
        if verbose and out.strip():
            print(out)
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    subprocess.check_call(cmd)
    return LIB


def build_sanitized() -> str:
    """The same library with its HOST code under AddressSanitizer and UndefinedBehaviorSanitizer (device code is
    compiled as usual): librbgp_asan.so, for the CPU tests of the host logic -- sampler, index tables, layouts,
    transposes -- which run it in a child process with the sanitizer runtime preloaded (tests/test_host_sanitizers.py)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host",
           "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer", "-g"]
    flags = [f if f != "-O3" else "-O1" for f in FLAGS]
    lib = os.path.join(_HERE, "librbgp_asan.so")
    objs, procs = [], []
    for src in SOURCES:
        obj = os.path.join(CSRC, os.path.splitext(src)[0] + ".asan.o")
        cmd = [hipcc, *flags, *san, "-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj]
        procs.append((cmd, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    for cmd, p in procs:
        out, _ = p.communicate()
        if p.returncode:
            raise RuntimeError("hipcc failed:\n" + " ".join(cmd) + "\n" + out)
    subprocess.check_call([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-fsanitize=address", "-fsanitize=undefined",
                           "-shared-libsan", "-o", lib, *objs])
    return lib


def sanitizer_runtime() -> str:
    """The AddressSanitizer runtime that librbgp_asan.so needs preloaded (clang's, from the ROCm toolchain)."""
    import glob
    found = sorted(glob.glob("/opt/rocm/llvm/lib/clang/*/lib/linux/libclang_rt.asan-x86_64.so"))
    if not found:
        raise RuntimeError("no libclang_rt.asan-x86_64.so under /opt/rocm/llvm")
    return found[-1]


if __name__ == "__main__":
    print(build_sanitized() if "sanitized" in sys.argv else build(verbose="-v" in sys.argv))
