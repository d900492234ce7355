"""Builds libcsbrnn.so (host packer/planner + gfx950 kernels) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libcsbrnn.so")
SOURCES = ["csb_pack.cpp", "csb_plan.cpp", "csb_stream.cpp", "csb_sharing.cpp", "csb_spmv.hip", "csb_spmv_stream.hip", "csb_spmm.hip", "csb_project.hip", "csb_rnn.hip"]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


def sanitizer_runtime() -> str:
    """The shared AddressSanitizer runtime of hipcc's clang (what a sanitized build needs preloaded)."""
    out = subprocess.run([hipcc(), "-print-file-name=libclang_rt.asan-x86_64.so"], stdout=subprocess.PIPE, text=True).stdout.strip()
    if os.path.isabs(out) and os.path.exists(out):
        return out
    import glob
    hits = sorted(glob.glob("/opt/rocm/lib/llvm/lib/clang/*/lib/linux/libclang_rt.asan-x86_64.so"))
    return hits[-1] if hits else out


def build(verbose: bool = False, sanitize: bool = False) -> str:
    """Compile every source for gfx950 and link the shared library.  Always compiles.
    sanitize: the HOST code (packer, planners, validators, launch wrappers) is built with
    AddressSanitizer and UndefinedBehaviorSanitizer; device code is untouched.  The CPU test suite
    then runs as
        LD_PRELOAD=<sanitizer_runtime()> ASAN_OPTIONS=detect_leaks=0 python -m pytest tests -m "not gpu"
    (the interpreter itself is not instrumented, hence the preload and no leak report).  Build
    again without the flag afterwards: a sanitized library is not for the GPU machine."""
    cmd = [hipcc(), "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared",
           "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
           # packed-FP32 VALU forms are switched off for all device code
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Wall", "-Wno-unused-command-line-argument"]
    if sanitize:
        cmd[1] = "-O1"
        cmd += ["-g", "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                "-Xarch_host", "-fno-omit-frame-pointer", "-Xarch_host", "-fno-sanitize-recover=undefined", "-shared-libsan"]
    cmd += [os.path.join(CSRC, s) for s in SOURCES]
    tmp = LIB + f".tmp{os.getpid()}"
    cmd += ["-o", tmp]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines() if "is not a recognized feature" not in l)
    if res.returncode != 0:
        sys.stderr.write(out + "\n")
        raise RuntimeError("hipcc failed")
    if verbose and out.strip():
        print(out)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    san = "--sanitize" in sys.argv[1:]
    print(build(verbose=True, sanitize=san))
    if san:
        print("run the CPU tests with: LD_PRELOAD=" + sanitizer_runtime() + " ASAN_OPTIONS=detect_leaks=0 python -m pytest tests -m 'not gpu'")
