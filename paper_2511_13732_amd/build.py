"""Build libpcg.so (hand-written HIP for gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
LIB = os.path.join(_HERE, "libpcg.so")
SOURCES = ["pcg_kernels.hip", "pcg_asg.hip", "pcg_api.cpp", "pcg_prepare.cpp"]
HEADERS = ["pcg_kernels.h", "pcg_device.h", "pcg_layout.h", os.path.join("..", "..", "include", "pcg.h")]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-pthread",
    # keep hipcc from forming packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # no implicit fused multiply-adds: the kernels spell out fmaf() where one is wanted, and
    # (a*b - c*d) must round both products so that equal rows cancel exactly
    "-ffp-contract=off",
    "-Wall", "-Wno-unused-command-line-argument",
]


# Host-side sanitizer build (the device code is compiled as always): AddressSanitizer and
# UndefinedBehaviorSanitizer on everything that runs on the CPU -- argument checks, workspace
# carving, the membership helpers, the prepared-layout builder.  Loaded instead of libpcg.so when
# PCG_SANITIZE=1 (see tests/conftest.py for the command line).
LIB_SAN = os.path.join(_HERE, "libpcg_san.so")
SANITIZE_FLAGS = ["-O1", "-g", "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                  "-Xarch_host", "-fno-omit-frame-pointer", "-shared-libsan"]


def sanitize_requested() -> bool:
    return os.environ.get("PCG_SANITIZE", "") not in ("", "0")


def asan_runtime() -> str:
    """Path of the sanitizer runtime that must be preloaded into a Python that loads the
    sanitized libraries (the one of ROCm's clang, which compiles both of them)."""
    clang = os.path.join(os.path.dirname(os.path.realpath(os.environ.get("HIPCC", "/opt/rocm/bin/hipcc"))),
                         "..", "llvm", "bin", "clang")
    if not os.path.exists(clang):
        clang = "/opt/rocm/llvm/bin/clang"
    out = subprocess.run([clang, "-print-file-name=libclang_rt.asan-x86_64.so"], capture_output=True, text=True)
    return os.path.realpath(out.stdout.strip())


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(os.path.join(CSRC, f)) > t for f in SOURCES + HEADERS)


def build(verbose: bool = False, sanitize: bool = False) -> str:
    """Compile unconditionally; returns the path of the shared library."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    flags = [f for f in HIPCC_FLAGS if f != "-O3"] + SANITIZE_FLAGS if sanitize else HIPCC_FLAGS
    out = LIB_SAN if sanitize else LIB
    cmd = [hipcc, *flags, "-x", "hip", *[os.path.join(CSRC, s) for s in SOURCES], "-o", out]
    if verbose:
        print(" ".join(cmd))
    proc = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    msgs = "\n".join(l for l in (proc.stdout + proc.stderr).splitlines() if noise not in l)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + msgs)
    if verbose and msgs.strip():
        print(msgs)
    return out


if __name__ == "__main__":
    print(build(verbose=True))
