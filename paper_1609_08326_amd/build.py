"""Compile the HIP library for gfx950 (``hipcc`` cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess

_PKG = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_PKG, "csrc")
SOURCES = [os.path.join(CSRC, "dcasgd.hip")]
DEPENDS = SOURCES + [os.path.join(CSRC, "dcasgd_kernels.hip.h"),
                     os.path.join(os.path.dirname(_PKG), "include", "dcasgd.h")]
LIB = os.path.join(_PKG, "libdcasgd.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
# -ffp-contract=off: one rounding per operation (the results are compared bit
# for bit with a CPU build).  Packed FP32 instructions are switched off.
HIPFLAGS = ["--offload-arch=gfx950", "-std=c++17", "-O3", "-ffp-contract=off",
            "-fPIC", "-shared", "-Wall",
            "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    built = os.path.getmtime(LIB)
    return any(os.path.getmtime(p) > built for p in DEPENDS)


def build_library(force: bool = True, verbose: bool = False) -> str:
    """Build ``libdcasgd.so`` next to this file and return its path."""
    if force or is_stale():
        tmp = LIB + ".tmp.%d" % os.getpid()
        cmd = [HIPCC, *HIPFLAGS, *SOURCES, "-o", tmp]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.check_call(cmd)
        os.replace(tmp, LIB)
    return LIB


PROBE_SRC = os.path.join(CSRC, "membw_probe.hip")
PROBE = os.path.join(_PKG, "membw_probe")


def build_probe(force: bool = True, verbose: bool = False) -> str:
    """Build the stand-alone memory-system probe (an executable, not part of the library)."""
    stale = (not os.path.exists(PROBE)) or os.path.getmtime(PROBE) < os.path.getmtime(PROBE_SRC)
    if force or stale:
        tmp = PROBE + ".tmp.%d" % os.getpid()
        cmd = [HIPCC, "--offload-arch=gfx950", "-std=c++17", "-O3",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", PROBE_SRC, "-o", tmp]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.check_call(cmd)
        os.replace(tmp, PROBE)
    return PROBE


CHECKER_SRC = os.path.join(CSRC, "lambda_check.hip")
CHECKER = os.path.join(_PKG, "lambda_check")


def build_checker(force: bool = True, verbose: bool = False) -> str:
    """Build the stand-alone checker of the short sqrt/divide forms (an executable that
    includes the kernels' header, so it tests the very functions the library runs)."""
    deps = [CHECKER_SRC, os.path.join(CSRC, "dcasgd_kernels.hip.h")]
    stale = (not os.path.exists(CHECKER)) or \
        any(os.path.getmtime(CHECKER) < os.path.getmtime(p) for p in deps)
    if force or stale:
        tmp = CHECKER + ".tmp.%d" % os.getpid()
        cmd = [HIPCC, "--offload-arch=gfx950", "-std=c++17", "-O3", "-ffp-contract=off",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-I", CSRC,
               CHECKER_SRC, "-o", tmp]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.check_call(cmd)
        os.replace(tmp, CHECKER)
    return CHECKER


CLIENT_SRC = os.path.join(CSRC, "abi_client.c")
CLIENT = os.path.join(_PKG, "abi_client")


def build_client(force: bool = True, verbose: bool = False) -> str:
    """Build the plain-C client of the ABI (compiled as C99, linked against the library)."""
    deps = [CLIENT_SRC, os.path.join(os.path.dirname(_PKG), "include", "dcasgd.h")]
    stale = (not os.path.exists(CLIENT)) or \
        any(os.path.getmtime(CLIENT) < os.path.getmtime(p) for p in deps)
    if force or stale:
        tmp = CLIENT + ".tmp.%d" % os.getpid()
        cmd = ["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-O1", "-D__HIP_PLATFORM_AMD__",
               "-I", os.path.join(os.path.dirname(_PKG), "include"), "-I", "/opt/rocm/include",
               CLIENT_SRC, "-o", tmp, "-L", _PKG, "-ldcasgd", "-L", "/opt/rocm/lib", "-lamdhip64",
               "-Wl,-rpath,$ORIGIN", "-Wl,-rpath,/opt/rocm/lib"]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.check_call(cmd)
        os.replace(tmp, CLIENT)
    return CLIENT


if __name__ == "__main__":
    print(build_library(force=True, verbose=True))
    print(build_probe(force=True, verbose=True))
    print(build_checker(force=True, verbose=True))
    print(build_client(force=True, verbose=True))
