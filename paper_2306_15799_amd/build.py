"""Builds libflurka.so (gfx950 only) from csrc/ with hipcc, in-tree."""
from __future__ import annotations

import os
import shutil
import subprocess

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG_DIR)
CSRC = os.path.join(PKG_DIR, "csrc")
LIB_PATH = os.path.join(PKG_DIR, "libflurka.so")

SOURCES = ["flurka_api.hip", "flurka_generic.hip", "flurka_fast.hip", "flurka_keystate.hip", "flurka_bwd.hip"]

HIPCC_FLAGS = [
    "-O3", "-std=c++17", "-fPIC", "-shared",
    "--offload-arch=gfx950",
    # packed-fp32 VALU forms are kept off for every kernel in this library
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-fvisibility=hidden",
    "-Wall", "-Wno-unused-function", "-Wno-unused-command-line-argument",
]


def find_hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found; libflurka needs the ROCm toolchain")


def build(verbose: bool = False) -> str:
    """Compile every source for gfx950 and link libflurka.so next to the package."""
    hipcc = find_hipcc()
    cmd = [hipcc, *HIPCC_FLAGS, "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           *[os.path.join(CSRC, s) for s in SOURCES], "-o", LIB_PATH]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout + res.stderr)
    if verbose and res.stderr.strip():
        print(res.stderr)
    return LIB_PATH


SAN_LIB_PATH = os.path.join(PKG_DIR, "libflurka_asan.so")
SAN_DRIVER_SRC = os.path.join(ROOT, "tests", "host", "abi_sanitizer_driver.cpp")
SAN_DRIVER_PATH = os.path.join(PKG_DIR, "abi_sanitizer_driver")
# host code only: hipcc applies what follows -Xarch_host to the host pass, the gfx950 pass is untouched
SAN_FLAGS = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
             "-Xarch_host", "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer", "-g"]


def build_sanitized(verbose: bool = False):
    """AddressSanitizer + UBSan build of the library's HOST side (validation, layout and workspace
    arithmetic, launch-fact cache, stage timer) plus the small driver program that exercises it without a
    GPU (tests/host/abi_sanitizer_driver.cpp).  Returns (library path, driver path).  CPU machines only:
    sanitizer runs on the GPU machine are not what this is for."""
    hipcc = find_hipcc()
    lib_cmd = [hipcc, *[f for f in HIPCC_FLAGS if f != "-O3"], "-O1", *SAN_FLAGS, "-I", os.path.join(ROOT, "include"),
               "-I", CSRC, *[os.path.join(CSRC, s) for s in SOURCES], "-o", SAN_LIB_PATH]
    drv_cmd = [hipcc, "-x", "c++", "-std=c++17", "-O1", "-g", "-fsanitize=address", "-fsanitize=undefined",
               "-fno-sanitize-recover=undefined", "-I", os.path.join(ROOT, "include"), SAN_DRIVER_SRC,
               "-L", PKG_DIR, "-l:libflurka_asan.so", "-Wl,-rpath," + PKG_DIR, "-o", SAN_DRIVER_PATH]
    for cmd in (lib_cmd, drv_cmd):
        if verbose:
            print(" ".join(cmd), flush=True)
        res = subprocess.run(cmd, capture_output=True, text=True)
        if res.returncode != 0:
            raise RuntimeError("sanitized build failed:\n" + res.stdout + res.stderr)
    return SAN_LIB_PATH, SAN_DRIVER_PATH


if __name__ == "__main__":
    print(build(verbose=True))
