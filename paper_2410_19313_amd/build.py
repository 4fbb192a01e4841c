"""Build the HIP library for gfx950 in-tree (paper_2410_19313_amd/libcoat.so)."""
from __future__ import annotations

import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(_HERE)
SOURCES = [os.path.join(_HERE, "csrc", "coat_kernels.hip")]
HEADERS = [os.path.join(ROOT, "include", "coat.h")] + [os.path.join(_HERE, "csrc", f) for f in (
    "coat_tables.inc", "coat_device.hpp", "coat_step.hpp", "coat_multi.hpp", "coat_quant.hpp", "coat_act.hpp", "coat_copy.hpp")]
LIB = os.path.join(_HERE, "libcoat.so")

# packed fp32 instructions are switched off on purpose (some forms have misbehaved on this
# hardware); the option belongs to the device pass, the host pass only warns about it
# -fno-strict-aliasing: the kernels view one LDS tile as fp32 rows, as packed bf16 rows and as bytes;
# the order of those accesses must follow the program, not the types
HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-fno-strict-aliasing",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
               "-Wno-unused-command-line-argument"]


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(p) > t for p in SOURCES + HEADERS)


def build(force: bool = True, verbose: bool = False) -> str:
    """Compile every HIP source into libcoat.so.  Cross-compiles without a GPU."""
    if not force and not is_stale():
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = LIB + ".tmp%d" % os.getpid()
    cmd = [hipcc] + HIPCC_FLAGS + ["-I", os.path.join(ROOT, "include")] + SOURCES + ["-o", tmp]
    if verbose:
        print(" ".join(cmd))
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout)
    os.replace(tmp, LIB)
    return LIB


NATIVE_DIR = os.path.join(ROOT, "tests", "native")
NATIVE_TEST_SRC = os.path.join(NATIVE_DIR, "abi_smoke.cpp")
NATIVE_TEST_BIN = os.path.join(NATIVE_DIR, "abi_smoke")
CONVERT_TEST_SRC = os.path.join(NATIVE_DIR, "convert_band.cpp")
CONVERT_TEST_BIN = os.path.join(NATIVE_DIR, "convert_band")


def _hipcc_program(src: str, out: str, force: bool, link_lib: bool) -> str:
    newest = max([os.path.getmtime(src)] + ([os.path.getmtime(LIB)] if link_lib else []))
    if not force and os.path.exists(out) and os.path.getmtime(out) >= newest:
        return out
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, "--offload-arch=gfx950", "-O2", "-std=c++17", "-I", os.path.join(ROOT, "include"), src]
    if link_lib:
        cmd += ["-L", _HERE, "-lcoat", "-Wl,-rpath,$ORIGIN/../../paper_2410_19313_amd"]
    res = subprocess.run(cmd + ["-o", out], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout)
    return out


def build_native_test(force: bool = True) -> str:
    """Compile the plain-HIP host program that uses the C ABI without Python (tests/native)."""
    return _hipcc_program(NATIVE_TEST_SRC, NATIVE_TEST_BIN, force, link_lib=True)


def build_convert_test(force: bool = True) -> str:
    """Compile the program that pins the hardware FP32 -> FP8 converts around the largest finite value
    (tests/native); it does not use the library."""
    return _hipcc_program(CONVERT_TEST_SRC, CONVERT_TEST_BIN, force, link_lib=False)


if __name__ == "__main__":
    print(build(force=True, verbose=True))
    print(build_native_test(force=True))
    print(build_convert_test(force=True))
