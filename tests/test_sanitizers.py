"""Address and undefined-behaviour sanitizers over the host code, on the CPU.

(1) The oracle (oracle/coat_ref.c) compiled into a small C driver that calls every entry point on
    ragged sizes with heap blocks of exactly the documented sizes (tests/native/oracle_sanitize.c).
(2) The host side of the HIP library (argument validation, plan building, shard ranges, launch
    shapes, step constants), compiled with the sanitizers on the host pass only, driven by
    tests/native/host_sanitize.cpp.  The device code is compiled as usual and never runs here.
The sanitizer runtimes are linked into the programs; nothing is preloaded."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
NATIVE = os.path.join(ROOT, "tests", "native")
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")


def run(cmd, **kw):
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, **kw)
    assert res.returncode == 0, "%s\n%s" % (" ".join(cmd), res.stdout[-4000:])
    return res.stdout


def test_oracle_under_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_sanitize")
    run(["gcc", "-O1", "-g", "-std=c99", "-fopenmp", "-ffp-contract=off", "-Wall", "-Wextra",
         "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan",
         "-I", os.path.join(ROOT, "oracle"), os.path.join(NATIVE, "oracle_sanitize.c"),
         os.path.join(ROOT, "oracle", "coat_ref.c"), "-lm", "-o", exe])
    out = run([exe], env=ENV, timeout=300)
    assert "oracle_sanitize ok" in out, out


@pytest.mark.skipif(shutil.which(os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")) is None, reason="no hipcc")
def test_library_host_code_under_sanitizers(tmp_path):
    from paper_2410_19313_amd import build
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    host_san = []
    for flag in ("-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=all", "-g"):
        host_san += ["-Xarch_host", flag]            # the sanitizers instrument the host pass only
    lib = str(tmp_path / "libcoat.so")
    run([hipcc] + build.HIPCC_FLAGS + host_san + ["-I", os.path.join(ROOT, "include")] + build.SOURCES + ["-o", lib])
    exe = str(tmp_path / "host_sanitize")
    run([hipcc, "--offload-arch=gfx950", "-O1", "-std=c++17"] + host_san +
        ["-I", os.path.join(ROOT, "include"), os.path.join(NATIVE, "host_sanitize.cpp"),
         "-L", str(tmp_path), "-lcoat", "-Wl,-rpath," + str(tmp_path), "-o", exe])
    out = run([exe], env=ENV, timeout=300)
    assert "host_sanitize ok" in out, out
