"""The C ABI from a plain HIP host program (tests/native/abi_smoke.cpp): no Python, no PyTorch in
the process that makes the calls."""
import subprocess

import pytest

pytestmark = pytest.mark.gpu


def test_c_abi_from_a_plain_hip_program():
    from paper_2410_19313_amd import build
    exe = build.build_native_test(force=False)
    res = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=120)
    assert res.returncode == 0 and "abi_smoke ok" in res.stdout, res.stdout


def test_hardware_converts_around_the_largest_finite_value():
    # every fp32 pattern from fmax to past the half-way point, both formats, both signs
    from paper_2410_19313_amd import build
    exe = build.build_convert_test(force=False)
    res = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=120)
    assert res.returncode == 0 and "convert_band ok" in res.stdout, res.stdout
    print(res.stdout)
