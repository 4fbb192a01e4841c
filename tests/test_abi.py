"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol
include/coat.h declares, and rejects bad arguments before anything is launched."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def coat():
    import paper_2410_19313_amd as C
    from paper_2410_19313_amd import build
    if build.is_stale():
        build.build()
    return C


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "coat.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(coat_[a-z0-9_]+)\s*\(", text)))


def test_header_symbols_are_exported(coat):
    names = declared_symbols()
    assert set(names) == set(coat.EXPORTS)
    L = coat.lib()
    for name in names:
        assert getattr(L, name) is not None
    assert coat.lib().coat_version() >= 100


def test_error_codes_have_text(coat):
    for code in range(0, -8, -1):
        assert coat.strerror(code) and "unknown" not in coat.strerror(code)
    assert "unknown" in coat.strerror(-99)


def test_step_rejects_bad_arguments_before_launch(coat):
    L = coat.lib()
    ok = 0x1000                                       # a fake, aligned, never dereferenced address

    def call(hp, ptrs=None, n=4096):
        p = [ctypes.c_void_p(ok)] * 8 if ptrs is None else [ctypes.c_void_p(x) for x in ptrs]
        return L.coat_fp8_adamw_step(*p, n, ctypes.byref(hp) if hp is not None else None, None)

    assert call(None) == -1
    assert call(coat.make_hparams(group_size=100)) == -3
    assert call(coat.make_hparams(group_size=16)) == -3
    assert call(coat.make_hparams(step=0)) == -4
    assert call(coat.make_hparams(lr=float("nan"))) == -5
    assert call(coat.make_hparams(beta1=1.0)) == -5
    assert call(coat.make_hparams(beta2=-0.1)) == -5
    assert call(coat.make_hparams(eps=-1.0)) == -5
    assert call(coat.make_hparams(lr=float("inf"))) == -5
    assert call(coat.make_hparams(k_min=4.0, k_max=2.0)) == -5
    assert call(coat.make_hparams(k_min=1e-3, k_max=2.0)) == -5
    assert call(coat.make_hparams(k_min=1.0, k_max=1e6)) == -5
    hp = coat.make_hparams()
    hp.flags = 1 | 32
    assert call(hp) == -5                               # unknown flag bit
    assert call(coat.make_hparams(), ptrs=[ok, ok, 0, ok, ok, ok, ok, ok]) == -1
    assert call(coat.make_hparams(), ptrs=[ok + 4, ok, ok, ok, ok, ok, ok, ok]) == -2
    assert call(coat.make_hparams(), ptrs=[ok, ok, ok, ok, ok, ok + 8, ok, ok]) == -2
    assert call(coat.make_hparams(), n=1 << 50) == -7
    assert call(coat.make_hparams(), ptrs=[0] * 8, n=0) == 0      # empty input: successful no-op


def test_quant_dequant_reject_bad_arguments(coat):
    L = coat.lib()
    ok = ctypes.c_void_p(0x1000)
    bad = ctypes.c_void_p(0x1004)
    assert L.coat_quant_group(ok, 1024, 48, 1, 0.0, 0.0, ok, ok, ok, None) == -3
    assert L.coat_quant_group(None, 1024, 128, 1, 0.0, 0.0, ok, ok, ok, None) == -1
    assert L.coat_quant_group(ok, 1024, 128, 1, 0.0, 0.0, bad, ok, ok, None) == -2
    assert L.coat_quant_group(ok, 1024, 128, 1, 2.0, 1.0, ok, ok, ok, None) == -5
    assert L.coat_quant_group(None, 0, 128, 1, 0.0, 0.0, None, None, None, None) == 0
    assert L.coat_quant_group(ok, 1024, 128, 64, 0.0, 0.0, ok, ok, ok, None) == -5     # unknown flag bit
    assert L.coat_dequant_group(ok, ok, ok, 1024, 7, 0, ok, None) == -3
    assert L.coat_dequant_group(ok, None, ok, 1024, 128, 0, ok, None) == -1
    assert L.coat_dequant_group(ok, ok, bad, 1024, 128, 0, ok, None) == -2
    assert L.coat_dequant_group(ok, ok, ok, 1024, 128, 8, ok, None) == -5
    assert L.coat_dequant_group(None, None, None, 0, 128, 2, None, None) == 0


def test_act_quantizers_reject_bad_arguments(coat):
    L = coat.lib()
    ok = ctypes.c_void_p(0x1000)
    bad16 = ctypes.c_void_p(0x1004)
    bad4 = ctypes.c_void_p(0x1002)
    assert L.coat_act_quant_group(ok, 1024, 8, ok, ok, None) == -3
    assert L.coat_act_quant_group(ok, 1024, 48, ok, ok, None) == -3
    assert L.coat_act_quant_group(ok, 1024, 16, None, ok, None) == -1
    assert L.coat_act_quant_group(bad16, 1024, 16, ok, ok, None) == -2
    assert L.coat_act_quant_group(ok, 1 << 50, 16, ok, ok, None) == -7
    assert L.coat_act_quant_group(None, 0, 16, None, None, None) == 0
    for f in (L.coat_act_quant_tensor, L.coat_act_quant_tensor_from_group_amax):
        #  x, n, G, group_amax, workspace, tensor_amax, tensor_scale, q, stream
        assert f(ok, 1024, 24, ok, ok, ok, ok, ok, None) == -3
        assert f(ok, 1024, 16, None, ok, ok, ok, ok, None) == -1
        assert f(ok, 1024, 16, ok, None, ok, ok, ok, None) == -1
        assert f(ok, 1024, 16, ok, ok, None, ok, ok, None) == -1
        assert f(ok, 1024, 16, ok, ok, ok, ok, None, None) == -1
        assert f(ok, 1024, 16, bad16, ok, ok, ok, ok, None) == -2
        assert f(ok, 1024, 16, ok, bad16, ok, ok, ok, None) == -2
        assert f(ok, 1024, 16, ok, ok, bad4, ok, ok, None) == -2
        assert f(ok, 1 << 50, 16, ok, ok, ok, ok, ok, None) == -7
        assert f(None, 0, 16, None, None, None, None, None, None) == 0


def test_binding_refuses_host_tensors(coat):
    import torch
    x = torch.zeros(1024)
    with pytest.raises(TypeError):
        coat.coat_quant_group(x, 128)
