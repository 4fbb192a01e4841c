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


def test_header_is_plain_c_and_cplusplus():
    """The boundary is a C ABI: the header must compile on its own as C99 and as C++."""
    import subprocess
    h = os.path.join(ROOT, "include", "coat.h")
    subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Werror", "-fsyntax-only", "-x", "c", h], check=True)
    subprocess.run(["g++", "-std=c++11", "-Wall", "-Werror", "-fsyntax-only", "-x", "c++", h], check=True)


def test_error_codes_have_text(coat):
    for code in range(0, -9, -1):
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
    hp.flags = 1 | 256
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
    assert L.coat_quant_group(ok, 1024, 128, 128, 0.0, 0.0, ok, ok, ok, None) == -5     # unknown flag bit
    assert L.coat_dequant_group(ok, ok, ok, 1024, 7, 0, ok, None) == -3
    assert L.coat_dequant_group(ok, None, ok, 1024, 128, 0, ok, None) == -1
    assert L.coat_dequant_group(bad, ok, ok, 1024, 128, 0, ok, None) == -2
    # per-group arrays need 4-byte alignment only (a shard may start at any even group)
    assert L.coat_dequant_group(ok, ok, ctypes.c_void_p(0x1002), 1024, 128, 0, ok, None) == -2
    assert L.coat_quant_group(ok, 1024, 128, 1, 0.0, 0.0, ok, ctypes.c_void_p(0x1002), ok, None) == -2
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


def fake_desc(coat, n, wd=0.0, base=0x10000, **over):
    kw = dict(w=base, w_bf16=0, grad_bf16=base, m_q=base, m_scale=base, m_k=base, v_q=base, v_scale=base, v_k=base)
    kw.update(over)
    return coat.TensorDesc(kw["w"], kw["w_bf16"], kw["grad_bf16"], kw["m_q"], kw["m_scale"], kw["m_k"],
                           kw["v_q"], kw["v_scale"], kw["v_k"], n, wd, 0)


def test_multi_plan_layout_is_what_the_header_documents(coat):
    """The plan is host-built data: check it against the documented layout with an independent
    reconstruction (one record per span of 32 chunks, every tensor starting a new span)."""
    import numpy as np
    sizes = [5000, 0, 1024, 7, 1 << 20, 1023, 1025, 32 * 1024, 32 * 1024 + 1]
    descs = [fake_desc(coat, n, wd=0.01 * i, base=0x10000 * (i + 1)) for i, n in enumerate(sizes)]
    blob = coat.coat_multi_plan_build(descs)
    spans = [((n + 1023) // 1024 + 31) // 32 for n in sizes]
    assert spans == [1, 0, 1, 1, 32, 1, 1, 1, 2]
    assert len(blob) == 128 + 128 * sum(spans)
    assert bytes(blob[:8]) == b"COATPLN2"
    version, count = np.frombuffer(blob[8:16], np.uint32)
    total, r_off, nbytes = np.frombuffer(blob[16:40], np.uint64)
    assert (version, count, total, r_off, nbytes) == (2, len(sizes), sum(spans), 128, len(blob))
    rec = 0
    for t, n in enumerate(sizes):
        for i in range(spans[t]):
            raw = blob[128 + 128 * rec: 128 + 128 * (rec + 1)]
            ptrs = np.frombuffer(raw[:72], np.uint64)
            assert ptrs[0] == 0x10000 * (t + 1) and ptrs[1] == 0 and np.all(ptrs[2:] == 0x10000 * (t + 1))
            assert np.frombuffer(raw[72:88], np.uint64).tolist() == [n, 32 * i]          # n, chunk_base
            assert np.frombuffer(raw[88:92], np.float32)[0] == np.float32(0.01 * t)
            assert np.frombuffer(raw[92:96], np.uint32)[0] == t
            rec += 1
    assert rec == total


def test_multi_plan_and_step_reject_bad_arguments(coat):
    L = coat.lib()
    good = [fake_desc(coat, 4096)]
    arr = (coat.TensorDesc * 1)(*good)
    size = L.coat_multi_plan_bytes(arr, 1)
    assert size == 128 + 128
    buf = ctypes.create_string_buffer(size)
    assert L.coat_multi_plan_bytes(None, 1) == 0
    assert L.coat_multi_plan_bytes(None, 0) == 128                    # an empty plan is legal
    assert L.coat_multi_plan_build(arr, 1, None, size) == -1
    assert L.coat_multi_plan_build(arr, 1, buf, size - 1) == -7
    for field, bad, code in (("w", 0, -1), ("v_k", 0, -1), ("w", 0x10004, -2), ("m_q", 0x10008, -2), ("w_bf16", 0x10002, -2),
                             ("m_k", 0x10002, -2), ("v_scale", 0x10006, -2)):
        arr2 = (coat.TensorDesc * 1)(fake_desc(coat, 4096, **{field: bad}))
        assert L.coat_multi_plan_build(arr2, 1, buf, size) == code, field
    arr3 = (coat.TensorDesc * 1)(fake_desc(coat, 4096, wd=float("nan")))
    assert L.coat_multi_plan_build(arr3, 1, buf, size) == -5
    arr4 = (coat.TensorDesc * 1)(fake_desc(coat, 1 << 50))
    assert L.coat_multi_plan_bytes(arr4, 1) == 0
    assert L.coat_multi_plan_build(arr, 1, buf, size) == 0
    dev = ctypes.c_void_p(0x20000)
    hp = coat.make_hparams()
    assert L.coat_fp8_adamw_step_multi(None, dev, ctypes.byref(hp), None) == -1
    assert L.coat_fp8_adamw_step_multi(buf, None, ctypes.byref(hp), None) == -1
    assert L.coat_fp8_adamw_step_multi(buf, ctypes.c_void_p(0x20004), ctypes.byref(hp), None) == -2
    assert L.coat_fp8_adamw_step_multi(buf, dev, None, None) == -1
    assert L.coat_fp8_adamw_step_multi(buf, dev, ctypes.byref(coat.make_hparams(group_size=48)), None) == -3
    assert L.coat_fp8_adamw_step_multi(buf, dev, ctypes.byref(coat.make_hparams(step=0)), None) == -4
    junk = ctypes.create_string_buffer(b"\x01" * size, size)
    assert L.coat_fp8_adamw_step_multi(junk, dev, ctypes.byref(hp), None) == -8
    empty = ctypes.create_string_buffer(128)
    assert L.coat_multi_plan_build(None, 0, empty, 128) == 0
    assert L.coat_fp8_adamw_step_multi(empty, None, ctypes.byref(hp), None) == 0      # nothing to do


def test_step_consts_are_the_documented_formulas(coat):
    import math
    import struct
    for lr, b1, b2, t in ((3e-4, 0.9, 0.95, 1), (1e-3, 0.8, 0.999, 17), (0.0, 0.9, 0.95, 1000000)):
        hp = coat.make_hparams(lr=lr, beta1=b1, beta2=b2, step=t)
        denom_mul, denom_add, neg_lr = struct.unpack("<ffd", coat.coat_step_consts_compute(hp)[:16])
        f = lambda x: struct.unpack("<f", struct.pack("<f", x))[0]      # what the fp32 fields hold
        lr32, b1f, b2f, eps32 = f(lr), f(b1), f(b2), f(hp.eps)
        omb1, omb2 = f(1.0 - b1f), f(1.0 - b2f)
        assert neg_lr == -lr32
        c = -lr32 * omb1 / (1.0 - b1f ** t)
        if lr == 0.0:
            assert denom_mul == 0.0 and denom_add == math.inf
        else:
            assert denom_mul == f(math.sqrt(omb2 / (1.0 - b2f ** t)) / c)
            assert denom_add == f(eps32 / c)
    L = coat.lib()
    c = coat.StepConsts()
    assert L.coat_step_consts_compute(None, ctypes.byref(c)) == -1
    assert L.coat_step_consts_compute(ctypes.byref(coat.make_hparams()), None) == -1
    assert L.coat_step_consts_compute(ctypes.byref(coat.make_hparams(step=0)), ctypes.byref(c)) == -4
    buf = ctypes.create_string_buffer(256)
    arr = (coat.TensorDesc * 1)(fake_desc(coat, 4096))
    assert L.coat_multi_plan_build(arr, 1, buf, 256) == 0
    dev = ctypes.c_void_p(0x20000)
    hp = coat.make_hparams()
    assert L.coat_fp8_adamw_step_multi_consts(buf, dev, ctypes.byref(hp), None, None) == -1
    assert L.coat_fp8_adamw_step_multi_consts(buf, dev, ctypes.byref(hp), ctypes.c_void_p(0x30004), None) == -2


def test_shard_range_partitions_at_group_boundaries(coat):
    for n, G, world in ((0, 128, 4), (1, 128, 4), (1000, 128, 3), (4096, 128, 8), (4097, 32, 5), (10 ** 9 + 7, 512, 64),
                        (300, 128, 8)):
        prev = 0
        sizes = []
        for r in range(world):
            b, e = coat.coat_shard_range(n, G, r, world)
            assert b == prev and b <= e <= n
            assert b % (2 * G) == 0 or b == n                    # cut at pairs of groups
            assert e % (2 * G) == 0 or e == n
            sizes.append((e - b + 2 * G - 1) // (2 * G))
            prev = e
        assert prev == n                                         # the shards tile [0, n)
        assert max(sizes) - min(sizes) <= 1                      # in pairs of groups: balanced to one pair
        assert sizes == sorted(sizes, reverse=True)              # the larger shards come first
    L = coat.lib()
    b, e = ctypes.c_uint64(), ctypes.c_uint64()
    assert L.coat_shard_range(10, 128, 4, 4, ctypes.byref(b), ctypes.byref(e)) == -5
    assert L.coat_shard_range(10, 128, 0, 0, ctypes.byref(b), ctypes.byref(e)) == -5
    assert L.coat_shard_range(10, 0, 0, 1, ctypes.byref(b), ctypes.byref(e)) == -3
    assert L.coat_shard_range(10, 128, 0, 1, None, ctypes.byref(e)) == -1


def test_binding_refuses_host_tensors(coat):
    import torch
    x = torch.zeros(1024)
    with pytest.raises(TypeError):
        coat.coat_quant_group(x, 128)


def test_launch_shape_and_plan_limits(coat):
    """A dispatch counts its work-items in 32 bits: the main launch stays below 2^32 / 256 workgroups
    whatever n is (the kernels loop beyond), and a plan whose spans would need more than one launch
    is refused.  Host logic only: nothing is launched and no pointer is dereferenced."""
    L = coat.lib()
    b, t = ctypes.c_uint32(), ctypes.c_uint32()
    for n, want in ((0, 0), (1023, 0), (1024, 1), (4096, 1), (4097, 1), (8192, 2), (6738149376, 1645056),
                    (13015449600, 3177600), (1 << 36, (1 << 24) - 1), (1 << 46, (1 << 24) - 1)):
        assert L.coat_launch_shape(n, ctypes.byref(b), ctypes.byref(t)) == 0
        assert (b.value, t.value) == (want, 256), (n, b.value)
        assert b.value * t.value < 1 << 32
    assert L.coat_launch_shape((1 << 46) + 1, ctypes.byref(b), ctypes.byref(t)) == -7
    assert L.coat_launch_shape(4096, None, ctypes.byref(t)) == -1
    # plan limit: 2^21 - 1 spans of 32768 elements fit one launch, one more does not
    span = 32 * 1024
    fits = (coat.TensorDesc * 1)(fake_desc(coat, span * ((1 << 21) - 1)))
    assert L.coat_multi_plan_bytes(fits, 1) == 128 + 128 * ((1 << 21) - 1)
    too_many = (coat.TensorDesc * 2)(fake_desc(coat, span * ((1 << 21) - 1)), fake_desc(coat, 1))
    assert L.coat_multi_plan_bytes(too_many, 2) == 0
