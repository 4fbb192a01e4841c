"""Pins for the oracle's activation quantizers (Sec. 5.2): the 1xG per-group quantizer and the
per-tensor quantizer with Group Scaling's two-stage max reduction.  No GPU needed."""
import numpy as np
import pytest
import torch

import synth_inputs as S


def acts(n, seed, spikes=True):
    """bf16 activations ~ N(0,1) with a few large outliers (the spikes GLU-style layers produce)."""
    rng = np.random.default_rng(seed)
    x = rng.standard_normal(n).astype(np.float32)
    if spikes and n > 64:
        x[rng.integers(0, n, max(1, n // 500))] *= 60.0
    return S.f32_to_bf16_bits(x)


@pytest.mark.parametrize("G", [16, 64, 128])
def test_per_group_is_the_plain_quantizer_on_bf16_input(ref, G):
    n = 257 * G + 5
    xb = acts(n, G)
    x = S.bf16_bits_to_f32(xb)
    q, s = ref.act_quant_group(xb, G)
    # same thing as the separately pinned optimizer-state quantizer with the expansion off
    q2, s2, k2 = ref.quant_group(x, G, expand=False)
    assert np.array_equal(q, q2) and np.array_equal(s, s2) and np.all(k2 == 1)
    # Sec. 3 with library routines: S = max|X|/448 per group, X_fp8 = cast(X / S)
    ng = (n + G - 1) // G
    pad = np.zeros(ng * G, np.float32)
    pad[:n] = x
    amax = np.abs(pad).reshape(ng, G).max(1)
    assert np.array_equal(s, amax / np.float32(448.0))
    quot = (pad.reshape(ng, G) / np.where(s > 0, s, 1)[:, None]).astype(np.float32).reshape(-1)[:n]
    lib = torch.from_numpy(quot).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(q, lib)
    top = np.abs(pad).reshape(ng, G).argmax(1)
    full = np.arange(ng) * G + top < n
    assert np.all((q[(np.arange(ng) * G + top)[full]] & 0x7F) == 0x7E)      # the group maximum takes the top code


@pytest.mark.parametrize("G", [16, 128])
def test_group_scaling_two_stage_max_and_per_tensor_codes(ref, G):
    n = 100 * 1024 + 77
    xb = acts(n, 100 + G)
    x = S.bf16_bits_to_f32(xb)
    q, ts, gmax = ref.act_quant_tensor(xb, G)
    # stage 1 is the per-group maximum, stage 2 its maximum: together the tensor's max |x|
    ng = (n + G - 1) // G
    pad = np.zeros(ng * G, np.float32)
    pad[:n] = x
    assert np.array_equal(gmax, np.abs(pad).reshape(ng, G).max(1))
    assert gmax.max() == np.abs(x).max()
    assert ts == np.float32(np.abs(x).max()) / np.float32(448.0)
    # per-tensor quantization with that scale: library cast of the fp32 quotient
    lib = torch.from_numpy((x / np.float32(ts)).astype(np.float32)).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(q, lib)
    assert (q[np.abs(x).argmax()] & 0x7F) == 0x7E
    # the group size only shapes the reduction, not the result
    q2, ts2, _ = ref.act_quant_tensor(xb, 64)
    assert ts2 == ts and np.array_equal(q2, q)


@pytest.mark.parametrize("where", ["first", "last_ragged", "middle"])
def test_group_scaling_finds_the_maximum_wherever_it_is(ref, where):
    # the tensor's largest element in the first group, in the short last group, or in between
    G, n = 16, 40 * 16 + 5
    x = (np.random.default_rng(9).standard_normal(n) * 0.1).astype(np.float32)
    pos = {"first": 3, "last_ragged": n - 2, "middle": 17 * G + 9}[where]
    x[pos] = -7.0
    xb = S.f32_to_bf16_bits(x)
    q, ts, gmax = ref.act_quant_tensor(xb, G)
    assert ts == np.float32(7.0) / np.float32(448.0)
    assert gmax[pos // G] == 7.0 and q[pos] == 0xFE                   # -448
    assert np.all(gmax[np.arange(gmax.size) != pos // G] < 7.0)


def test_per_group_beats_per_tensor_on_spiky_activations(ref):
    # the reason for the mixed granularity (Sec. 5.2): with outliers a single scale wastes the range
    n, G = 64 * 1024, 16
    xb = acts(n, 7)
    x = S.bf16_bits_to_f32(xb).astype(np.float64)
    tab = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    qg, sg = ref.act_quant_group(xb, G)
    qt, ts, _ = ref.act_quant_tensor(xb, G)
    err_g = np.mean((tab[qg] * np.repeat(sg.astype(np.float64), G)[:n] - x) ** 2)
    err_t = np.mean((tab[qt] * ts - x) ** 2)
    assert err_g < err_t / 4


def test_zero_groups_and_empty_input(ref):
    xb = np.zeros(64, np.uint16)
    xb[40] = 0x8000                                    # -0.0
    q, s = ref.act_quant_group(xb, 16)
    assert np.all(s == 0) and np.all((q & 0x7F) == 0) and q[40] == 0x80
    q, ts, gmax = ref.act_quant_tensor(xb, 16)
    assert ts == 0.0 and np.all((q & 0x7F) == 0)
    assert ref.act_quant_group(np.zeros(0, np.uint16), 16)[0].size == 0
