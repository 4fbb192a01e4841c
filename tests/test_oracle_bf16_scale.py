"""Pins for the oracle's BF16-scale option (Sec. 3: the scaling factor of the optimizer states is
stored in BF16).  Reading taken: the stored scale is amax/fmax rounded UP to a bf16 value, the
quantizer and the dequantizer both use that stored value, and k is chosen from the range
(fmax * scale) / amin that the normalized group really spans.  No GPU needed."""
import math

import numpy as np
import pytest
import torch

import synth_inputs as S

HP = dict(lr=3e-4, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1)
FMT = {False: (448.0, 2.0 ** -9), True: (57344.0, 2.0 ** -16)}


def groups(n, G, seed, spread=3.0):
    rng = np.random.default_rng(seed)
    scale = np.exp(rng.normal(0.0, 2.0, n // G))[:, None]
    x = scale * 1e-3 * np.exp(rng.uniform(0.0, spread, (n // G, G))) * rng.choice([-1.0, 1.0], (n // G, G))
    return x.astype(np.float32).reshape(-1)


def bf16_ceil_by_torch(s):
    """Independent route to 'the smallest bf16 that is not below s': torch's nearest-even cast,
    bumped by one bf16 step where it fell below."""
    t = torch.from_numpy(s.astype(np.float32))
    b = t.to(torch.bfloat16)
    low = b.to(torch.float32) < t
    bits = b.view(torch.int16).to(torch.int32) + low.to(torch.int32)     # positive values: next bf16 up
    return bits.to(torch.int16).view(torch.bfloat16).to(torch.float32).numpy()


@pytest.mark.parametrize("e5m2", [False, True])
@pytest.mark.parametrize("expand", [True, False])
def test_scale_is_the_bf16_ceiling_and_nothing_saturates(ref, e5m2, expand):
    fmax, fmin = FMT[e5m2]
    n, G = 512 * 128, 128
    x = groups(n, G, 1)
    q, s, k = ref.quant_group(x, G, expand=expand, e5m2=e5m2, bf16_scale=True)
    q0, s0, k0 = ref.quant_group(x, G, expand=expand, e5m2=e5m2)
    assert np.all(s.view(np.uint32) & 0xFFFF == 0)                        # a bf16 value
    assert np.array_equal(s, bf16_ceil_by_torch(s0))                      # ... the ceiling of the fp32 scale
    ax = np.abs(x.astype(np.float64)).reshape(-1, G)
    assert np.all(fmax * s.astype(np.float64) >= ax.max(1))               # every |x| / (fmax scale) <= 1
    assert np.all(s <= s0 * (1 + 2.0 ** -7))
    dec = ref.e5m2_decode if e5m2 else ref.e4m3_decode
    mag = np.abs(np.array([dec(int(c)) for c in range(256)]))[q].reshape(-1, G)
    assert np.all(np.isfinite(mag)) and np.all(mag <= fmax)
    if expand:
        # k from the range the normalized group spans: (fmax scale / amin)^k = R_format, so the smallest
        # element still lands on the smallest subnormal (it is NOT flushed), the largest just below fmax
        free = (k > 0.0625) & (k < 1024.0)
        want = math.log2(fmax / fmin) / np.log2(fmax * s.astype(np.float64) / ax.min(1))
        assert np.allclose(k[free], want[free], rtol=2e-7)
        rows = np.arange(mag.shape[0])
        assert np.all(mag[rows, ax.argmin(1)][free] == fmin)
        assert np.all(mag[rows, ax.argmax(1)] > 0.3 * fmax)               # (1 - 2^-7)^k with k <= ~9 here
        assert np.all(k <= k0)                                            # never more expansion than with the exact scale
    else:
        assert np.all(k == 1.0)


@pytest.mark.parametrize("e5m2", [False, True])
def test_round_trip_error_is_that_of_the_format(ref, e5m2):
    # x -> codes -> x': for codes that are normal numbers the relative error is at most half a code
    # step seen through the inverse expansion, 1 - (1 - 2^-(p+1))^(1/k), whatever the scale's rounding
    fmax, fmin = FMT[e5m2]
    p = 2 if e5m2 else 3
    n, G = 256 * 128, 128
    x = groups(n, G, 2)
    q, s, k = ref.quant_group(x, G, e5m2=e5m2, bf16_scale=True)
    xh = ref.dequant_group(q, s, k, G, f64=True, e5m2=e5m2)
    dec = ref.e5m2_decode if e5m2 else ref.e4m3_decode
    mag = np.abs(np.array([dec(int(c)) for c in range(256)]))[q]
    normal = mag >= fmin * 2 ** p * 2
    kk = np.repeat(k.astype(np.float64), G)
    rel = np.abs(xh / x.astype(np.float64) - 1.0)
    bound = (1 + 2.0 ** -(p + 1)) ** (1 / kk) - 1 + 1e-6
    assert np.all(rel[normal] <= bound[normal])
    assert np.all(np.sign(xh) == np.sign(x))


def test_tiny_inner_range_does_not_collapse(ref):
    # amax/amin = 1.01: k from amax/amin alone would be ~1240 (clamped to 1024) and, with a scale that
    # is up to 0.8 % too large, (amax / (448 scale))^k would shrink the whole group by e^-8.  With the
    # range taken against 448*scale the group keeps its resolution.
    rng = np.random.default_rng(3)
    G = 128
    x = (1e-3 * (1.0 + 0.01 * rng.random(64 * G))).astype(np.float32)
    q, s, k = ref.quant_group(x, G, bf16_scale=True)
    xh = ref.dequant_group(q, s, k, G, f64=True)
    assert np.all((q & 0x7F) > 0)                                          # nothing flushed
    assert np.max(np.abs(xh / x - 1.0)) < 2e-3                             # far finer than E4M3's 6 %
    assert len(np.unique(q)) > 8                                           # the codes still tell values apart


def test_step_with_bf16_scale_is_dequant_update_quant(ref):
    n, G, t = 8 * 128 + 50, 128, 4
    w0 = S.weights(n, seed=3)
    g_bits = S.grads_normal(n, seed=3, step=t, outlier_frac=0.1, G=G)
    rng = np.random.default_rng(5)
    m0 = (rng.standard_normal(n) * 2e-4).astype(np.float32)
    v0 = ((rng.standard_normal(n) * 1e-3) ** 2 * 0.3).astype(np.float32)
    mq, ms, mk = ref.quant_group(m0, G, bf16_scale=True)
    vq, vs, vk = ref.quant_group(v0, G, bf16_scale=True)
    st = dict(m_q=mq.copy(), m_scale=ms.copy(), m_k=mk.copy(), v_q=vq.copy(), v_scale=vs.copy(), v_k=vk.copy())
    w = w0.copy()
    hp = ref.make_hparams(step=t, group_size=G, bf16_scale=True, **HP)
    assert ref.fp8_adamw_step(w, g_bits, st["m_q"], st["m_scale"], st["m_k"], st["v_q"], st["v_scale"], st["v_k"], hp) == 0
    m = ref.dequant_group(mq, ms, mk, G, f64=True)
    v = ref.dequant_group(vq, vs, vk, G, f64=True)
    g = S.bf16_bits_to_f32(g_bits).astype(np.float64)
    b1, b2, lr, eps, wd = (float(np.float32(HP[k_])) for k_ in ("beta1", "beta2", "lr", "eps", "weight_decay"))
    m_t = b1 * m + (1 - b1) * g
    v_t = b2 * v + (1 - b2) * g * g
    w_exp = w0 - lr * ((m_t / (1 - b1 ** t)) / (np.sqrt(v_t / (1 - b2 ** t)) + eps) + wd * w0)
    assert np.array_equal(w, w_exp.astype(np.float32))
    mq2, ms2, mk2 = ref.quant_group(m_t.astype(np.float32), G, bf16_scale=True)
    vq2, vs2, vk2 = ref.quant_group(v_t.astype(np.float32), G, bf16_scale=True)
    assert np.array_equal(st["m_q"], mq2) and np.array_equal(st["m_scale"], ms2) and np.array_equal(st["m_k"], mk2)
    assert np.array_equal(st["v_q"], vq2) and np.array_equal(st["v_scale"], vs2) and np.array_equal(st["v_k"], vk2)
    assert np.all(st["m_scale"].view(np.uint32) & 0xFFFF == 0) and np.all(st["v_scale"].view(np.uint32) & 0xFFFF == 0)
