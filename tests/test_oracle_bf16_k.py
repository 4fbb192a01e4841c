"""Pins for the oracle's BF16-exponent option.  Sec. 4.2 computes the expansion exponent k for every
group at every step and keeps it with the group's scale, whose storage Sec. 3 gives as BF16.
Reading taken: the stored k is the clamped fp32 exponent rounded to the NEAREST bf16 value (ties to
even: what a cast to bf16 does), and the quantizer and the dequantizer both use that stored value.
The stored exponent is within 2^-8 of the exact one (half a bf16 step), so R_X^k exceeds R_format by
at most R_format^(2^-8): the group's smallest element lands at 0.95 (E4M3; 0.92 for E5M2) of the
smallest subnormal or above and still rounds to it; and a group that receives no gradient keeps its exponent.  No GPU needed."""
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


def bf16_by_torch(k):
    """Independent route to 'the nearest bf16, ties to even': torch's cast."""
    return torch.from_numpy(np.asarray(k, dtype=np.float32)).to(torch.bfloat16).to(torch.float32).numpy()


def bf16_neighbours(k):
    """The bf16 values just below / at and just above a positive fp32 k, by bit truncation."""
    lo = (np.asarray(k, dtype=np.float32).view(np.uint32) & np.uint32(0xFFFF0000))
    return lo.view(np.float32), (lo + np.uint32(0x10000)).view(np.float32)


def test_closed_form_two_magnitudes(ref):
    # a group of a and a * 2^-j: R_X = 2^j, k = log2(448 * 512) / j, stored as the nearest bf16
    G = 32
    for j, a in ((1, 3e-4), (3, 1.0), (7, 2e-6), (17, 5.0), (30, 1e-2)):
        x = np.full(G, a, np.float32)
        x[5::2] = np.float32(a) * np.float32(2.0 ** -j)
        q, s, k = ref.quant_group(x, G, bf16_k=True)
        exact = math.log2(448.0 * 512.0) / j
        assert k[0] == bf16_by_torch([np.float32(exact)])[0]
        assert abs(k[0] / exact - 1.0) <= 2.0 ** -8                       # half a bf16 step at most
        lo, hi = bf16_neighbours([np.float32(exact)])
        assert k[0] == (lo[0] if exact - lo[0] < hi[0] - exact else hi[0])   # the nearer of its two neighbours, by hand
        # the largest elements get the largest code, the smallest a non-zero code
        assert np.all((q[x == x.max()] & 0x7F) == 0x7E) and np.all((q[x == x.min()] & 0x7F) >= 1)


@pytest.mark.parametrize("e5m2", [False, True])
@pytest.mark.parametrize("bf16_scale", [False, True])
def test_stored_k_is_the_nearest_bf16_and_nothing_flushes(ref, e5m2, bf16_scale):
    fmax, fmin = FMT[e5m2]
    n, G = 512 * 128, 128
    x = groups(n, G, 2, spread=6.0)
    q, s, k = ref.quant_group(x, G, e5m2=e5m2, bf16_scale=bf16_scale, bf16_k=True)
    q0, s0, k0 = ref.quant_group(x, G, e5m2=e5m2, bf16_scale=bf16_scale)
    assert np.array_equal(s, s0)                                          # the scale does not depend on how k is stored
    assert np.all(k.view(np.uint32) & 0xFFFF == 0)                        # a bf16 value
    assert np.array_equal(k, bf16_by_torch(k0))                           # ... the one nearest to the fp32 exponent
    assert np.all(np.abs(k.astype(np.float64) / k0 - 1.0) <= 2.0 ** -8)
    assert 0.3 < np.mean(k > k0) < 0.7 and 0.3 < np.mean(k < k0) < 0.7    # to either side, about as often
    # no flush: every non-zero input keeps a non-zero code (k is not on its lower clamp here) ...
    assert np.all(k0 > 0.0625)
    assert np.all((q & 0x7F) != 0)
    # ... because the expanded group leaves the format's range by a factor range^(2^-8) at most: its
    # smallest element lands at that fraction of the smallest subnormal or above, and rounds to it
    ax = np.abs(x.astype(np.float64)).reshape(-1, G)
    top = fmax * s.astype(np.float64)
    low = fmax * (ax.min(1) / top) ** k.astype(np.float64)
    slack = (fmax / fmin) ** -(2.0 ** -8)
    assert np.all(low >= fmin * slack * (1 - 1e-6)) and slack > 0.9
    assert np.mean(low < fmin) > 0.3                                      # and it does land below in the groups rounded up
    assert np.all((q.reshape(-1, G)[np.arange(ax.shape[0]), ax.argmin(1)] & 0x7F) == 1)


@pytest.mark.parametrize("G", [32, 128])
def test_round_trip_with_the_stored_exponent(ref, G):
    # DQ(Q(x)) with the stored (bf16) k: a value between two normal codes (3 mantissa bits) moves by at
    # most half a code step, 2^-4 relative, in the expanded domain: 1 - (1 - 2^-4)^(1/k) on the way back
    n = 256 * G
    x = groups(n, G, 3)
    q, s, k = ref.quant_group(x, G, bf16_k=True)
    back = ref.dequant_group(q, s, k, G, f64=True)
    kk = np.repeat(k.astype(np.float64), G)
    normal = (q & 0x7F) >= 9                                            # the value itself was at or above the smallest normal
    rel = np.abs(back / x.astype(np.float64) - 1.0)
    assert np.all(rel[normal] <= (1.0 - (1.0 - 2.0 ** -4) ** (1.0 / kk[normal])) * (1 + 1e-6) + 1e-6)
    assert np.all(np.sign(back) == np.sign(x))
    # the same codes dequantized with the unrounded exponent would be off by the rounding of k
    q0, s0, k0 = ref.quant_group(x, G)
    moved = ref.dequant_group(q, s, k0, G, f64=True)
    assert np.mean(np.abs(moved / x.astype(np.float64) - 1.0)[normal]) > 1.05 * np.mean(rel[normal])


def test_clamped_and_trivial_groups(ref):
    G = 32
    x = np.full(3 * G, 1e-3, np.float32)
    x[G + 1] = np.nextafter(np.float32(1e-3), np.float32(1))             # R barely above 1: k on its upper clamp
    x[2 * G: 3 * G] = 0.0
    x[2 * G + 3] = 7.0
    x[2 * G + 4] = 7.0e-30                                                # R = 1e30: k = 0.1786, below a lower clamp of 0.3
    q, s, k = ref.quant_group(x, G, bf16_k=True)
    assert k[0] == 1.0 and k[1] == 1024.0                                 # 1 and the default upper clamp: bf16 values already
    assert k[2] == bf16_by_torch([np.float32(math.log2(448.0 * 512.0) / math.log2(1e30))])[0]
    q, s, k = ref.quant_group(x, G, bf16_k=True, k_min=0.3, k_max=777.7)  # bounds that are no bf16 values
    assert k[1] == bf16_by_torch([np.float32(777.7)])[0] and k[2] == bf16_by_torch([np.float32(0.3)])[0]
    # without expansion k is 1 whatever the flag says
    q, s, k = ref.quant_group(x, G, expand=False, bf16_k=True)
    assert np.all(k == 1.0)


def test_step_stores_bf16_exponents_for_both_moments(ref):
    n, G = 64 * 128 + 40, 128
    w = S.weights(n, 1)
    st = S.zero_state(n, G)
    st0 = {key: v.copy() for key, v in st.items()}
    w0 = w.copy()
    for t in (1, 2, 3):
        g = S.grads_normal(n, 1, t, G=G, outlier_frac=0.02)
        assert ref.fp8_adamw_step(w, g, st["m_q"], st["m_scale"], st["m_k"], st["v_q"], st["v_scale"], st["v_k"],
                                  ref.make_hparams(step=t, group_size=G, bf16_k=True, **HP)) == 0
        assert ref.fp8_adamw_step(w0, g, st0["m_q"], st0["m_scale"], st0["m_k"], st0["v_q"], st0["v_scale"], st0["v_k"],
                                  ref.make_hparams(step=t, group_size=G, **HP)) == 0
        for name in ("m_k", "v_k"):
            assert np.all(st[name].view(np.uint32) & 0xFFFF == 0)
            if t == 1:                                                    # same inputs on both sides at the first step
                assert np.array_equal(st[name], bf16_by_torch(st0[name]))
        assert np.all(st["v_q"] < 0x80)
    # the trajectories stay close: the stored exponent moves a dequantized value by less than its own quantization step
    assert np.max(np.abs(w - w0)) < 1e-4


def test_groups_without_gradient_keep_their_exponent(ref):
    """A group that receives no gradient only decays (m_t = beta1 m, v_t = beta2 v): the range of its
    dequantized values is the one its stored k made of the format's range, so the exponent computed
    from it is the stored one again -- a bf16 value, which the rounding keeps.  Wherever the group's
    extremes sat at the format's two ends (code fmax and the smallest subnormal) the exponent must
    not move over idle steps, and the codes stay as they are."""
    G, n = 128, 128 * 512
    keys = ("m_q", "m_scale", "m_k", "v_q", "v_scale", "v_k")
    w, st = S.weights(n, 5), S.zero_state(n, G)
    assert ref.fp8_adamw_step(w, S.grads_normal(n, 5, 1), *(st[k] for k in keys),
                              ref.make_hparams(step=1, group_size=G, bf16_k=True, **HP)) == 0
    first = {k: v.copy() for k, v in st.items()}
    idle = np.zeros(n, np.uint16)
    for t in range(2, 22):
        assert ref.fp8_adamw_step(w, idle, *(st[k] for k in keys), ref.make_hparams(step=t, group_size=G, bf16_k=True, **HP)) == 0
    for name in ("m", "v"):
        mag = (first[name + "_q"] & 0x7F).reshape(-1, G)
        ends = (mag.max(1) == 0x7E) & (np.where(mag > 0, mag, 0x7F).min(1) == 1)    # both ends of E4M3 in use
        assert ends.mean() > 0.9
        assert np.array_equal(st[name + "_k"][ends], first[name + "_k"][ends])
        assert np.array_equal(st[name + "_q"].reshape(-1, G)[ends], first[name + "_q"].reshape(-1, G)[ends])
