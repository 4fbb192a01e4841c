"""Pins for the oracle's fused AdamW step (no GPU).

  * G = 1 makes the FP8 state lossless up to fp32 rounding of the scale (a one-element group
    is stored as +-448 times its own scale), so ten steps reduce to torch.optim.AdamW, a
    library routine;
  * the first step from the zero state has a closed form: m_hat = g, v_hat = g^2, hence
    w1 = w0 - eta * (g / (|g| + eps) + lambda * w0), and the new moments are (1-beta1) g
    and (1-beta2) g^2;
  * a two-element group worked by hand;
  * the step is the composition dequantize -> update -> quantize of Appendix A, checked
    against the separately pinned quantizer around an AdamW update done in numpy fp64;
  * invariants: v codes never carry a sign, save/reload determinism, group independence.
"""
import math

import numpy as np
import pytest
import torch

import synth_inputs as S

HP = dict(lr=3e-4, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1)


def run_steps(ref, w, grads, G, expand=True, state=None, **over):
    n = w.size
    st = state if state is not None else S.zero_state(n, G)
    hp_kw = dict(HP)
    hp_kw.update(over)
    for t, g in enumerate(grads, start=1):
        hp = ref.make_hparams(step=t, group_size=G, expand=expand, **hp_kw)
        rc = ref.fp8_adamw_step(w, g, st["m_q"], st["m_scale"], st["m_k"],
                                st["v_q"], st["v_scale"], st["v_k"], hp)
        assert rc == 0
    return st


def test_group_size_one_reduces_to_library_adamw(ref):
    n, steps = 4096, 10
    w0 = S.weights(n, seed=0)
    grads = [S.grads_normal(n, seed=0, step=t) for t in range(1, steps + 1)]
    w = w0.copy()
    run_steps(ref, w, grads, G=1)

    p = torch.nn.Parameter(torch.from_numpy(w0.astype(np.float64)))
    opt = torch.optim.AdamW([p], lr=float(np.float32(HP["lr"])),
                            betas=(float(np.float32(HP["beta1"])), float(np.float32(HP["beta2"]))),
                            eps=float(np.float32(HP["eps"])),
                            weight_decay=float(np.float32(HP["weight_decay"])))
    for g in grads:
        p.grad = torch.from_numpy(S.bf16_bits_to_f32(g).astype(np.float64))
        opt.step()
    expect = p.detach().numpy()
    assert np.allclose(w, expect, rtol=1e-6, atol=1e-9)
    assert np.max(np.abs(w - w0)) > 1e-3 * np.max(np.abs(w0))      # the steps did move w


def test_first_step_closed_form(ref):
    n, G = 1024, 128
    w0 = S.weights(n, seed=1)
    g_bits = S.grads_normal(n, seed=1, step=1)
    w = w0.copy()
    st = run_steps(ref, w, [g_bits], G)
    g = S.bf16_bits_to_f32(g_bits).astype(np.float64)
    lr, eps, wd = (float(np.float32(HP[k])) for k in ("lr", "eps", "weight_decay"))
    expect = w0 - lr * (g / (np.abs(g) + eps) + wd * w0.astype(np.float64))
    assert np.allclose(w, expect, rtol=2e-7, atol=1e-10)
    b1, b2 = float(np.float32(HP["beta1"])), float(np.float32(HP["beta2"]))
    m1 = ref.dequant_group(st["m_q"], st["m_scale"], st["m_k"], G, f64=True)
    v1 = ref.dequant_group(st["v_q"], st["v_scale"], st["v_k"], G, f64=True)
    # the stored moments are (1-beta) g and (1-beta) g^2 up to the quantizer's error
    assert np.allclose(st["m_scale"], (1 - b1) * np.abs(g).reshape(-1, G).max(1) / 448.0, rtol=1e-6)
    assert np.allclose(st["v_scale"], (1 - b2) * (g * g).reshape(-1, G).max(1) / 448.0, rtol=1e-6)
    assert np.median(np.abs(m1 / ((1 - b1) * g) - 1)) < 0.02
    assert np.median(np.abs(v1 / ((1 - b2) * g * g) - 1)) < 0.04
    assert np.all(np.sign(m1) == np.sign(g))


def test_two_element_group_by_hand(ref):
    # w = (1, -2), g = (2^-8, -2^-10) (exact in bf16), zero state, t = 1, lambda = 0.
    # m1 = 0.1*g (beta1 = 0.9 as fp32), v1 = 0.05*g^2; |m| ratio 4 -> k_m = log2(229376)/2,
    # |v| ratio 16 -> k_v = log2(229376)/4; max -> code 0x7E, min -> code 0x01, signs kept.
    w = np.array([1.0, -2.0], np.float32)
    g = S.f32_to_bf16_bits(np.array([2.0 ** -8, -(2.0 ** -10)], np.float32))
    st = run_steps(ref, w, [g], G=2, weight_decay=0.0)
    lr, eps = float(np.float32(3e-4)), float(np.float32(1e-8))
    assert w[0] == np.float32(1.0 - lr * (2.0 ** -8 / (2.0 ** -8 + eps)))
    assert w[1] == np.float32(-2.0 + lr * (2.0 ** -10 / (2.0 ** -10 + eps)))
    L = math.log2(229376.0)
    assert st["m_k"][0] == np.float32(L / 2.0) and st["v_k"][0] == np.float32(L / 4.0)
    assert list(st["m_q"]) == [0x7E, 0x81] and list(st["v_q"]) == [0x7E, 0x01]
    one_minus_b1 = 1.0 - float(np.float32(0.9))
    one_minus_b2 = 1.0 - float(np.float32(0.95))
    assert st["m_scale"][0] == np.float32(np.float32(one_minus_b1 * 2.0 ** -8) / 448.0)
    assert st["v_scale"][0] == np.float32(np.float32(one_minus_b2 * 2.0 ** -16) / 448.0)


@pytest.mark.parametrize("G", [32, 128, 512])
def test_step_is_dequant_update_quant(ref, G):
    n = 16 * 512 + 77                                    # ragged tail
    w0 = S.weights(n, seed=2)
    st0 = S.random_state(n, G, seed=2)
    g_bits = S.grads_normal(n, seed=2, step=5, outlier_frac=0.05, G=G)
    t = 5
    w = w0.copy()
    st = {k: v.copy() for k, v in st0.items()}
    hp = ref.make_hparams(step=t, group_size=G, **HP)
    assert ref.fp8_adamw_step(w, g_bits, st["m_q"], st["m_scale"], st["m_k"],
                              st["v_q"], st["v_scale"], st["v_k"], hp) == 0
    # the same, composed by hand around the pinned quantizer
    m = ref.dequant_group(st0["m_q"], st0["m_scale"], st0["m_k"], G, f64=True)
    v = ref.dequant_group(st0["v_q"], st0["v_scale"], st0["v_k"], G, f64=True)
    g = S.bf16_bits_to_f32(g_bits).astype(np.float64)
    b1, b2, lr, eps, wd = (float(np.float32(HP[k])) for k in ("beta1", "beta2", "lr", "eps", "weight_decay"))
    m_t = b1 * m + (1 - b1) * g
    v_t = b2 * v + (1 - b2) * g * g
    w_exp = w0 - lr * ((m_t / (1 - b1 ** t)) / (np.sqrt(v_t / (1 - b2 ** t)) + eps) + wd * w0)
    assert np.array_equal(w, w_exp.astype(np.float32))
    mq, ms, mk = ref.quant_group(m_t.astype(np.float32), G)
    vq, vs, vk = ref.quant_group(v_t.astype(np.float32), G)
    assert np.array_equal(st["m_q"], mq) and np.array_equal(st["m_scale"], ms) and np.array_equal(st["m_k"], mk)
    assert np.array_equal(st["v_q"], vq) and np.array_equal(st["v_scale"], vs) and np.array_equal(st["v_k"], vk)


def test_weight_uses_unquantized_new_moments(ref):
    # Appendix A orders the weight update before Q(m_t), Q(v_t): perturbing nothing but the
    # quantizer (expansion on/off) must leave w after ONE step from a given state unchanged.
    n, G = 2048, 128
    w0 = S.weights(n, seed=3)
    g = S.grads_normal(n, seed=3, step=1)
    wa, wb = w0.copy(), w0.copy()
    run_steps(ref, wa, [g], G, expand=True, state=S.random_state(n, G, seed=3))
    run_steps(ref, wb, [g], G, expand=False, state=S.random_state(n, G, seed=3))
    assert np.array_equal(wa, wb)


def test_second_moment_codes_stay_non_negative(ref):
    n, G = 8192, 128
    w = S.weights(n, seed=4)
    grads = [S.grads_lognormal(n, seed=4, step=t) for t in range(1, 6)]
    st = run_steps(ref, w, grads, G)
    assert np.all(st["v_q"] < 0x80)
    assert np.all(np.isfinite(w))
    assert np.all((st["m_q"] & 0x7F) != 0x7F) and np.all(st["v_q"] != 0x7F)


def test_sign_symmetry_of_the_step(ref):
    # negating w and g negates m and w and leaves v alone (f is odd, Appendix E)
    n, G = 4096, 128
    w0 = S.weights(n, seed=5)
    grads = [S.grads_normal(n, seed=5, step=t) for t in range(1, 4)]
    wa, wb = w0.copy(), -w0
    sa = run_steps(ref, wa, grads, G)
    sb = run_steps(ref, wb, [g ^ np.uint16(0x8000) for g in grads], G)
    assert np.array_equal(wa, -wb)
    assert np.array_equal(sa["m_q"] ^ 0x80, sb["m_q"]) and np.array_equal(sa["v_q"], sb["v_q"])
    assert np.array_equal(sa["m_k"], sb["m_k"]) and np.array_equal(sa["v_scale"], sb["v_scale"])


def test_groups_are_independent_and_reload_is_deterministic(ref):
    n, G = 10 * 128, 128
    w0 = S.weights(n, seed=6)
    grads = [S.grads_normal(n, seed=6, step=t, outlier_frac=0.2, G=G) for t in range(1, 5)]
    w_full = w0.copy()
    st_full = run_steps(ref, w_full, grads, G)
    # group 3 alone gives the same result as inside the batch
    sl = slice(3 * G, 4 * G)
    w_one = w0[sl].copy()
    st_one = run_steps(ref, w_one, [g[sl].copy() for g in grads], G)
    assert np.array_equal(w_one, w_full[sl]) and np.array_equal(st_one["m_q"], st_full["m_q"][sl])
    assert st_one["v_k"][0] == st_full["v_k"][3]
    # stop after two steps, copy the state, continue: identical to uninterrupted stepping
    w_a = w0.copy()
    st_a = run_steps(ref, w_a, grads[:2], G)
    w_b = w_a.copy()
    st_b = {k: v.copy() for k, v in st_a.items()}
    for t in (3, 4):
        hp = ref.make_hparams(step=t, group_size=G, **HP)
        ref.fp8_adamw_step(w_b, grads[t - 1], st_b["m_q"], st_b["m_scale"], st_b["m_k"],
                           st_b["v_q"], st_b["v_scale"], st_b["v_k"], hp)
    assert np.array_equal(w_b, w_full) and np.array_equal(st_b["v_q"], st_full["v_q"])


def test_expansion_lowers_update_error_direction(ref):
    # Table 1 reports that the expansion lowers the error of m / sqrt(v).  Its values need the
    # paper's real optimizer states (parity unpinned); the direction is checked on synthetic
    # moments with the small dynamic ranges Sec. 4.1 describes.
    rng = np.random.default_rng(7)
    n, G = 64 * 128, 128
    m = (rng.standard_normal(n) * 1e-3).astype(np.float32)
    v = (1e-6 * np.exp(rng.uniform(0, math.log(8.0), n))).astype(np.float32)   # range < 1e1
    exact = m.astype(np.float64) / np.sqrt(v.astype(np.float64))

    def mse(expand):
        mq, ms, mk = ref.quant_group(m, G, expand=expand)
        vq, vs, vk = ref.quant_group(v, G, expand=expand)
        mh = ref.dequant_group(mq, ms, mk, G, f64=True)
        vh = ref.dequant_group(vq, vs, vk, G, f64=True)
        return float(np.mean((mh / np.sqrt(vh) - exact) ** 2))

    assert mse(True) < mse(False) / 1.3


def test_argument_errors_and_empty_input(ref):
    hp = ref.make_hparams(step=0, group_size=128, **HP)
    w = np.zeros(128, np.float32)
    st = S.zero_state(128, 128)
    g = np.zeros(128, np.uint16)
    assert ref.fp8_adamw_step(w, g, st["m_q"], st["m_scale"], st["m_k"], st["v_q"], st["v_scale"], st["v_k"], hp) == -1
    hp = ref.make_hparams(step=1, group_size=0, **HP)
    assert ref.lib().coat_ref_fp8_adamw_step(None, None, None, None, None, None, None, None, 0, hp) == 0


def test_bf16_weight_copy_is_library_rounding(ref):
    # the optional bf16 copy is the new fp32 weight rounded to nearest even: torch's cast is the pin
    n, G = 4096 + 33, 128
    w = S.weights(n, seed=8)
    w[:4] = [1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, -(1.0 + 2.0 ** -8), 0.0]      # exact bf16 ties and a zero
    st = S.zero_state(n, G)
    g = S.grads_normal(n, seed=8, step=1)
    g[:4] = 0
    wb = np.zeros(n, np.uint16)
    hp = ref.make_hparams(step=1, group_size=G, lr=3e-4, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.0)
    w_plain = w.copy()
    st2 = S.zero_state(n, G)
    assert ref.fp8_adamw_step(w, g, st["m_q"], st["m_scale"], st["m_k"], st["v_q"], st["v_scale"], st["v_k"], hp, w_bf16=wb) == 0
    assert ref.fp8_adamw_step(w_plain, g, st2["m_q"], st2["m_scale"], st2["m_k"], st2["v_q"], st2["v_scale"], st2["v_k"], hp) == 0
    assert np.array_equal(w, w_plain) and np.array_equal(st["m_q"], st2["m_q"])   # the copy changes nothing else
    lib = torch.from_numpy(w).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(wb, lib)
    assert list(wb[:4]) == [0x3F80, 0x3F82, 0xBF80, 0x0000]                        # ties go to the even mantissa


def test_effect_of_rounding_the_dequantized_moments_to_fp32(ref, capsys):
    """Appendix A writes "dequantize to FP32".  The oracle's default takes the dequantizer as the real
    function and rounds to fp32 what the method stores or decides on; the other reading also rounds
    the dequantized moments (COAT_REF_FLAG_DQ_FP32).  This measures what separates the two: far less
    than the parity bar on the weights, a few codes in 10^5 and, where the update cancels, the group
    exponent k.  (A measurement with loose limits.)"""
    n, G = 512 * 1024, 128
    st_a, st_b = S.zero_state(n, G), S.zero_state(n, G)
    w_a = S.weights(n, 4)
    w_b = w_a.copy()
    worst_w, differ, total, k_off, groups = 0.0, 0, 0, 0, 0
    for t in range(1, 7):
        g = S.grads_normal(n, 4, t, G=G, outlier_frac=0.01)
        hp_a = ref.make_hparams(step=t, group_size=G, **HP)
        hp_b = ref.make_hparams(step=t, group_size=G, **HP)
        hp_b.flags |= ref.FLAG_DQ_FP32
        # lock-step: both readings start every step from the default reading's state
        st_b = {k: v.copy() for k, v in st_a.items()}
        w_b = w_a.copy()
        assert ref.fp8_adamw_step(w_a, g, st_a["m_q"], st_a["m_scale"], st_a["m_k"], st_a["v_q"], st_a["v_scale"], st_a["v_k"], hp_a) == 0
        assert ref.fp8_adamw_step(w_b, g, st_b["m_q"], st_b["m_scale"], st_b["m_k"], st_b["v_q"], st_b["v_scale"], st_b["v_k"], hp_b) == 0
        worst_w = max(worst_w, float(np.max(np.abs(w_a.astype(np.float64) - w_b) / (1e-6 * np.abs(w_a) + 1e-9))))
        for name in ("m", "v"):
            differ += int(np.sum(st_a[name + "_q"] != st_b[name + "_q"]))
            total += n
            k_off += int(np.sum(np.abs(st_a[name + "_k"].astype(np.float64) / st_b[name + "_k"] - 1.0) > 1e-6))
            groups += st_a[name + "_k"].size
    with capsys.disabled():
        print("\n[dequantize to FP32] codes that differ: %d of %d (%.2e); groups with k apart by more than 1e-6: %d of %d; "
              "weights: worst %.3f of the parity tolerance" % (differ, total, differ / total, k_off, groups, worst_w))
    assert worst_w < 0.5 and differ / total < 1e-4 and k_off / groups < 0.05


def test_trajectories_are_sensitive_to_one_ulp_of_metadata(ref, capsys):
    """Why parity is defined in lock-step: the quantized optimizer state is a discontinuous map.  Two runs
    of the ORACLE that differ by one ulp in the first-moment exponents after the first step drift apart
    within ten steps (the difference is amplified where beta1 m + (1 - beta1) g cancels, moves group
    minima, hence k, hence every code of those groups), while the weights stay within a fraction of the
    learning rate of each other and the second moment, which has no cancellation, hardly moves."""
    n, G = 256 * 1024, 128
    w_a = S.weights(n, 6)
    w_b = w_a.copy()
    st_a, st_b = S.zero_state(n, G), S.zero_state(n, G)
    for t in range(1, 11):
        g = S.grads_normal(n, 6, t, G=G, outlier_frac=0.01)
        hp = ref.make_hparams(step=t, group_size=G, **HP)
        for w, st in ((w_a, st_a), (w_b, st_b)):
            assert ref.fp8_adamw_step(w, g, st["m_q"], st["m_scale"], st["m_k"], st["v_q"], st["v_scale"], st["v_k"], hp) == 0
        if t == 1:
            assert all(np.array_equal(st_a[k], st_b[k]) for k in st_a)
            st_b["m_k"] = np.nextafter(st_b["m_k"], np.float32(np.inf))          # one ulp, 6e-8 relative
    m_differ = float(np.mean(st_a["m_q"] != st_b["m_q"]))
    v_differ = float(np.mean(st_a["v_q"] != st_b["v_q"]))
    dw = float(np.max(np.abs(w_a.astype(np.float64) - w_b)))
    with capsys.disabled():
        print("\n[one ulp of k after step 1, ten steps on] first-moment codes that differ: %.3f; second-moment codes: %.1e; "
              "worst |dw| %.2e (lr %.0e)" % (m_differ, v_differ, dw, HP["lr"]))
    assert m_differ > 0.05                       # far beyond any per-step parity rate
    assert v_differ < 1e-2 and dw < HP["lr"]
