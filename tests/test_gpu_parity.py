"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element,
on identical seeded inputs.  Multi-step cases run in lock-step: at every step both sides
start from the oracle's state, so that an allowed one-step code difference at a rounding tie
cannot grow into a weight difference at the next step."""
import numpy as np
import pytest
import torch

import synth_inputs as S
from parity import (K_EXCEPTION_MAX, allowed_mismatches, assert_codes, assert_k, assert_scale, assert_w, eps_dq, k_bar,
                    k_tolerance)

pytestmark = pytest.mark.gpu

HP = dict(lr=3e-4, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1)
GROUPS = [32, 64, 128, 256, 512]


@pytest.fixture(scope="module")
def coat():
    import paper_2410_19313_amd as C
    assert torch.cuda.is_available(), "these tests need the GPU"
    C.lib()
    return C


def dev(a):
    t = torch.from_numpy(np.ascontiguousarray(a))
    return t.cuda()


def dev_bf16(bits):
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)


def gpu_step(coat, w, g_bits, st, G, step, expand=True, **over):
    kw = dict(HP)
    kw.update(over)
    hp = coat.make_hparams(step=step, group_size=G, expand=expand, **kw)
    tw, tg = dev(w), dev_bf16(g_bits)
    ts = {k: dev(v) for k, v in st.items()}
    # the oracle keeps bf16 scales / exponents as floats whose values are bf16: the conversion is exact
    for flag, keys in (("bf16_scale", ("m_scale", "v_scale")), ("bf16_k", ("m_k", "v_k"))):
        if kw.get(flag):
            for k in keys:
                assert np.all(st[k].view(np.uint32) & 0xFFFF == 0)
                ts[k] = ts[k].to(torch.bfloat16)
    coat.coat_fp8_adamw_step(tw, tg, ts["m_q"], ts["m_scale"], ts["m_k"], ts["v_q"], ts["v_scale"], ts["v_k"], hp)
    torch.cuda.synchronize()
    return tw.cpu().numpy(), {k: v.float().cpu().numpy() if v.dtype == torch.bfloat16 else v.cpu().numpy()
                              for k, v in ts.items()}, tg


def ref_step(ref, w, g_bits, st, G, step, expand=True, **over):
    kw = dict(HP)
    kw.update(over)
    kw.pop("precise_dq", None)                   # a choice of the kernels' arithmetic: the reference is the same
    hp = ref.make_hparams(step=step, group_size=G, expand=expand, **kw)
    w = w.copy()
    st = {k: v.copy() for k, v in st.items()}
    assert ref.fp8_adamw_step(w, g_bits, st["m_q"], st["m_scale"], st["m_k"],
                              st["v_q"], st["v_scale"], st["v_k"], hp) == 0
    return w, st


def new_moments(ref, st_old, g_bits, G, hp_over):
    """The fp64 new moments of the reference side and the bound dx on how far the fp32 side's
    moments may be from them (see parity.py).  Used for the k bar (ln R) and for the bound that
    exception groups must obey, never as expected values."""
    kw = dict(HP)
    kw.update({k: v for k, v in hp_over.items() if k in HP})
    b1, b2 = float(np.float32(kw["beta1"])), float(np.float32(kw["beta2"]))
    n = st_old["m_q"].size
    m_e5, v_e5 = bool(hp_over.get("m_e5m2")), bool(hp_over.get("v_e5m2"))
    m_old = ref.dequant_group(st_old["m_q"], st_old["m_scale"], st_old["m_k"], G, f64=True, e5m2=m_e5)
    v_old = ref.dequant_group(st_old["v_q"], st_old["v_scale"], st_old["v_k"], G, f64=True, e5m2=v_e5)
    g = S.bf16_bits_to_f32(g_bits).astype(np.float64)
    m_t = b1 * m_old + (1 - b1) * g
    v_t = b2 * v_old + (1 - b2) * g * g
    em = eps_dq(st_old["m_k"].astype(np.float64), 31.81 if m_e5 else 17.81)
    ev = eps_dq(st_old["v_k"].astype(np.float64), 31.81 if v_e5 else 17.81)
    dm = np.repeat(em, G)[:n] * b1 * np.abs(m_old) + 2.0 ** -22 * np.abs(m_t)
    dv = np.repeat(ev, G)[:n] * b2 * v_old + 2.0 ** -22 * v_t
    return m_t, dm, v_t, dv


def check_step(ref, tag, w_g, st_g, w_r, st_r, st_old, g_bits, G, expand=True, extra_w_tol=None, **over):
    """The parity bar of tests/parity.py on one step.  st_old: the state both sides started from.
    Returns per-moment statistics (mismatches, mismatches of more than a step, exception groups)."""
    k_min = over.get("k_min", 0.0) or 0.0625
    k_max = over.get("k_max", 0.0) or 1024.0
    stats = {"w": assert_w(w_g, w_r, tag + " w", extra_w_tol)}
    m_t, dm, v_t, dv = new_moments(ref, st_old, g_bits, G, over)
    k_unrounded = None
    if over.get("bf16_k"):
        # the reference exponents BEFORE their rounding to bf16: the same oracle step without that flag
        # (scales and moments do not depend on how k is stored)
        _, k_unrounded = ref_step(ref, np.zeros(st_old["m_q"].size, np.float32), g_bits, st_old, G, 1, expand,
                                  **{**over, "bf16_k": False})
    for name, x, dx in (("m", m_t, dm), ("v", v_t, dv)):
        x32 = x.astype(np.float32).astype(np.float64)     # both sides hold the new moments as fp32
        bound, _ = k_tolerance(st_r[name + "_k"], x32, dx, G, k_min, k_max)
        bar = k_bar(x32, G)
        excused = None
        if over.get("bf16_scale"):
            # The stored scale is a rounding DECISION (the bf16 ceiling of amax/fmax).  Where the two
            # sides' amax (fp32 against fp64 arithmetic, within dx of each other) straddle a bf16
            # boundary they may decide differently, by one bf16 step; such a group's k and codes then
            # all shift and it is an exception group.  Everywhere else: EQUAL.
            near, lo16, hi16 = bf16_scale_candidates(x, dx, G, 57344.0 if over.get(name + "_e5m2") else 448.0)
            sg, sr = st_g[name + "_scale"], st_r[name + "_scale"]
            assert np.all(sg.view(np.uint32) & 0xFFFF == 0), tag + ": a stored scale is not a bf16 value"
            assert np.array_equal(sg[~near], sr[~near]), tag + " %s scale (bf16)" % name
            assert np.all((sg[near] == lo16[near]) | (sg[near] == hi16[near])), tag + " %s scale near a bf16 boundary" % name
            # (How many groups sit that near a boundary depends on the data: a few in 10^4 for generic
            # gradients, but a group whose gradient is all zero has the new maximum beta1 * fmax * (its
            # old bf16 scale), and 0.9f times a bf16 significand that is a multiple of ten lies within
            # 3e-8 of a bf16 value: with sparse gradients about one group in a hundred is a coin flip
            # of the last fp32 rounding, on either side.  So the count is not limited, only where.)
            excused = near & (sg != sr)
            bound = np.where(excused, np.inf, bound)
        else:
            assert_scale(st_g[name + "_scale"], st_r[name + "_scale"], tag + " %s scale" % name)
        if not expand or over.get(name + "_plain"):
            assert np.all(st_g[name + "_k"] == 1.0) and np.all(st_r[name + "_k"] == 1.0)   # k is 1 on both sides
        if over.get("bf16_k"):
            exc, kstats = check_bf16_k(tag + " %s k" % name, st_g[name + "_k"], st_r[name + "_k"], k_unrounded[name + "_k"],
                                       bar, bound, excused)
            excused = exc                                     # their codes are relative to another exponent
        else:
            exc, kstats = assert_k(st_g[name + "_k"], st_r[name + "_k"], bar, tag + " %s k" % name, bound=bound, excused=excused)
        n_bad, n_far = assert_codes(ref, st_g[name + "_q"], st_r[name + "_q"], G, tag + " %s codes" % name, exception=exc,
                                    x_ref=x, dx=dx, scale_ref=st_r[name + "_scale"], k_ref=st_r[name + "_k"], bound=bound,
                                    e5m2=bool(over.get(name + "_e5m2")), other_scale=excused)
        stats[name] = dict(bad=n_bad, far=n_far, n=int(x.size), groups=int(bar.size), **kstats)
    # the second moment has no cancellation and takes no exception: plain bar everywhere
    if not over.get("bf16_scale") and not over.get("bf16_k"):
        assert stats["v"]["k_out"] == 0, tag + ": v k outside the bar in %d groups" % stats["v"]["k_out"]
    assert np.all(st_g["v_q"] < 0x80), tag + ": a second-moment code carries a sign"
    return stats


def bf16_nearest(k):
    """The nearest bf16, ties to even, by integer arithmetic on the fp32 bits (positive finite k)."""
    u = np.asarray(k, dtype=np.float32).view(np.uint32)
    return ((u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)).view(np.float32)


def check_bf16_k(tag, k_gpu, k_ref, k_exact, bar, bound, excused):
    """BF16-stored exponents: the stored k is a rounding DECISION (the clamped exponent rounded to the
    nearest bf16).  k_exact: the reference exponent before that rounding.  Where k_exact is further
    than twice the plain bar from a rounding boundary (the midpoint of two bf16 values) both sides
    must store the SAME value; nearer than that either neighbour is right -- how many groups sit
    there depends on the data and is not limited.  The "two candidates" exception of parity.py keeps
    its own limit (1e-4 of the groups, each within its bound plus one bf16 step).  Returns (groups
    whose stored k differs, statistics)."""
    assert np.all(k_gpu.view(np.uint32) & 0xFFFF == 0), tag + ": a stored k is not a bf16 value"
    assert np.array_equal(k_ref, bf16_nearest(k_exact)), tag + ": the reference k is not its own exponent rounded to bf16"
    k64 = k_exact.astype(np.float64)
    lo16, hi16 = bf16_nearest(k64 * (1.0 - 2.0 * bar)), bf16_nearest(k64 * (1.0 + 2.0 * bar))
    near = lo16 != hi16
    differ = k_gpu != k_ref
    if excused is not None:
        differ_own = differ & ~excused                         # a different bf16 scale moves k as a whole
    else:
        differ_own = differ
    decided = differ_own & near
    assert np.all((k_gpu[decided] == lo16[decided]) | (k_gpu[decided] == hi16[decided])), tag + ": near a bf16 boundary"
    out = differ_own & ~near
    assert int(out.sum()) <= int(np.ceil(K_EXCEPTION_MAX * differ.size)), \
        tag + ": stored k differs away from a bf16 boundary in %d of %d groups" % (int(out.sum()), differ.size)
    rel = np.abs(k_gpu.astype(np.float64) / k_ref - 1.0)
    assert np.all(rel[out] <= bound[out] + 2.0 ** -7), tag + ": an exception group's k outside its bound"
    return (differ if excused is None else differ | excused), dict(k_out=int(out.sum()), k_in_bar=float(1.0 - out.mean()),
                                                                    k_max_rel=float(rel.max()), k_decisions=int(decided.sum()))


def bf16_ceil(s):
    s = np.asarray(s, dtype=np.float32)
    return ((s.view(np.uint32) + np.uint32(0xFFFF)) & np.uint32(0xFFFF0000)).view(np.float32)


def bf16_scale_candidates(x, dx, G, fmax):
    """Per group: the bf16 scales that amax - dx and amax + dx lead to, and whether they differ."""
    ax = np.abs(np.asarray(x, dtype=np.float64))
    n = ax.size
    ng = (n + G - 1) // G
    pad_lo, pad_hi = np.zeros(ng * G), np.zeros(ng * G)
    pad_lo[:n] = np.maximum(ax - dx, 0.0)
    pad_hi[:n] = ax + dx
    lo = (pad_lo.reshape(ng, G).max(1) / fmax * (1 - 2.0 ** -22)).astype(np.float32)
    hi = (pad_hi.reshape(ng, G).max(1) / fmax * (1 + 2.0 ** -22)).astype(np.float32)
    lo16, hi16 = bf16_ceil(lo), bf16_ceil(hi)
    return lo16 != hi16, lo16, hi16


TOTALS = {}     # tag -> accumulated statistics of the lock-step runs, printed at the end of the module


def lockstep(coat, ref, n, G, grads_fn, steps, seed, expand=True, state=None, update_model=False, **over):
    """update_model: add the fp32 error model of the update itself to the weight tolerance.  Only for
    cells in which the second moment is stored WITHOUT expansion: its small entries flush to zero,
    the update m / (sqrt(v) + eps) then exceeds the weight (up to 1e4 times under log-normal gradients;
    under normal ones an element whose stored v is zero and whose next gradient is tiny, one weight in
    2e8 element-steps was seen at 2.4 times the plain tolerance), and 1e-6 of the weight is below the
    fp32 resolution of the update."""
    w = S.weights(n, seed)
    st = state if state is not None else S.zero_state(n, G)
    tot = dict(bad=0, far=0, k_out=0, elems=0, groups=0, w=0.0)
    for t in range(1, steps + 1):
        g = grads_fn(t)
        w_g, st_g, _ = gpu_step(coat, w, g, st, G, t, expand, **over)
        st_old = st
        w, st = ref_step(ref, w, g, st, G, t, expand, **over)
        extra = update_error_model(ref, st_old, g, G, t, **over) if update_model else None
        stats = check_step(ref, "n=%d G=%d step %d" % (n, G, t), w_g, st_g, w, st, st_old, g, G, expand,
                           extra_w_tol=extra, **over)
        for name in ("m", "v"):
            tot["bad"] += stats[name]["bad"]; tot["far"] += stats[name]["far"]; tot["k_out"] += stats[name]["k_out"]
            tot["elems"] += stats[name]["n"]; tot["groups"] += stats[name]["groups"]
        tot["w"] = max(tot["w"], stats["w"])
    # over the whole run the rate must hold too
    assert tot["bad"] <= allowed_mismatches(tot["elems"]), tot
    key = "G=%d%s" % (G, "" if not over and expand else " other")
    acc = TOTALS.setdefault(key, dict(bad=0, far=0, k_out=0, elems=0, groups=0, w=0.0))
    for k_ in ("bad", "far", "k_out", "elems", "groups"):
        acc[k_] += tot[k_]
    acc["w"] = max(acc["w"], tot["w"])
    return tot


def update_error_model(ref, st, g, G, t, m_e5m2=False, v_e5m2=False, **_):
    """Extra weight tolerance for states that come from no optimizer trajectory (random codes,
    scales and exponents): there |m| / sqrt(v) reaches 1e5, the update dwarfs the weight and the
    fp32 error of the update itself shows.  For u = (lr/bc1) m_t / (sqrt(v_t/bc2) + eps) the
    dequantized m carries EPS_DQ_M, the dequantized v eps_dq_v (halved by the square root), the
    remaining operations a few ulp."""
    n = st["m_q"].size
    b1, b2, lr, eps = (float(np.float32(HP[k])) for k in ("beta1", "beta2", "lr", "eps"))
    m_old = np.abs(ref.dequant_group(st["m_q"], st["m_scale"], st["m_k"], G, f64=True, e5m2=m_e5m2))
    v_old = ref.dequant_group(st["v_q"], st["v_scale"], st["v_k"], G, f64=True, e5m2=v_e5m2)
    gf = S.bf16_bits_to_f32(g).astype(np.float64)
    denom = np.sqrt((b2 * v_old + (1 - b2) * gf * gf) / (1 - b2 ** t)) + eps
    u_scale = lr / (1 - b1 ** t) * (b1 * m_old + (1 - b1) * np.abs(gf)) / denom
    em = np.repeat(eps_dq(st["m_k"].astype(np.float64), 31.81 if m_e5m2 else 17.81), G)[:n]
    ev = np.repeat(eps_dq(st["v_k"].astype(np.float64), 31.81 if v_e5m2 else 17.81), G)[:n]
    return u_scale * (em + 0.5 * ev + 6 * 2.0 ** -24)


# --- dequantizer -------------------------------------------------------------------------------

@pytest.mark.parametrize("G", GROUPS)
def test_dequant_every_code(coat, ref, G):
    # every code byte under a spread of exponents and scales; n spans several chunks + a tail
    n = 5 * 1024 + 3 * G + 5
    rng = np.random.default_rng(G)
    q = (np.arange(n) % 256).astype(np.uint8)
    rng.shuffle(q)
    ng = (n + G - 1) // G
    scale = np.exp(rng.uniform(np.log(1e-14), np.log(1e-2), ng)).astype(np.float32)
    k = np.exp(rng.uniform(np.log(0.3), np.log(40.0), ng)).astype(np.float32)
    k[::5] = 1.0
    x_g = coat.coat_dequant_group(dev(q), dev(scale), dev(k), G).cpu().numpy()
    x_r = ref.dequant_group(q, scale, k, G, f64=True)
    nan = (q & 0x7F) == 0x7F
    assert np.all(np.isnan(x_g[nan]))
    ok = ~nan
    # x = a * exp2(L / k), L = log2|c/448| in [-17.81, 0].  fp32 error model: L (table) and 1/k are
    # each rounded, their product is rounded (3 * 2^-24 relative on the exponent, i.e. an absolute
    # exponent error of |L/k| * 3 * 2^-24 and a relative error of ln2 times that on x), the hardware
    # exp2 is good to ~1.5 ulp and two more roundings follow (448*scale and the final product).
    L = np.log2(np.maximum(np.abs(np.array([ref.e4m3_decode(int(c) & 0x7F) for c in range(256)])), 1e-300) / 448.0)
    expo = np.abs(L[q]) / np.repeat(k.astype(np.float64), G)[:n]
    tol = (expo * 3 * 2.0 ** -24 * np.log(2.0) + 4 * 2.0 ** -24) * 1.25
    err = np.abs(x_g[ok] - x_r[ok]) / np.abs(np.where(x_r[ok] == 0, 1.0, x_r[ok]))
    assert np.all(err <= tol[ok]), float((err / tol[ok]).max())
    assert np.array_equal(np.signbit(x_g[ok]), np.signbit(x_r[ok]))
    assert np.all(x_g[(q & 0x7F) == 0] == 0)
    # the standalone dequantizer uses the compensated exponent: a few ulp whatever the exponent
    assert np.all(err <= 8 * 2.0 ** -24), float(err.max())


# --- quantizer ---------------------------------------------------------------------------------

def quant_inputs(kind, n, seed):
    rng = np.random.default_rng(seed)
    if kind == "normal":
        return (rng.standard_normal(n) * 1e-3).astype(np.float32)
    if kind == "square":
        return ((rng.standard_normal(n) * 1e-3) ** 2).astype(np.float32)
    if kind == "lognormal":
        return (1e-3 * np.exp(2 * rng.standard_normal(n)) * rng.choice([-1.0, 1.0], n)).astype(np.float32)
    if kind == "zeros_mixed":
        x = (rng.standard_normal(n) * 1e-3).astype(np.float32)
        x[rng.random(n) < 0.3] = 0.0
        x[: min(n, 700)] = 0.0                       # whole groups of zeros
        return x
    raise ValueError(kind)


def check_quant(ref, tag, x, G, gpu, expect, expand, e5m2=False):
    """Standalone quantizer: both sides see the same fp32 inputs, so the stated bar applies as it
    stands and no exception is allowed (k: 1e-6, on ln R for groups narrower than e)."""
    (q_g, s_g, k_g), (q_r, s_r, k_r) = gpu, expect
    assert_scale(s_g, s_r, tag)
    if not expand:
        assert np.all(k_g == 1.0) and np.all(k_r == 1.0)
    assert_k(k_g, k_r, k_bar(x, G), tag)
    assert_codes(ref, q_g, q_r, G, tag, e5m2=e5m2)


@pytest.mark.parametrize("G", GROUPS)
@pytest.mark.parametrize("kind", ["normal", "square", "lognormal", "zeros_mixed"])
@pytest.mark.parametrize("expand", [True, False])
def test_quant_parity(coat, ref, G, kind, expand):
    n = 37 * 1024 + 2 * G + 17
    x = quant_inputs(kind, n, seed=G + len(kind))
    q_g, s_g, k_g = (t.cpu().numpy() for t in coat.coat_quant_group(dev(x), G, expand=expand))
    q_r, s_r, k_r = ref.quant_group(x, G, expand=expand)
    tag = "quant %s G=%d expand=%s" % (kind, G, expand)
    check_quant(ref, tag, x, G, (q_g, s_g, k_g), (q_r, s_r, k_r), expand)
    if kind == "square":
        assert np.all(q_g < 0x80)


@pytest.mark.parametrize("n", [1, 15, 16, 17, 127, 128, 129, 1023, 1024, 1025, 4096 + 511])
def test_quant_small_and_ragged_sizes(coat, ref, n):
    x = quant_inputs("normal", n, seed=n)
    q_g, s_g, k_g = (t.cpu().numpy() for t in coat.coat_quant_group(dev(x), 128))
    q_r, s_r, k_r = ref.quant_group(x, 128)
    check_quant(ref, "n=%d" % n, x, 128, (q_g, s_g, k_g), (q_r, s_r, k_r), True)


def test_quant_roundtrip_through_dequant(coat, ref):
    n, G = 64 * 1024, 128
    x = quant_inputs("normal", n, seed=3)
    q, s, k = coat.coat_quant_group(dev(x), G)
    xh = coat.coat_dequant_group(q, s, k, G).cpu().numpy()
    rel = np.abs(xh / x - 1.0)
    assert np.median(rel) < 2.0 ** -5 and np.all(np.sign(xh) == np.sign(x))


def test_quant_does_not_touch_neighbours(coat):
    # outputs are written only inside [0, n): canaries around every buffer survive
    n, G, pad = 3 * 1024 + 77, 128, 256
    x = dev(quant_inputs("normal", n, 5))
    ng = (n + G - 1) // G
    qbuf = torch.full((n + 2 * pad,), 0xAB, dtype=torch.uint8, device="cuda")
    sbuf = torch.full((ng + 2 * pad,), -7.0, dtype=torch.float32, device="cuda")
    kbuf = torch.full((ng + 2 * pad,), -7.0, dtype=torch.float32, device="cuda")
    coat.coat_quant_group(x, G, out=(qbuf[pad:pad + n], sbuf[pad:pad + ng], kbuf[pad:pad + ng]))
    torch.cuda.synchronize()
    assert torch.all(qbuf[:pad] == 0xAB) and torch.all(qbuf[pad + n:] == 0xAB)
    assert torch.all(sbuf[:pad] == -7.0) and torch.all(sbuf[pad + ng:] == -7.0)
    assert torch.all(kbuf[:pad] == -7.0) and torch.all(kbuf[pad + ng:] == -7.0)


# --- the fused step ------------------------------------------------------------------------------

def test_step_cfg1_ten_steps(coat, ref):
    # 1024 x 1024 master weight, grads ~ N(0, 1e-3), G = 128, ten steps, seed 0
    n = S.workload_numel("cfg1")
    lockstep(coat, ref, n, 128, lambda t: S.grads_normal(n, 0, t), steps=10, seed=0)


@pytest.mark.parametrize("G", GROUPS)
def test_step_outlier_groups_ragged(coat, ref, G):
    n = 300 * 1024 + 5 * G + 9
    lockstep(coat, ref, n, G, lambda t: S.grads_normal(n, 1, t, G=G, outlier_frac=0.01), steps=4, seed=1)


@pytest.mark.parametrize("G", [32, 128, 512])
def test_step_lognormal_grads(coat, ref, G):
    n = 256 * 1024
    lockstep(coat, ref, n, G, lambda t: S.grads_lognormal(n, 2, t), steps=4, seed=2)


@pytest.mark.parametrize("G", GROUPS)
def test_step_from_arbitrary_state(coat, ref, G):
    n = 128 * 1024 + G + 3
    st = S.random_state(n, G, seed=4)
    w = S.weights(n, 4)
    g = S.grads_normal(n, 4, 1, G=G, outlier_frac=0.02)
    t = 7
    w_g, st_g, _ = gpu_step(coat, w, g, st, G, t)
    w_r, st_r = ref_step(ref, w, g, st, G, t)
    extra = update_error_model(ref, st, g, G, t)
    check_step(ref, "random state G=%d" % G, w_g, st_g, w_r, st_r, st, g, G, extra_w_tol=extra)


@pytest.mark.parametrize("last_bit", [False, True])
def test_step_two_deep_cancellations_in_one_lane(coat, ref, last_bit):
    """Two elements of one lane whose beta1 m and (1 - beta1) g cancel to about 2^-22 of either term
    (same old code, same gradient, the group's scale tuned to the last bit): fp32 holds no correct
    digit of them.  One is the lane's candidate and is recomputed exactly; the other must come out
    right as well, not merely the one that is named.  last_bit: the scale NEAREST to exact
    cancellation, so that the residue is a fraction of the terms' last bit and the fp32 value often
    has the wrong sign, now and then with the right magnitude."""
    G, ng = 32, 8192
    n = G * ng
    st = S.random_state(n, G, seed=81)
    rng = np.random.default_rng(81)
    b1 = float(np.float32(HP["beta1"]))
    ratio = b1 / (1.0 - b1)
    g = S.grads_normal(n, 81, 1).copy()
    a_pos, b_pos = np.arange(ng) * G + 2, np.arange(ng) * G + 11      # both among the group's first 16 elements
    st["m_k"][:] = 1.0                                                # so that the old value is code * scale exactly
    mq = st["m_q"]
    mq[:] = (mq & 0x80) | np.minimum(mq & 0x7F, 0x70)
    mq[a_pos] = 0x7E
    mq[b_pos] = 0x7E                                                  # +448 * scale
    g0 = -(2.0 ** rng.integers(-12, -6, ng)) * rng.choice([1.0, 1.25, 1.5, 1.75], ng)   # bf16 values
    sc = (-g0 / (ratio * 448.0)).astype(np.float32)                   # the fp32 nearest to exact cancellation
    if not last_bit:                                                  # ... or a few ulp off
        for _ in range(64):
            d = np.abs(ratio * 448.0 * sc.astype(np.float64) + g0) / np.abs(g0)
            sc = np.where(d < 2.0 ** -23.5, np.nextafter(sc, np.float32(np.inf)), sc)
    depth = np.abs(ratio * 448.0 * sc.astype(np.float64) + g0) / np.abs(g0)
    if last_bit:
        assert np.mean(depth < 2.0 ** -24) > 0.5 and np.all(depth < 2.0 ** -22)
    else:
        assert np.mean((depth >= 2.0 ** -23.5) & (depth <= 2.0 ** -21)) > 0.9
    st["m_scale"][:] = sc
    gb = S.f32_to_bf16_bits(g0.astype(np.float32))
    g[a_pos] = gb
    g[b_pos] = gb
    w = S.weights(n, 81)
    t = 4
    w_g, st_g, _ = gpu_step(coat, w, g, st, G, t)
    w_r, st_r = ref_step(ref, w, g, st, G, t)
    # (the two elements' codes are far from the top and not zero in most groups)
    assert np.mean((st_r["m_q"][b_pos] & 0x7F) > 0) > 0.5
    check_step(ref, "two deep cancellations", w_g, st_g, w_r, st_r, st, g, G, extra_w_tol=update_error_model(ref, st, g, G, t))


def sparse_grads(n, G, seed, t, live=0.1):
    """Normal gradients in a tenth of the groups, exactly zero in the others (a different tenth every
    step): what an embedding table sees.  A group without gradient only decays: m_t = beta1 m."""
    rng = np.random.default_rng([seed, t])
    x = rng.standard_normal(n) * 1e-3
    x *= np.repeat(rng.random((n + G - 1) // G) < live, G)[:n]
    return S.f32_to_bf16_bits(x.astype(np.float32))


@pytest.mark.parametrize("G", [32, 128, 512])
@pytest.mark.parametrize("bf16_meta", [False, True])
def test_step_sparse_gradients(coat, ref, G, bf16_meta):
    n = 300 * 1024 + 3 * G + 11
    over = dict(bf16_scale=True, bf16_k=True) if bf16_meta else {}
    lockstep(coat, ref, n, G, lambda t: sparse_grads(n, G, 61, t), steps=8, seed=61, **over)


def test_step_decaying_gradients_bf16_k(coat, ref):
    """Gradients that shrink by a fifth per step: from about step 17 on their squares are below the
    second moment's smallest code and its groups are nearly idle: their exponents must stay where
    they are on both sides."""
    n, G = 100 * 1024 + 77, 128

    def grads(t):
        return S.f32_to_bf16_bits((np.random.default_rng([62, t]).standard_normal(n) * 1e-3 * 0.8 ** t).astype(np.float32))
    lockstep(coat, ref, n, G, grads, steps=24, seed=62, bf16_k=True)


@pytest.mark.parametrize("m_e5m2", [False, True])
def test_step_group_maximum_among_near_ties(coat, ref, m_e5m2):
    """Groups whose old codes are all small, so that the new maximum is far below beta1 * fmax * scale
    (the case in which the kernel takes the maximum from exact values), and whose two largest
    elements have the same old code, sit in ONE lane and differ by their tiny gradients only, a few
    1e-7 to 1e-6 of their size: whichever of the two fp32 ranks first, the scale must hold 1e-6."""
    G, ng = 32, 8192
    n = G * ng
    st = S.random_state(n, G, seed=31)
    rng = np.random.default_rng(31)
    mq = st["m_q"]
    mq[:] = (mq & 0x80) | np.minimum(mq & 0x7F, 0x50)
    a_pos, b_pos = np.arange(ng) * G + 3, np.arange(ng) * G + 9       # both among the group's first 16 elements
    mq[a_pos] = (mq[a_pos] & 0x80) | 0x58
    mq[b_pos] = (mq[b_pos] & 0x80) | 0x58
    m_old = ref.dequant_group(mq, st["m_scale"], st["m_k"], G, f64=True, e5m2=m_e5m2)
    b1 = float(np.float32(HP["beta1"]))
    gf = np.zeros(n)
    for pos in (a_pos, b_pos):                      # same sign as the old moment: the magnitudes add
        gf[pos] = 3e-6 * rng.random(ng) * (b1 / (1 - b1)) * m_old[pos]
    g = S.f32_to_bf16_bits(gf.astype(np.float32))
    w = S.weights(n, 31)
    t = 5
    over = dict(m_e5m2=True) if m_e5m2 else {}
    w_g, st_g, _ = gpu_step(coat, w, g, st, G, t, **over)
    w_r, st_r = ref_step(ref, w, g, st, G, t, **over)
    # the case is exercised: in many groups the two are closer than 1e-6 and the new maximum is small
    m_t = b1 * m_old + (1 - b1) * S.bf16_bits_to_f32(g).astype(np.float64)
    gap = np.abs(np.abs(m_t[a_pos]) / np.abs(m_t[b_pos]) - 1.0)
    fmax = 57344.0 if m_e5m2 else 448.0
    fell = np.maximum(np.abs(m_t[a_pos]), np.abs(m_t[b_pos])) < 0.3 * b1 * fmax * st["m_scale"].astype(np.float64)
    assert int((fell & (gap > 2e-7) & (gap < 2e-6)).sum()) > ng // 8
    check_step(ref, "near ties at the maximum", w_g, st_g, w_r, st_r, st, g, G,
               extra_w_tol=update_error_model(ref, st, g, G, t, **over), **over)


@pytest.mark.parametrize("G", [32, 128, 512])
def test_step_bf16_scale(coat, ref, G):
    """Scales stored in BF16 (Sec. 3): lock-step against the oracle's same option."""
    n = 200 * 1024 + 3 * G + 7
    lockstep(coat, ref, n, G, lambda t: S.grads_normal(n, 21, t, G=G, outlier_frac=0.01), steps=4, seed=21, bf16_scale=True)
    lockstep(coat, ref, n, G, lambda t: S.grads_lognormal(n, 22, t), steps=3, seed=22, bf16_scale=True)


def test_step_bf16_scale_with_other_cells(coat, ref):
    n = 64 * 1024 + 50
    lockstep(coat, ref, n, 128, lambda t: S.grads_normal(n, 23, t), steps=3, seed=23, bf16_scale=True, expand=False)
    lockstep(coat, ref, n, 128, lambda t: S.grads_normal(n, 24, t), steps=3, seed=24, bf16_scale=True,
             m_e5m2=True, v_plain=True)


@pytest.mark.parametrize("G", [32, 128, 512])
@pytest.mark.parametrize("kind", ["normal", "square", "lognormal", "zeros_mixed"])
def test_quant_bf16_scale(coat, ref, G, kind):
    """Standalone quantizer with BF16 scales: identical inputs, so the stored scales must be EQUAL;
    then dequantize through the GPU and compare with the oracle's dequantizer."""
    n = 37 * 1024 + 2 * G + 17
    x = quant_inputs(kind, n, seed=G + len(kind))
    q, s, k = coat.coat_quant_group(dev(x), G, bf16_scale=True)
    assert s.dtype == torch.bfloat16
    q_g, s_g, k_g = q.cpu().numpy(), s.float().cpu().numpy(), k.cpu().numpy()
    q_r, s_r, k_r = ref.quant_group(x, G, bf16_scale=True)
    assert np.array_equal(s_g, s_r)
    check_quant(ref, "quant bf16 scale %s G=%d" % (kind, G), x, G, (q_g, s_g, k_g), (q_r, s_r, k_r), True)
    xh_g = coat.coat_dequant_group(q, s, k, G).cpu().numpy().astype(np.float64)
    xh_r = ref.dequant_group(q_g, s_g, k_g, G, f64=True)
    ok = np.isfinite(xh_r) & (xh_r != 0)
    assert np.all(np.abs(xh_g[ok] / xh_r[ok] - 1.0) <= 8 * 2.0 ** -24)
    assert np.all(xh_g[xh_r == 0] == 0)


@pytest.mark.parametrize("G", [32, 128, 512])
@pytest.mark.parametrize("bf16_scale", [False, True])
def test_step_bf16_k(coat, ref, G, bf16_scale):
    """Exponents stored in BF16 (with fp32 and with BF16 scales: 8 + 12/G and 8 + 8/G bytes per parameter)."""
    n = 96 * 1024 + 3 * G + 5
    tot = lockstep(coat, ref, n, G, lambda t: S.grads_normal(n, 12, t, G=G, outlier_frac=0.02), steps=4, seed=12,
                   bf16_k=True, bf16_scale=bf16_scale)
    tot2 = lockstep(coat, ref, n, G, lambda t: S.grads_lognormal(n, 13, t), steps=3, seed=13, bf16_k=True, bf16_scale=bf16_scale)
    print("bf16 k G=%d bf16_scale=%s:" % (G, bf16_scale), tot, tot2)


@pytest.mark.parametrize("G", [32, 128, 512])
def test_idle_groups_keep_their_bf16_exponent(coat, G):
    """Free-running on the GPU: one step with gradients, then twenty with none.  A group that only
    decays reproduces the range its stored k made, so its new exponent is the stored bf16 value to a
    few 1e-7 and the rounding to the nearest bf16 must keep it there (the oracle's same property is
    pinned on the CPU)."""
    n = 2048 * G
    hp = dict(HP, bf16_k=True)
    tw = dev(S.weights(n, 71))
    z = S.zero_state(n, G)
    ts = {k: dev(v) for k, v in z.items()}
    for k in ("m_k", "v_k"):
        ts[k] = ts[k].to(torch.bfloat16)
    args = lambda: (ts["m_q"], ts["m_scale"], ts["m_k"], ts["v_q"], ts["v_scale"], ts["v_k"])
    coat.coat_fp8_adamw_step(tw, dev_bf16(S.grads_normal(n, 71, 1)), *args(), coat.make_hparams(step=1, group_size=G, **hp))
    first = {k: v.clone() for k, v in ts.items()}
    idle = dev_bf16(np.zeros(n, np.uint16))
    for t in range(2, 22):
        coat.coat_fp8_adamw_step(tw, idle, *args(), coat.make_hparams(step=t, group_size=G, **hp))
    torch.cuda.synchronize()
    for name in ("m", "v"):
        mag = (first[name + "_q"] & 0x7F).view(-1, G)
        ends = (mag.max(1).values == 0x7E) & (torch.where(mag > 0, mag, 0x7F).min(1).values == 1)
        assert float(ends.float().mean()) > 0.9
        assert torch.equal(ts[name + "_k"][ends], first[name + "_k"][ends]), "%s: %d of %d idle groups moved their exponent" % (
            name, int((ts[name + "_k"][ends] != first[name + "_k"][ends]).sum()), int(ends.sum()))
        same = (ts[name + "_q"].view(-1, G)[ends] == first[name + "_q"].view(-1, G)[ends]).float().mean()
        assert float(same) > 0.9999, "%s: idle codes moved (%.6f equal)" % (name, float(same))


@pytest.mark.parametrize("G", [32, 128, 512])
@pytest.mark.parametrize("kind", ["normal", "square", "lognormal", "zeros_mixed"])
def test_quant_bf16_k(coat, ref, G, kind):
    """Standalone quantizer with BF16 exponents: identical inputs, so the scales are equal to 1e-6 and
    the stored exponents are EQUAL except where the exponent sits within the plain bar of a bf16
    boundary; then the dequantizer reads the bf16 exponents back."""
    n = 37 * 1024 + 2 * G + 17
    x = quant_inputs(kind, n, seed=G + len(kind))
    q, s, k = coat.coat_quant_group(dev(x), G, bf16_k=True)
    assert k.dtype == torch.bfloat16 and s.dtype == torch.float32
    q_g, s_g, k_g = q.cpu().numpy(), s.cpu().numpy(), k.float().cpu().numpy()
    q_r, s_r, k_r = ref.quant_group(x, G, bf16_k=True)
    _, _, k_exact = ref.quant_group(x, G)
    assert_scale(s_g, s_r, "quant bf16 k")
    differ, stats = check_bf16_k("quant bf16 k %s G=%d" % (kind, G), k_g, k_r, k_exact, k_bar(x, G), np.zeros(k_r.size), None)
    assert stats["k_out"] == 0
    assert_codes(ref, q_g, q_r, G, "quant bf16 k codes", other_scale=differ)
    xh_g = coat.coat_dequant_group(q, s, k, G).cpu().numpy().astype(np.float64)
    xh_r = ref.dequant_group(q_g, s_g, k_g, G, f64=True)
    ok = np.isfinite(xh_r) & (xh_r != 0)
    assert np.all(np.abs(xh_g[ok] / xh_r[ok] - 1.0) <= 8 * 2.0 ** -24)
    assert np.all(xh_g[xh_r == 0] == 0)


@pytest.mark.parametrize("G", [32, 128, 512])
def test_step_precise_dq(coat, ref, G):
    """The more accurate inverse expansion on request: same bar; under hyper-parameters that make the
    update a large fraction of the weight it is what keeps the weights inside it (whole-set test)."""
    n = 96 * 1024 + 3 * G + 5
    lockstep(coat, ref, n, G, lambda t: S.grads_lognormal(n, 14, t), steps=4, seed=14, precise_dq=True,
             lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01)
    lockstep(coat, ref, n, G, lambda t: S.grads_normal(n, 15, t, G=G, outlier_frac=0.02), steps=3, seed=15, precise_dq=True)


def test_step_expansion_off(coat, ref):
    n = 64 * 1024 + 50
    lockstep(coat, ref, n, 128, lambda t: S.grads_normal(n, 5, t), steps=3, seed=5, expand=False)


def test_step_other_hyperparameters(coat, ref):
    n = 64 * 1024
    lockstep(coat, ref, n, 128, lambda t: S.grads_normal(n, 6, t), steps=3, seed=6,
             lr=1e-3, beta1=0.8, beta2=0.999, eps=1e-6, weight_decay=0.0)
    lockstep(coat, ref, n, 64, lambda t: S.grads_normal(n, 7, t), steps=2, seed=7, k_min=1.0, k_max=8.0)


@pytest.mark.parametrize("n", [1, 31, 128, 1000, 1024, 1025, 2048 + 127])
def test_step_tiny_sizes(coat, ref, n):
    lockstep(coat, ref, n, 128, lambda t: S.grads_normal(n, 8, t), steps=2, seed=8)


def test_step_zero_gradients_and_zero_groups(coat, ref):
    n, G = 8 * 1024, 128
    def grads(t):
        g = S.grads_normal(n, 9, t)
        g[: 3 * G] = 0                               # groups that never receive a gradient
        g[5 * G: 6 * G: 2] = 0                       # zeros mixed into a live group
        g[7 * G] = 0x8000                            # a negative zero
        return g
    lockstep(coat, ref, n, G, grads, steps=3, seed=9)


def test_step_does_not_touch_gradients_or_neighbours(coat, ref):
    n, G, pad = 5 * 1024 + 200, 128, 512
    ng = (n + G - 1) // G
    w = S.weights(n, 10)
    g = S.grads_normal(n, 10, 1)
    st = S.random_state(n, G, seed=10)
    wbuf = torch.full((n + 2 * pad,), 3.0, dtype=torch.float32, device="cuda")
    wbuf[pad:pad + n] = dev(w)
    bufs = {}
    for name, arr in st.items():
        fill = 0xAB if arr.dtype == np.uint8 else -7.0
        b = torch.full((arr.size + 2 * pad,), fill, dtype=torch.from_numpy(arr).dtype, device="cuda")
        b[pad:pad + arr.size] = dev(arr)
        bufs[name] = b
    tg = dev_bf16(g)
    hp = coat.make_hparams(step=3, group_size=G, **HP)
    view = lambda name: bufs[name][pad:pad + st[name].size]
    coat.coat_fp8_adamw_step(wbuf[pad:pad + n], tg, view("m_q"), view("m_scale"), view("m_k"),
                             view("v_q"), view("v_scale"), view("v_k"), hp)
    torch.cuda.synchronize()
    assert torch.all(wbuf[:pad] == 3.0) and torch.all(wbuf[pad + n:] == 3.0)
    for name, arr in st.items():
        fill = 0xAB if arr.dtype == np.uint8 else -7.0
        assert torch.all(bufs[name][:pad] == fill) and torch.all(bufs[name][pad + arr.size:] == fill), name
    assert np.array_equal(tg.view(torch.int16).cpu().numpy().view(np.uint16), g)
    w_r, st_r = ref_step(ref, w, g, st, G, 3)
    check_step(ref, "padded", wbuf[pad:pad + n].cpu().numpy(), {k: view(k).cpu().numpy() for k in st}, w_r, st_r,
               st, g, G, extra_w_tol=update_error_model(ref, st, g, G, 3))


def test_step_is_deterministic_and_reloadable(coat):
    n, G = 64 * 1024, 128
    w = S.weights(n, 11)
    grads = [S.grads_normal(n, 11, t) for t in (1, 2, 3)]

    def run(split):
        tw = dev(w)
        ts = {k: dev(v) for k, v in S.zero_state(n, G).items()}
        for t, g in enumerate(grads, start=1):
            if split and t == 3:                       # save -> load -> continue
                tw = dev(tw.cpu().numpy())
                ts = {k: dev(v.cpu().numpy()) for k, v in ts.items()}
            hp = coat.make_hparams(step=t, group_size=G, **HP)
            coat.coat_fp8_adamw_step(tw, dev_bf16(g), ts["m_q"], ts["m_scale"], ts["m_k"],
                                     ts["v_q"], ts["v_scale"], ts["v_k"], hp)
        torch.cuda.synchronize()
        return tw.cpu().numpy(), {k: v.cpu().numpy() for k, v in ts.items()}

    w_a, s_a = run(False)
    w_b, s_b = run(True)
    assert np.array_equal(w_a, w_b)
    for k in s_a:
        assert np.array_equal(s_a[k], s_b[k]), k


def test_non_finite_gradient_stays_in_its_group(coat, ref):
    n, G = 4 * 1024, 128
    w = S.weights(n, 12)
    st = S.random_state(n, G, seed=12)
    g = S.grads_normal(n, 12, 1)
    g_bad = g.copy()
    g_bad[5 * G + 3] = 0x7FC0                          # NaN
    g_bad[9 * G + 100] = 0x7F80                        # +Inf
    w_a, st_a, _ = gpu_step(coat, w, g, st, G, 2)
    w_b, st_b, _ = gpu_step(coat, w, g_bad, st, G, 2)
    keep = np.ones(n, bool)
    keep[5 * G:6 * G] = False
    keep[9 * G:10 * G] = False
    assert np.array_equal(w_a[keep], w_b[keep])
    assert np.array_equal(st_a["m_q"][keep], st_b["m_q"][keep]) and np.array_equal(st_a["v_q"][keep], st_b["v_q"][keep])
    gk = np.ones(n // G, bool)
    gk[[5, 9]] = False
    for name in ("m_scale", "m_k", "v_scale", "v_k"):
        assert np.array_equal(st_a[name][gk], st_b[name][gk]), name
    assert not np.isfinite(w_b[5 * G + 3])
    # inside a poisoned group the other weights are still the clean result
    rest = np.arange(5 * G, 6 * G) != 5 * G + 3
    assert np.array_equal(w_a[5 * G:6 * G][rest], w_b[5 * G:6 * G][rest])


def test_quant_nearly_constant_groups(coat, ref):
    # groups whose range is a few ulp: k sits on its upper clamp on both sides
    n, G = 4 * 1024, 128
    rng = np.random.default_rng(21)
    base = np.float32(3.0e-4)
    x = np.full(n, base, np.float32)
    ulps = rng.integers(0, 3, n).astype(np.int32)
    x = (x.view(np.int32) + ulps).view(np.float32) * rng.choice([-1.0, 1.0], n).astype(np.float32)
    x[:G] = base                                     # one exactly constant group: k = 1
    q_g, s_g, k_g = (t.cpu().numpy() for t in coat.coat_quant_group(dev(x), G))
    q_r, s_r, k_r = ref.quant_group(x, G)
    assert k_r[0] == 1.0 and k_g[0] == 1.0
    assert np.all(k_r[1:] == 1024.0) and np.all(k_g[1:] == 1024.0)
    assert_scale(s_g, s_r, "tight groups")
    # with k = 1024 a 1-ulp difference of x moves the value by 1.2e-4: codes stay within a step
    n_bad = int(np.sum(q_g != q_r))
    assert np.all(np.abs((q_g & 0x7F).astype(int) - (q_r & 0x7F).astype(int)) <= 1)
    assert n_bad <= n // 100


# --- the format / expansion grid of Table 1 ----------------------------------------------------------

import itertools

GRID = [c for c in itertools.product([False, True], repeat=4) if any(c)]   # all but the default cell


@pytest.mark.parametrize("G", [32, 128, 512])
@pytest.mark.parametrize("expand", [True, False])
def test_quant_dequant_e5m2(coat, ref, G, expand):
    n = 21 * 1024 + 3 * G + 9
    x = quant_inputs("normal", n, seed=G)
    q_g, s_g, k_g = (t.cpu().numpy() for t in coat.coat_quant_group(dev(x), G, expand=expand, e5m2=True))
    q_r, s_r, k_r = ref.quant_group(x, G, expand=expand, e5m2=True)
    check_quant(ref, "e5m2 quant G=%d expand=%s" % (G, expand), x, G, (q_g, s_g, k_g), (q_r, s_r, k_r), expand, e5m2=True)
    assert np.all((q_g & 0x7F) <= 0x7B)                 # never infinity or NaN
    # dequantizer on every code byte of the format
    codes = (np.arange(n) % 256).astype(np.uint8)
    ng = (n + G - 1) // G
    rng = np.random.default_rng(G)
    scale = np.exp(rng.uniform(np.log(1e-14), np.log(1e-4), ng)).astype(np.float32)
    k = np.exp(rng.uniform(np.log(0.5), np.log(40.0), ng)).astype(np.float32)
    x_g = coat.coat_dequant_group(dev(codes), dev(scale), dev(k), G, e5m2=True).cpu().numpy().astype(np.float64)
    x_r = ref.dequant_group(codes, scale, k, G, f64=True, e5m2=True)
    fin = np.isfinite(x_r)
    # infinity / NaN codes (never written by the quantizer) come back non-finite
    assert not np.any(np.isfinite(x_g[~fin]))
    nz = fin & (x_r != 0)
    assert np.all(np.abs(x_g[nz] / x_r[nz] - 1.0) <= 8 * 2.0 ** -24)
    assert np.all(x_g[fin & (x_r == 0)] == 0)


@pytest.mark.parametrize("m_e5m2,m_plain,v_e5m2,v_plain", GRID)
def test_step_format_grid(coat, ref, m_e5m2, m_plain, v_e5m2, v_plain):
    n, G = 96 * 1024 + 2 * 128 + 5, 128
    lockstep(coat, ref, n, G, lambda t: S.grads_normal(n, 13, t, G=G, outlier_frac=0.01), steps=3, seed=13,
             update_model=v_plain, m_e5m2=m_e5m2, m_plain=m_plain, v_e5m2=v_e5m2, v_plain=v_plain)


@pytest.mark.parametrize("G", [32, 64, 256, 512])
def test_step_format_grid_other_group_sizes(coat, ref, G):
    n = 64 * 1024 + G + 1
    lockstep(coat, ref, n, G, lambda t: S.grads_lognormal(n, 14, t), steps=2, seed=14, m_e5m2=True, v_plain=True,
             update_model=True)
    lockstep(coat, ref, n, G, lambda t: S.grads_normal(n, 15, t), steps=2, seed=15, m_plain=True, v_e5m2=True)


# --- the step that also emits the bf16 model weights ------------------------------------------------

@pytest.mark.parametrize("n,G,generic", [(40 * 1024 + 3 * 128 + 7, 128, False), (9 * 1024 + 65, 64, True), (700, 128, False)])
def test_step_with_bf16_weight_copy(coat, ref, n, G, generic):
    w = S.weights(n, 16)
    st = S.random_state(n, G, seed=16) if not generic else S.zero_state(n, G)
    g = S.grads_normal(n, 16, 1, G=G, outlier_frac=0.02)
    kw = dict(m_e5m2=True) if generic else {}
    hp = coat.make_hparams(step=4, group_size=G, **HP, **kw)
    pad = 64
    # plain entry
    tw, tg = dev(w), dev_bf16(g)
    ts = {k: dev(v) for k, v in st.items()}
    coat.coat_fp8_adamw_step(tw, tg, ts["m_q"], ts["m_scale"], ts["m_k"], ts["v_q"], ts["v_scale"], ts["v_k"], hp)
    # emitting entry, canaries around the bf16 buffer
    tw2 = dev(w)
    ts2 = {k: dev(v) for k, v in st.items()}
    wb = torch.full((n + 2 * pad,), 7.0, dtype=torch.bfloat16, device="cuda")
    coat.coat_fp8_adamw_step_bf16w(tw2, wb[pad:pad + n], tg, ts2["m_q"], ts2["m_scale"], ts2["m_k"],
                                   ts2["v_q"], ts2["v_scale"], ts2["v_k"], hp)
    torch.cuda.synchronize()
    assert torch.equal(tw, tw2)                                        # nothing else changes
    for k in ts:
        assert torch.equal(ts[k], ts2[k]), k
    assert torch.all(wb[:pad] == 7.0) and torch.all(wb[pad + n:] == 7.0)
    got = wb[pad:pad + n]
    assert torch.equal(got.view(torch.int16), tw2.to(torch.bfloat16).view(torch.int16))   # RNE of its own fp32 weights
    # against the oracle's copy: equal except where the two fp32 weights straddle a bf16 rounding tie
    w_r = w.copy()
    st_r = {k: v.copy() for k, v in st.items()}
    wb_r = np.zeros(n, np.uint16)
    rh = ref.make_hparams(step=4, group_size=G, **HP, **kw)
    assert ref.fp8_adamw_step(w_r, g, st_r["m_q"], st_r["m_scale"], st_r["m_k"], st_r["v_q"], st_r["v_scale"],
                              st_r["v_k"], rh, w_bf16=wb_r) == 0
    got_bits = got.view(torch.int16).cpu().numpy().view(np.uint16).astype(np.int32)
    diff = np.abs(got_bits - wb_r.astype(np.int32))
    assert diff.max() <= 1 and np.mean(diff != 0) <= 2e-3


def test_bf16_entry_rejects_misaligned_copy(coat):
    import ctypes
    L = coat.lib()
    ok = ctypes.c_void_p(0x1000)
    hp = coat.make_hparams()
    args = [ok, ctypes.c_void_p(0x1002)] + [ok] * 7
    assert L.coat_fp8_adamw_step_bf16w(*args, 4096, ctypes.byref(hp), None) == -2


# --- the experiment of Table 1 on the GPU path --------------------------------------------------

def test_table1_structure_on_the_gpu_path(coat, ref):
    """The sixteen cells of Table 1 computed through the HIP quantizer / dequantizer on synthetic
    moments: each cell must agree with the same cell computed by the oracle, and the structure
    the paper reports must hold (expansion helps either moment in either format; the best cells are
    those with E4M3+Expand for the first moment and an expanded second moment, whose two formats
    differ by about a percent in the paper as well).  The paper's absolute values need its real
    optimizer states: unpinned."""
    from table1_experiment import CELLS, table1
    n, G, seed = 1 << 18, 128, 4
    labels, rows = table1(n, G, seed)
    gen = S.torch_generator(torch.device("cuda:0"), seed)
    m, v = (t.cpu().numpy() for t in S.torch_moments(n, torch.device("cuda:0"), gen, G=G))
    exact = m.astype(np.float64) / (np.sqrt(v.astype(np.float64)) + 1e-8)

    def through(x, e5, ex):
        return ref.dequant_group(*ref.quant_group(x, G, expand=ex, e5m2=e5), G, f64=True, e5m2=e5)

    mh = [through(m, e5, ex) for _, e5, ex in CELLS]
    vh = [through(v, e5, ex) for _, e5, ex in CELLS]
    for i in range(4):
        for j in range(4):
            want = float(np.mean((mh[i] / (np.sqrt(vh[j]) + 1e-8) - exact) ** 2))
            assert abs(rows[i][j] - want) <= 2e-3 * want, (labels[i], labels[j], rows[i][j], want)
    r = np.asarray(rows)
    plain = {0: 1, 2: 3}                                  # index of a plain cell -> its +Expand twin
    for p, e in plain.items():
        assert np.all(r[e, :] < r[p, :]) and np.all(r[:, e] < r[:, p])
    assert min(r[1, 1], r[1, 3]) == r.min() and r[1, 1] <= 1.1 * r.min()
    assert r[0, 0] > 1.3 * r[1, 1]                        # the direction of the paper's 1.63x
    # and the order the paper's own sixteen values establish (tests/golden/table1_mse.txt)
    from test_oracle_formats import concordance, paper_table1
    pairs, wrong = concordance(paper_table1(), r)
    assert len(pairs) == 110 and not wrong, wrong


# --- seeded sweep over sizes, group sizes and storage modes ------------------------------------

def test_step_seeded_sweep_of_configurations(coat, ref):
    """Forty seeded combinations of size (around chunk and group boundaries), group size, storage
    mode of each moment, BF16 scales and hyper-parameters, two lock-step steps each."""
    rng = np.random.default_rng(2024)
    edges = [1, 2, 15, 16, 17, 31, 33, 127, 128, 129, 511, 513, 1023, 1024, 1025, 2047, 2049, 3 * 1024 + 1]
    for case in range(40):
        G = int(rng.choice(GROUPS))
        n = int(rng.choice(edges)) if case % 2 else int(rng.integers(1, 40 * 1024))
        over = dict(m_e5m2=bool(rng.integers(2)), v_e5m2=bool(rng.integers(2)), m_plain=bool(rng.integers(2)),
                    v_plain=bool(rng.integers(2)), bf16_scale=bool(rng.integers(2)))
        if case % 5 == 0:
            over = {}                                                   # the default kernel gets its share
        if case % 7 == 0:
            over.update(lr=1e-3, beta1=0.8, beta2=0.99, weight_decay=0.0)
        kind = case % 3
        seed = 1000 + case

        def grads(t, n=n, G=G, kind=kind, seed=seed):
            if kind == 0:
                return S.grads_normal(n, seed, t, G=G, outlier_frac=0.05)
            if kind == 1:
                return S.grads_lognormal(n, seed, t)
            return S.grads_normal(n, seed, t, sigma=3e-5)

        try:
            lockstep(coat, ref, n, G, grads, steps=2, seed=seed, update_model=bool(over.get("v_plain")), **over)
        except AssertionError as e:
            raise AssertionError("case %d: n=%d G=%d %r: %s" % (case, n, G, over, e))


def test_zz_print_totals():
    """Not a check: prints what the lock-step runs of this module measured (run with -s)."""
    for key in sorted(TOTALS):
        t = TOTALS[key]
        print("%-12s mismatch rate %.2e (%d of %d), more than one step %d, k outside the bar %d of %d groups, w err/tol %.3f" % (
            key, t["bad"] / max(1, t["elems"]), t["bad"], t["elems"], t["far"], t["k_out"], t["groups"], t["w"]))
