"""Pins for the oracle's per-group quantizer with dynamic range expansion (no GPU).

Each test checks the oracle against something the paper or the mathematics fixes:
  * expansion off (k = 1) is the plain quantizer of Sec. 3: S = max|X|/448, X_fp8 = round(X/S),
    checked with a library cast and a brute-force nearest search;
  * the range identity of Sec. 4.2, R_f(X) = R_X^k = 448*512, i.e. the group's largest
    element lands on 448 and its smallest non-zero element on 2^-9;
  * the optimal exponent k = log_{R_X}(R_E4M3) as a closed form, with spot values inside
    the bands the paper reports;
  * the axioms of Appendix E: f is odd, monotone, f(0) = 0 and scale invariant;
  * f^-1 o f = id up to the E4M3 rounding bound.
"""
import math

import numpy as np
import pytest
import torch

from test_oracle_codec import golden

LOG2_R = math.log2(448 * 512)


def decode_table():
    return torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).to(torch.float64).numpy()


def nearest_codes(vals):
    """Brute force: index of the nearest non-negative E4M3 value, ties to the even code."""
    table = decode_table()[:0x7F]
    a = np.minimum(np.abs(vals), 448.0)
    d = np.abs(a[:, None] - table[None, :])
    best = d.min(axis=1, keepdims=True)
    cand = d == best
    lo = np.argmax(cand, 1)                       # first of the (at most two) nearest codes
    idx = np.where((cand.sum(1) > 1) & (lo % 2 == 1), lo + 1, lo)
    return (idx | np.where(np.signbit(vals), 0x80, 0)).astype(np.uint8)


def groups(seed, ng=64, G=128, sigma=1e-3):
    return (np.random.default_rng(seed).standard_normal(ng * G) * sigma).astype(np.float32)


# --- k = 1: the plain per-group quantizer ------------------------------------------------

@pytest.mark.parametrize("G", [1, 2, 16, 128, 512])
def test_expansion_off_is_plain_per_group_quantizer(ref, G):
    x = groups(10, ng=32, G=G)
    q, s, k = ref.quant_group(x, G, expand=False)
    xg = x.reshape(-1, G).astype(np.float64)
    amax = np.abs(xg).max(1)
    assert np.array_equal(s, (amax / 448.0).astype(np.float32))       # S_X = max|X| / 448
    assert np.all(k == 1.0)
    scaled = (xg / s.astype(np.float64)[:, None]).reshape(-1)          # X / S_X ...
    scaled = scaled.astype(np.float32).astype(np.float64)              # ... as an fp32 number (Appendix A)
    assert np.array_equal(q, nearest_codes(scaled))
    # library cast of the same quotient (fp32 quotient; skip the rare double-rounding ties)
    lib = torch.from_numpy(scaled.astype(np.float32)).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.mean(lib == q) > 0.999
    # DQ = S * X_fp8
    xh = ref.dequant_group(q, s, k, G)
    expect = (decode_table()[q].reshape(-1, G) * s.astype(np.float64)[:, None]).reshape(-1)
    assert np.allclose(xh, expect.astype(np.float32), rtol=1e-7, atol=0)
    # the largest element of every group takes the largest code
    top = np.abs(xg).argmax(1)
    assert np.all((q.reshape(-1, G)[np.arange(len(top)), top] & 0x7F) == 0x7E)


# --- the expansion exponent ----------------------------------------------------------------

def test_k_closed_form_and_paper_bands(ref):
    g = golden()
    for R, lo, hi in [(10.0, g["k_v_band_lo"], g["k_v_band_hi"]),       # v: range < 1e1 -> k in 5..15
                      (1e4, g["k_m_band_lo"], g["k_m_band_hi"]),        # m: range < 1e4 -> k in 1..3
                      (229376.0, 1.0, 1.0), (2.0, LOG2_R, LOG2_R), (1e9, 0.0, 1.0)]:
        x = np.array([1e-5, 1e-5 * R], dtype=np.float32)
        _, _, k = ref.quant_group(x, 2)
        Rf = float(x[1]) / float(x[0])
        assert k[0] == np.float32(LOG2_R / math.log2(Rf))
        assert lo * (1 - 1e-6) <= k[0] <= hi * (1 + 1e-6) or (lo, hi) == (0.0, 1.0) and 0 < k[0] < 1
    # R_X = R_E4M3 exactly -> k = 1 exactly
    x = np.array([2.0 ** -9, 448.0], dtype=np.float32)
    assert ref.quant_group(x, 2)[2][0] == 1.0


def test_k_clamp_and_degenerate_groups(ref):
    # a single distinct magnitude: R_X = 1, any k gives the same codes; the oracle says k = 1
    q, s, k = ref.quant_group(np.array([3e-4, -3e-4, 3e-4, 0.0], np.float32), 4)
    assert k[0] == 1.0 and list(q) == [0x7E, 0xFE, 0x7E, 0x00]
    # all zeros: scale 0, k 1, zero codes (sign of zero kept)
    q, s, k = ref.quant_group(np.array([0.0, -0.0, 0.0, 0.0], np.float32), 4)
    assert s[0] == 0.0 and k[0] == 1.0 and list(q) == [0, 0x80, 0, 0]
    # very tight group: k would be ~1.2e6, clamped to the default upper bound 2^10
    x = np.array([1.0, 1.0 + 2.0 ** -16], np.float32)
    assert ref.quant_group(x, 2)[2][0] == 1024.0
    assert ref.quant_group(x, 2, k_min=1.0, k_max=8.0)[2][0] == 8.0
    # k below 1 (range wider than E4M3's) is allowed by default and can be clamped away
    x = np.array([1e-12, 1.0], np.float32)
    assert 0.4 < ref.quant_group(x, 2)[2][0] < 0.5
    assert ref.quant_group(x, 2, k_min=1.0, k_max=1024.0)[2][0] == 1.0


# --- R_f(X) = R_X^k = R_E4M3 ---------------------------------------------------------------

@pytest.mark.parametrize("G", [2, 32, 128, 512])
@pytest.mark.parametrize("kind", ["normal", "square", "lognormal"])
def test_expanded_group_fills_the_e4m3_range(ref, G, kind):
    x = groups(20 + G, ng=48, G=G)
    if kind == "square":
        x = (x * x).astype(np.float32)                  # like second moments: non-negative
    elif kind == "lognormal":
        z = np.random.default_rng(5).standard_normal(x.size)
        x = (1e-3 * np.exp(2 * z) * np.sign(x)).astype(np.float32)
    q, s, k = ref.quant_group(x, G)
    table = decode_table()
    mag = np.abs(table[q]).reshape(-1, G)
    ax = np.abs(x.astype(np.float64)).reshape(-1, G)
    rows = np.arange(ax.shape[0])
    assert np.all(mag[rows, ax.argmax(1)] == 448.0)     # max |x|  -> Delta_max
    free = (k > 0.0625) & (k < 1024.0)                  # groups whose k was not clamped
    assert free.sum() >= 0.9 * free.size
    assert np.all(mag[rows, ax.argmin(1)][free] == 2.0 ** -9)  # min |x|  -> Delta_min
    R = ax.max(1) / ax.min(1)
    assert np.allclose((R ** k.astype(np.float64))[free], 229376.0, rtol=2e-5)   # (R_X)^k = R_E4M3
    assert np.allclose(s, ax.max(1) / 448.0, rtol=1e-7)
    if kind == "square":
        assert np.all(q < 0x80)                         # v >= 0 keeps the sign bit clear


# --- axioms of the expand function (Appendix E) ----------------------------------------------

def test_oddness_sign_symmetry(ref):
    x = groups(30)
    q, s, k = ref.quant_group(x, 128)
    qn, sn, kn = ref.quant_group(-x, 128)
    assert np.array_equal(qn, q ^ 0x80) and np.array_equal(sn, s) and np.array_equal(kn, k)
    xh, xhn = ref.dequant_group(q, s, k, 128), ref.dequant_group(qn, sn, kn, 128)
    assert np.array_equal(xh, -xhn)


@pytest.mark.parametrize("p", [-20, -3, 1, 7])
def test_scale_invariance(ref, p):
    x = groups(31)
    q, s, k = ref.quant_group(x, 128)
    q2, s2, k2 = ref.quant_group(np.ldexp(x, p), 128)
    assert np.array_equal(q2, q) and np.array_equal(k2, k)
    assert np.array_equal(s2, np.ldexp(s, p))


def test_monotone_order_preserved(ref):
    x = groups(32, ng=16)
    q, s, k = ref.quant_group(x, 128)
    val = decode_table()[q].reshape(-1, 128)
    xg = x.reshape(-1, 128)
    for r in range(xg.shape[0]):
        order = np.argsort(xg[r], kind="stable")
        assert np.all(np.diff(val[r][order]) >= 0)


def test_zero_maps_to_zero(ref):
    x = groups(33, ng=8)
    x[::7] = 0.0
    x[3::11] = -0.0
    q, s, k = ref.quant_group(x, 128)
    assert np.all((q[x == 0] & 0x7F) == 0)
    assert np.all((q[x != 0] & 0x7F) != 0)              # with unclamped k nothing non-zero flushes
    xh = ref.dequant_group(q, s, k, 128)
    assert np.all(xh[x == 0] == 0)
    # the minimum is taken over the non-zero elements
    ax = np.abs(x.astype(np.float64)).reshape(-1, 128)
    amin = np.where(ax > 0, ax, np.inf).min(1)
    assert np.allclose(k, LOG2_R / np.log2(ax.max(1) / amin), rtol=1e-6)


# --- inverse expansion ----------------------------------------------------------------------

@pytest.mark.parametrize("kind", ["normal", "square"])
def test_roundtrip_error_bound(ref, kind):
    x = groups(40, ng=64)
    if kind == "square":
        x = (x * x).astype(np.float32)
    q, s, k = ref.quant_group(x, 128)
    xh = ref.dequant_group(q, s, k, 128, f64=True)
    rel = np.abs(xh / x.astype(np.float64) - 1.0).reshape(-1, 128)
    # a normal code c is within 2^-4 relative of the expanded value y: c/y in [1-2^-4, 1+2^-4];
    # through the inverse expansion the recovered ratio is (c/y)^(1/k), whose larger deviation
    # is 1 - (1-2^-4)^(1/k).  Subnormal y (< 2^-6, codes 0..8) has absolute spacing instead.
    normal = ((q & 0x7F) > 8).reshape(-1, 128)
    bound = (1.0 - (1 - 2.0 ** -4) ** (1.0 / k.astype(np.float64)))[:, None] * (1 + 1e-6) + 1e-7
    assert np.all(rel[normal] <= np.broadcast_to(bound, rel.shape)[normal])
    assert np.all(np.sign(xh) == np.sign(x))
    # the expansion helps exactly when k > 1: tighter than the plain quantizer's 2^-4
    assert np.median(rel[normal]) < 2.0 ** -5


def test_f_inverse_of_f_identity_on_codes(ref):
    # quantizing a dequantized group reproduces the codes: DQ o Q idempotent at group level
    x = groups(41, ng=32)
    q, s, k = ref.quant_group(x, 128)
    xh = ref.dequant_group(q, s, k, 128)
    q2, s2, k2 = ref.quant_group(xh, 128)
    assert np.mean(q2 == q) > 0.995                     # fp32 rounding of xh can move a tie
    assert np.all(np.abs(q2.astype(int) - q.astype(int)) <= 1)
    assert np.allclose(s2, s, rtol=1e-6) and np.allclose(k2, k, rtol=1e-4)


def test_normalizer_route_gives_same_codes(ref):
    # Appendix F.4 normalizes by C_X = sqrt(Xmin*Xmax) before raising to k.  Then
    # Xmax/C_X = sqrt(R_X), the expanded maximum is sqrt(R_E4M3) and the plain quantizer's
    # scale is the constant sqrt(512*448)/448 = sqrt(8/7).  Same codes as the oracle's route.
    x = groups(42, ng=32)
    q, s, k = ref.quant_group(x, 128)
    xg = x.astype(np.float64).reshape(-1, 128)
    ax = np.abs(xg)
    C = np.sqrt(ax.max(1) * ax.min(1))[:, None]
    kk = k.astype(np.float64)[:, None]
    f = np.sign(xg) * (ax / C) ** kk
    S = np.abs(f).max(1, keepdims=True) / 448.0
    assert np.allclose(S, math.sqrt(8.0 / 7.0), rtol=1e-5)
    alt = nearest_codes((f / S).reshape(-1))
    assert np.mean(alt == q) > 0.999
    assert np.all(np.abs((alt & 0x7F).astype(int) - (q & 0x7F).astype(int)) <= 1)


def test_ragged_last_group(ref):
    x = groups(43, ng=3)[: 2 * 128 + 37]
    q, s, k = ref.quant_group(x, 128)
    assert q.size == x.size and s.size == 3
    q_tail, s_tail, k_tail = ref.quant_group(x[256:], 37)
    assert np.array_equal(q[256:], q_tail) and s[2] == s_tail[0] and k[2] == k_tail[0]
    assert ref.quant_group(np.zeros(0, np.float32), 128)[0].size == 0
