"""The hardware FP32 -> FP8 conversion as the library uses it, through the C ABI.

coat_quant_group without expansion (the plain quantizer of Sec. 3: code = round(x / scale)) on groups
whose largest magnitude is exactly fmax has scale == 1, so the quotient is the input itself and the
code is the hardware's rounding of a chosen fp32 value.  The expected codes come from the oracle's
encoder (round to nearest, ties to even, written from the format definition), BIT FOR BIT: every
midpoint between two neighbouring representable values and its two fp32 neighbours, every
representable value, the subnormals, values around half the smallest subnormal, and both zeros."""
import numpy as np
import pytest
import torch

from test_gpu_parity import check_quant, coat, dev  # noqa: F401  (coat is a fixture)

pytestmark = pytest.mark.gpu


def probe_values(decode, last_finite):
    vals = np.array([decode(c) for c in range(last_finite + 1)], dtype=np.float32)   # increasing, exact in fp32
    mid = ((vals[:-1].astype(np.float64) + vals[1:].astype(np.float64)) / 2).astype(np.float32)
    assert np.all(mid.astype(np.float64) * 2 == vals[:-1].astype(np.float64) + vals[1:].astype(np.float64))
    pts = [vals, mid, np.nextafter(mid, np.float32(0)), np.nextafter(mid, np.float32(np.inf)),
           np.nextafter(vals[1:], np.float32(0)), np.nextafter(vals[:-1], np.float32(np.inf))]
    tiny = vals[1] * np.array([0.25, 0.4999999, 0.5, 0.5000001, 0.75, 1.4999999, 1.5, 1.5000001], dtype=np.float32)
    x = np.concatenate(pts + [tiny, np.array([0.0, 2.0 ** -126, 2.0 ** -149], dtype=np.float32)])
    return np.concatenate([x, -x])


@pytest.mark.parametrize("e5m2", [False, True])
@pytest.mark.parametrize("G", [32, 128])
def test_plain_quantizer_is_the_format_rounding(coat, ref, e5m2, G):
    decode, encode = (ref.e5m2_decode, ref.e5m2_encode) if e5m2 else (ref.e4m3_decode, ref.e4m3_encode)
    fmax, last = (57344.0, 0x7B) if e5m2 else (448.0, 0x7E)
    p = probe_values(decode, last)
    # G - 1 probes per group, the group's last element is fmax itself: amax == fmax, scale == 1
    ng = (p.size + G - 2) // (G - 1)
    x = np.zeros((ng, G), dtype=np.float32)
    flat = np.zeros(ng * (G - 1), dtype=np.float32)
    flat[:p.size] = p
    x[:, :G - 1] = flat.reshape(ng, G - 1)
    x[:, G - 1] = fmax
    x = x.reshape(-1)
    q, s, k = (t.cpu().numpy() for t in coat.coat_quant_group(dev(x), G, expand=False, e5m2=e5m2))
    assert np.all(s == 1.0) and np.all(k == 1.0)
    expect = np.array([encode(float(v)) for v in x], dtype=np.uint8)
    canon = lambda c: np.where((c & 0x7F) == 0, 0, c)          # noqa: E731  (+0 and -0 are one value)
    bad = np.nonzero(canon(q) != canon(expect))[0]
    assert bad.size == 0, "x = %r: code %02x, format rounding %02x (%d in all)" % (
        float(x[bad[0]]), int(q[bad[0]]), int(expect[bad[0]]), bad.size)
    # and the oracle's quantizer as a whole agrees with its encoder on these inputs
    q_r, s_r, k_r = ref.quant_group(x, G, expand=False, e5m2=e5m2)
    assert np.array_equal(canon(q_r), canon(expect)) and np.all(s_r == 1.0)


def test_expansion_at_the_largest_exponent_never_leaves_the_format(coat, ref):
    # k_max = 65536 (the largest the kernels accept) on groups a few ulp wide: k sits on the clamp, the
    # largest element's expanded value is 448 * (1 + ulps)^65536, still below the half-way point 464,
    # so no code may be NaN and every group's largest element must get the largest finite code
    n, G = 16 * 1024, 128
    rng = np.random.default_rng(5)
    base = np.float32(7.0e-4)
    x = (np.full(n, base, np.float32).view(np.int32) + rng.integers(0, 4, n).astype(np.int32)).view(np.float32)
    x = x * rng.choice([-1.0, 1.0], n).astype(np.float32)
    q, s, k = (t.cpu().numpy() for t in coat.coat_quant_group(dev(x), G, k_min=0.0625, k_max=65536.0))
    q_r, s_r, k_r = ref.quant_group(x, G, k_min=0.0625, k_max=65536.0)
    assert np.all(k == 65536.0) and np.all(k_r == 65536.0)
    assert np.all((q & 0x7F) != 0x7F), "a NaN code"
    top = np.abs(x).reshape(-1, G).argmax(1) + np.arange(n // G) * G
    assert np.all((q[top] & 0x7F) == 0x7E) and np.all((q_r[top] & 0x7F) == 0x7E)
    assert np.all(np.abs(s / s_r - 1.0) <= 1e-6)
    # one ulp of x moves the expanded value by 65536 * 2^-23 = 0.8 %, a code step is 6 to 12 %: the two
    # sides may differ where a value sits that close to a rounding boundary, never by more than a step
    diff = np.abs((q & 0x7F).astype(int) - (q_r & 0x7F).astype(int))
    assert np.all((q & 0x80) == (q_r & 0x80)) and diff.max() <= 1
    assert np.mean(diff != 0) < 0.15


def test_gradients_whose_squares_underflow_stay_in_their_group(coat, ref):
    # |g| ~ 1e-20: g^2 is below the smallest normal fp32 number.  Such a second moment is far below
    # anything an optimizer holds and the header puts it outside the compared domain; what is promised
    # is that the group's stored state stays valid and that no other group notices.
    from test_gpu_parity import HP, gpu_step
    import synth_inputs as S
    n, G = 8 * 1024, 128
    w = S.weights(n, 3)
    st = S.zero_state(n, G)
    g = S.grads_normal(n, 3, 1, G=G)
    g_tiny = g.copy()
    tiny = S.f32_to_bf16_bits(np.full(G, 1e-20, np.float32) * np.resize(np.array([1, -1, 2, 0.5], np.float32), G))
    for grp in (0, 17, 63):
        g_tiny[grp * G + 5: grp * G + 60] = tiny[5:60]          # part of the group
    g_tiny[40 * G: 41 * G] = tiny                               # a whole group
    touched = np.zeros(n // G, bool)
    touched[[0, 17, 40, 63]] = True
    w_a, st_a, _ = gpu_step(coat, w, g, st, G, 1)
    w_b, st_b, _ = gpu_step(coat, w, g_tiny, st, G, 1)
    el = np.repeat(~touched, G)
    assert np.array_equal(w_a[el], w_b[el])
    for key in st_a:
        same = el if st_a[key].size == n else ~touched
        assert np.array_equal(st_a[key][same], st_b[key][same]), key
    assert np.all(np.isfinite(w_b))
    for name in ("m", "v"):
        assert np.all(np.isfinite(st_b[name + "_scale"])) and np.all(st_b[name + "_scale"] >= 0)
        assert np.all((st_b[name + "_k"] >= 0.0625) & (st_b[name + "_k"] <= 1024.0))
        assert np.all((st_b[name + "_q"] & 0x7F) != 0x7F)
    # the group made of such gradients only: its second moment's scale would be subnormal -> zero state
    assert np.all(st_b["v_q"][40 * G: 41 * G] == 0) and st_b["v_scale"][40] == 0.0 and st_b["v_k"][40] == 1.0
    # the first moment of those groups (1e-21, a normal number) is compared as usual
    w_r, st_r = w.copy(), {k_: v.copy() for k_, v in st.items()}
    assert ref.fp8_adamw_step(w_r, g_tiny, *(st_r[k_] for k_ in ("m_q", "m_scale", "m_k", "v_q", "v_scale", "v_k")),
                              ref.make_hparams(step=1, group_size=G, **HP)) == 0
    assert np.all(np.abs(st_b["m_scale"].astype(np.float64) - st_r["m_scale"]) <= 1e-6 * st_r["m_scale"])
