"""Pins for the oracle's E4M3 codec (no GPU needed).

The codec is pinned to things other than itself: the constants the paper prints
(tests/golden/e4m3_constants.txt), the bit-field definition of OCP E4M3 written out as a
table here, a brute-force nearest-value search, and torch's float8_e4m3fn casts used as a
black-box library routine.
"""
import math
import os

import numpy as np
import pytest
import torch

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "e4m3_constants.txt")


def golden():
    out = {}
    with open(GOLDEN) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                name, val = line.split()
                out[name] = float(val)
    return out


def torch_decode_table():
    return torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).to(torch.float64).numpy()


def finite_codes():
    return [c for c in range(256) if (c & 0x7F) != 0x7F]


def test_decode_matches_paper_constants(ref):
    g = golden()
    pos = [ref.e4m3_decode(c) for c in range(1, 0x7F)]
    assert min(pos) == g["delta_min_e4m3"] == 2.0 ** -9
    assert max(pos) == g["delta_max_e4m3"] == 448.0
    assert max(pos) / min(pos) == g["range_e4m3"]
    assert ref.e4m3_decode(0x01) == 2.0 ** -9 and ref.e4m3_decode(0x7E) == 448.0


def test_decode_all_codes_vs_library(ref):
    lib = torch_decode_table()
    for c in range(256):
        d = ref.e4m3_decode(c)
        if (c & 0x7F) == 0x7F:
            assert math.isnan(d) and math.isnan(lib[c])
        else:
            assert d == lib[c], (c, d, lib[c])
            assert math.copysign(1.0, d) == (-1.0 if c & 0x80 else 1.0)


def test_decode_bitfield_definition(ref):
    # sign / 4-bit exponent (bias 7) / 3-bit mantissa, subnormals at exponent field 0
    for c in finite_codes():
        s, e, m = c >> 7, (c >> 3) & 15, c & 7
        v = (m / 8.0) * 2.0 ** -6 if e == 0 else (1 + m / 8.0) * 2.0 ** (e - 7)
        assert ref.e4m3_decode(c) == (-v if s else v)


def test_decode_is_strictly_increasing_in_code(ref):
    vals = [ref.e4m3_decode(c) for c in range(0, 0x7F)]
    assert all(b > a for a, b in zip(vals, vals[1:]))


def test_encode_decode_idempotent_all_codes(ref):
    # DQ o Q is the identity on representable values: brute force over every code
    for c in finite_codes():
        assert ref.e4m3_encode(ref.e4m3_decode(c)) == c
    assert ref.e4m3_encode(float("nan")) & 0x7F == 0x7F


def brute_force_encode(ref, q):
    """Nearest representable value by exhaustive search; ties go to the even code."""
    best, best_d = None, None
    for c in range(0, 0x7F):
        d = abs(ref.e4m3_decode(c) - min(abs(q), 448.0))
        if best is None or d < best_d or (d == best_d and c % 2 == 0 and best % 2 == 1):
            best, best_d = c, d
    return best | (0x80 if math.copysign(1.0, q) < 0 else 0)


def test_encode_midpoints_and_neighbours(ref):
    vals = [ref.e4m3_decode(c) for c in range(0, 0x7F)]
    for c in range(0, 0x7E):
        lo, hi = vals[c], vals[c + 1]
        mid = (lo + hi) / 2.0                      # exact in fp64
        even = c if c % 2 == 0 else c + 1
        assert ref.e4m3_encode(mid) == even, (c, mid)
        assert ref.e4m3_encode(-mid) == (even | 0x80)
        assert ref.e4m3_encode(math.nextafter(mid, 0.0)) == c
        assert ref.e4m3_encode(math.nextafter(mid, 1e9)) == c + 1


def test_encode_saturates_never_nan(ref):
    for q in (448.0, 449.0, 463.99, 464.0, 480.0, 1e30, float("inf")):
        assert ref.e4m3_encode(q) == 0x7E
        assert ref.e4m3_encode(-q) == 0xFE
    assert ref.e4m3_encode(0.0) == 0x00 and ref.e4m3_encode(-0.0) == 0x80
    assert ref.e4m3_encode(2.0 ** -10) == 0x00          # tie between 0 and 2^-9 -> even
    assert ref.e4m3_encode(math.nextafter(2.0 ** -10, 1.0)) == 0x01


def test_encode_brute_force_random(ref):
    rng = np.random.default_rng(1)
    xs = np.concatenate([
        rng.uniform(-470, 470, 2000),
        np.exp(rng.uniform(np.log(2.0 ** -12), np.log(500.0), 4000)) * rng.choice([-1.0, 1.0], 4000),
    ])
    for q in xs:
        assert ref.e4m3_encode(float(q)) == brute_force_encode(ref, float(q)), q


def test_encode_monotone(ref):
    xs = np.sort(np.exp(np.random.default_rng(2).uniform(np.log(1e-4), np.log(460.0), 20000)))
    codes = [ref.e4m3_encode(float(x)) for x in xs]
    assert all(b >= a for a, b in zip(codes, codes[1:]))


def test_encode_vs_library_cast(ref):
    # torch's CPU cast is round-to-nearest-even inside the finite range
    rng = np.random.default_rng(3)
    xs = np.concatenate([
        rng.uniform(-448, 448, 100000),
        np.exp(rng.uniform(np.log(2.0 ** -11), np.log(448.0), 100000)) * rng.choice([-1.0, 1.0], 100000),
    ]).astype(np.float32)
    lib = torch.from_numpy(xs).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    mine = np.array([ref.e4m3_encode(float(x)) for x in xs], dtype=np.uint8)
    assert np.array_equal(mine, lib)


def test_encode_all_bf16_patterns_vs_library(ref):
    # every bf16 bit pattern with magnitude inside the finite range
    bits = np.arange(65536, dtype=np.uint32) << 16
    xs = bits.view(np.float32)
    keep = np.isfinite(xs) & (np.abs(xs) <= 448.0)
    xs = xs[keep]
    lib = torch.from_numpy(xs.copy()).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    mine = np.array([ref.e4m3_encode(float(x)) for x in xs], dtype=np.uint8)
    assert np.array_equal(mine, lib)
