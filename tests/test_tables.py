"""The logarithm tables the HIP kernels keep in LDS (csrc/coat_tables.inc) are data, not code:
check every entry against the format definitions and a double-precision logarithm.  No GPU."""
import math
import os
import re

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def parse_tables():
    text = open(os.path.join(ROOT, "paper_2410_19313_amd", "csrc", "coat_tables.inc")).read()
    text = re.sub(r"//[^\n]*", "", text)
    body = text[text.index("kLog2Code"):]
    pairs = re.findall(r"\{\s*([^{},]+?)\s*,\s*([^{},]+?)\s*\}", body)
    assert len(pairs) == 256

    def val(tok):
        tok = tok.strip()
        if tok.startswith("__builtin_huge_valf"):
            return math.inf
        if tok.startswith("__builtin_nanf"):
            return math.nan
        tok = tok.rstrip("f")
        return float.fromhex(tok) if "x" in tok else float(tok)

    vals = [(val(a), val(b)) for a, b in pairs]
    return vals[:128], vals[128:]


def e4m3(c):       # OCP E4M3: bias 7, subnormals at exponent field 0, no infinity, 0x7F NaN
    e, m = c >> 3, c & 7
    return m * 2.0 ** -9 if e == 0 else (1 + m / 8) * 2.0 ** (e - 7)


def e5m2(c):       # OCP E5M2: bias 15, IEEE-like
    e, m = c >> 2, c & 3
    return m * 2.0 ** -16 if e == 0 else (1 + m / 4) * 2.0 ** (e - 15)


def check(table, decode, fmax, last_finite):
    hi0, lo0 = table[0]
    assert hi0 <= -1e29 and math.isfinite(hi0) and lo0 == 0.0          # code 0: finite sentinel, exp2 gives exactly 0
    for c in range(1, last_finite + 1):
        hi, lo = table[c]
        L = math.log2(decode(c) / fmax)
        assert hi == float(np.float32(L)), (c, hi, L)                   # hi: the fp32 nearest to the logarithm
        assert lo == float(np.float32(lo)) and abs(lo) <= abs(hi) * 2.0 ** -24 + 1e-45
        assert abs((hi + lo) - L) <= 2.0 ** -44 * max(abs(L), 1.0), (c, hi + lo, L)
    assert table[last_finite] == (0.0, 0.0)                             # the largest code is fmax itself


def test_log2_tables_match_the_formats():
    t43, t52 = parse_tables()
    check(t43, e4m3, 448.0, 0x7E)
    assert math.isnan(t43[0x7F][0])
    check(t52, e5m2, 57344.0, 0x7B)
    assert t52[0x7C][0] == math.inf and all(math.isnan(t52[c][0]) for c in (0x7D, 0x7E, 0x7F))


def test_committed_tables_are_what_the_generator_writes():
    import importlib.util
    path = os.path.join(ROOT, "paper_2410_19313_amd", "csrc", "make_tables.py")
    spec = importlib.util.spec_from_file_location("make_tables", path)
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    assert open(mod.OUT).read() == mod.render(), "coat_tables.inc is stale: run make_tables.py"


def test_exp2_fraction_table_is_correctly_rounded():
    # kExp2Frac512[j] is the double nearest to 2^(j/512): with h half an ulp of v, exactly,
    # (v - h)^512 <= 2^j <= (v + h)^512 in rational arithmetic
    from fractions import Fraction
    text = open(os.path.join(ROOT, "paper_2410_19313_amd", "csrc", "coat_tables.inc")).read()
    body = text[text.index("kExp2Frac512[kExp2FracSize]"):]
    vals = [float.fromhex(t) for t in re.findall(r"-?0x[0-9a-f.]+p[+-]?\d+", body)]
    assert len(vals) == 512 and vals[0] == 1.0
    for j, v in enumerate(vals):
        assert 1.0 <= v < 2.0
        h = Fraction(1, 2 ** 53)                          # half an ulp of a double in [1, 2)
        assert (Fraction(v) - h) ** 512 <= Fraction(2) ** j <= (Fraction(v) + h) ** 512, j
