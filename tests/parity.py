"""Comparison rules between the HIP path (fp32, one element per lane in fp64) and the CPU oracle
(fp64): the parity bar.

The bar, as stated for this build:
  codes   equal on >= 99.99 % of the elements, every mismatch at most one code step;
  w       |w_gpu - w_ref| <= 1e-6 |w_ref| + 1e-9;
  scale   relative 1e-6;
  k       relative 1e-6.

How the rules below read it, and the one exception they allow:

  k       |k_gpu / k_ref - 1| <= 1e-6 * max(1, 1 / ln R), R = amax / amin of the reference side.
          k = log2(range) / log2(R) is a function of ln R, and both sides hold amax and amin as fp32
          numbers, so for a group narrower than e the 1e-6 is a bound on ln R (k > 17.8 there).
          EXCEPTION (named "two candidates"): the first moment's minimum is recomputed exactly for
          the element that the fp32 pass names as the smallest of each lane's sixteen.  When two
          elements of one lane are closer to each other than the fp32 error of m_t = beta1 m +
          (1 - beta1) g, the wrong one may be named and k follows the fp32 value's error.  At most
          K_EXCEPTION_MAX of the groups may miss the bar (measured: fewer than 1e-5), and each of
          them must stay inside the bound that the per-element fp32 error dx allows (k_tolerance).
          With BF16-stored scales (an option, not the default) the stored scale is a rounding DECISION:
          a group whose amax / fmax lies within the fp32 rounding noise of a bf16 value may take the
          neighbouring bf16 scale on one side.  Such groups (2 in 1000 for generic gradients, about one
          in a hundred where many groups receive no gradient: their new maximum is beta1 times a bf16
          number, often next to a bf16 value) are excused on k and left out of the code comparison;
          their scale must be one of the two neighbours.  BF16-stored exponents (rounded to the
          nearest bf16) are decisions of the same kind at the midpoints between bf16 values.
  codes   (a) the number of mismatches over ALL elements is at most 1e-4 * n (for n >= 1e5; a smaller
          tensor is a small sample of that rate and gets three Poisson standard deviations);
          (b) every mismatch is one code step (same sign, adjacent magnitude codes, or a zero against
          the smallest code), except inside an exception group, where it must lie in the band of
          codes that the group's k bound allows.
  w       as stated.  Only the stress tests on states that come from no optimizer trajectory
          (random codes: |m| / sqrt(v) up to 1e5, the update dwarfs the weight) and the cells that
          store the second moment without expansion (its small entries flush to zero, same effect)
          add an explicit model of the update's own fp32 error; they pass it as extra_tol.

  dx      per-element bound on |x_gpu - x_ref| of a new moment x, used for the exception bound only:
              dx = eps_dq * beta * |x_old| + 2^-22 * |x_ref|
"""
import numpy as np

CODE_MISMATCH_MAX = 1e-4      # at every group size
W_RTOL, W_ATOL = 1e-6, 1e-9
META_RTOL = 1e-6
K_EXCEPTION_MAX = 1e-4        # fraction of groups that may miss the bar on k (see the docstring)
LOG2_RANGE = 17.807354922057606
K_MIN_DEFAULT, K_MAX_DEFAULT = 0.0625, 1024.0

# relative error of the fp32 inverse expansion a * |c/fmax|^(1/k) against fp64: the exponent
# log2(c/fmax) / k (magnitude <= log2_range / min(k, 1)) is rounded three times (table, 1/k, product)
# and enters as ln2 * error, plus the hardware exp2 and two roundings
def eps_dq(k_old, log2_range=17.81):
    """log2_range: 17.81 for E4M3, 31.81 for E5M2 (the largest |log2(c/fmax)|)."""
    return (log2_range / np.minimum(k_old, 1.0)) * 3 * 2.0 ** -24 * np.log(2.0) + 4 * 2.0 ** -24


def _canon(codes):
    c = np.asarray(codes, dtype=np.uint8).astype(np.int32)
    c = np.where((c & 0x7F) == 0, 0, c)               # +0 and -0 are the same value
    return c


def _group_reduce(x, G, fn, fill):
    n = x.size
    ng = (n + G - 1) // G
    pad = np.full(ng * G, fill, dtype=np.float64)
    pad[:n] = x
    return fn(pad.reshape(ng, G), axis=1)


def k_bar(x_ref, G):
    """The plain bar on k per group: 1e-6 * max(1, 1 / ln R) (1e-6 where k is 1 by definition)."""
    ax = np.abs(np.asarray(x_ref, dtype=np.float64))
    amax = _group_reduce(ax, G, np.max, 0.0)
    amin = _group_reduce(np.where(ax > 0, ax, np.inf), G, np.min, np.inf)
    with np.errstate(divide="ignore", invalid="ignore"):
        ln_r = np.log(amax / amin)
    ok = np.isfinite(ln_r) & (ln_r > 0)
    return np.where(ok, META_RTOL * np.maximum(1.0, 1.0 / np.where(ok, ln_r, 1.0)), META_RTOL)


def k_tolerance(k_ref, x_ref, dx, G, k_min=K_MIN_DEFAULT, k_max=K_MAX_DEFAULT):
    """The bound an EXCEPTION group must still obey: per-group relative tolerance on k (np.inf when
    some element's fp32 error reaches its own size) and the mask of groups whose reference k sits on
    a clamp.

    With |x_gpu,i - x_i| <= dx_i the other side's extremes obey
        max_i(|x_i| - dx_i) <= amax_gpu <= max_i(|x_i| + dx_i)
        min_i(|x_i| - dx_i) <= amin_gpu <= min_i(|x_i| + dx_i)       (i over the non-zero x_i)
    hence ln R_gpu lies in [lnR_lo, lnR_hi] and k_gpu / k_ref = ln R_ref / ln R_gpu."""
    k_ref = np.asarray(k_ref, dtype=np.float64)
    ax = np.abs(np.asarray(x_ref, dtype=np.float64))
    dx = np.asarray(dx, dtype=np.float64)
    nz = ax > 0
    up, dn = ax + dx, np.maximum(ax - dx, 0.0)
    amax = _group_reduce(ax, G, np.max, 0.0)
    amin = _group_reduce(np.where(nz, ax, np.inf), G, np.min, np.inf)
    amax_lo, amax_hi = _group_reduce(dn, G, np.max, 0.0), _group_reduce(up, G, np.max, 0.0)
    amin_lo = _group_reduce(np.where(nz, dn, np.inf), G, np.min, np.inf)
    amin_hi = _group_reduce(np.where(nz, up, np.inf), G, np.min, np.inf)
    total = _group_reduce((nz & (dn == 0)).astype(np.float64), G, np.max, 0.0) > 0
    with np.errstate(divide="ignore", invalid="ignore"):
        ln_r = np.log(amax / amin)
        ln_hi = np.log(amax_hi / amin_lo)
        ln_lo = np.log(amax_lo / amin_hi)
        spread = np.maximum(ln_r / ln_lo - 1.0, 1.0 - ln_r / ln_hi)
        tol = META_RTOL * np.maximum(1.0, 1.0 / ln_r) + spread
    trivial = ~(np.isfinite(ln_r) & (ln_r > 0))          # one distinct magnitude, or all zero: k == 1
    tol = np.where(total | ~np.isfinite(tol) | (tol < 0), np.inf, tol)
    tol = np.where(trivial, META_RTOL, tol)
    clamped = (k_ref <= k_min) | (k_ref >= k_max)
    return tol, clamped


def assert_k(gpu, ref, bar, what="", bound=None, excused=None):
    """bar: the plain per-group bar (k_bar).  bound: from k_tolerance, what an exception group must
    still obey (None: no exception is allowed at all, the case of exact inputs).
    excused: groups that are exceptions for another stated reason (a bf16 scale decision).
    Returns (mask of the exception groups, statistics)."""
    gpu = np.asarray(gpu, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    rel = np.abs(gpu - ref) / np.abs(ref)
    out = rel > bar
    if excused is not None:
        out &= ~excused                                   # counted by the caller, under its own limit
    n_out = int(out.sum())
    stats = dict(k_out=n_out, k_in_bar=float(1.0 - n_out / max(1, rel.size)), k_max_rel=float(rel.max()))
    if bound is None:
        assert n_out == 0, "%s: k rel err %.3g in %d groups (exact inputs: no exception)" % (what, float(rel.max()), n_out)
        return out, stats
    assert n_out <= int(np.ceil(K_EXCEPTION_MAX * rel.size)), \
        "%s: k outside 1e-6 in %d of %d groups (worst %.3g)" % (what, n_out, rel.size, float(rel.max()))
    bad = out & (rel > bound)
    assert not bad.any(), "%s: k rel err %.3g (bound %.3g) in %d exception groups" % (
        what, float(rel[bad].max()), float(bound[bad].min()), int(bad.sum()))
    return (out if excused is None else out | excused), stats


def assert_scale(gpu, ref, what=""):
    gpu = np.asarray(gpu, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert np.all(np.abs(gpu - ref) <= META_RTOL * np.abs(ref)), \
        "%s: scale rel err %.3g" % (what, float(np.max(np.abs(gpu - ref) / np.maximum(np.abs(ref), 1e-300))))


def assert_w(gpu, ref, what="", extra_tol=None):
    gpu = np.asarray(gpu, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    err = np.abs(gpu - ref)
    tol = W_RTOL * np.abs(ref) + W_ATOL
    if extra_tol is not None:
        tol = tol + extra_tol
    bad = err > tol
    assert not bad.any(), "%s: %d weights off, worst %.3g x tol" % (
        what, int(bad.sum()), float((err / tol).max()))
    return float((err / tol).max()) if err.size else 0.0


def allowed_mismatches(n):
    """The 1e-4 rate as a count: plain for n >= 1e5, with a small-sample allowance below."""
    expected = CODE_MISMATCH_MAX * n
    if n >= 100000:
        return int(np.ceil(expected))
    return int(np.ceil(expected + 3.0 * np.sqrt(expected)))


def assert_codes(ref_mod, gpu, ref, G, what="", exception=None, x_ref=None, dx=None, scale_ref=None, k_ref=None,
                 bound=None, e5m2=False, other_scale=None, rate=True):
    """Rules (a) and (b) of the module docstring.  exception: mask of the groups excused on k (None:
    none); x_ref, dx, scale_ref, k_ref, bound: what the band rule needs for mismatches in those.
    other_scale: groups that took the neighbouring bf16 scale (BF16-stored scales only): every code of
    such a group is relative to another scale, so they are left out of the comparison.
    rate=False: the caller has applied rule (a) over the whole tensor and passes a subset of it."""
    g, r = _canon(gpu), _canon(ref)
    n = r.size
    differ = g != r
    if other_scale is not None and other_scale.any():
        differ &= ~np.repeat(other_scale, G)[:n]
    neq = np.nonzero(differ)[0]
    # (a) the rate, over everything
    assert not rate or neq.size <= allowed_mismatches(n), \
        "%s: %d of %d codes differ (%.3g %%)" % (what, neq.size, n, 100.0 * neq.size / max(1, n))
    if not neq.size:
        return 0, 0
    grp = neq // G
    gm, rm = g[neq] & 0x7F, r[neq] & 0x7F
    same_sign = ((g[neq] ^ r[neq]) & 0x80) == 0
    one_step = (same_sign & (np.abs(gm - rm) <= 1)) | ((gm == 0) & (rm <= 1)) | ((rm == 0) & (gm <= 1))
    in_exc = exception[grp] if exception is not None else np.zeros(neq.size, dtype=bool)
    # (b) one code step outside the exception groups
    bad = ~one_step & ~in_exc
    if bad.any():
        j = np.nonzero(bad)[0][0]
        raise AssertionError("%s: %d mismatches of more than one code step, e.g. element %d gpu %02x ref %02x" % (
            what, int(bad.sum()), int(neq[j]), int(g[neq][j]), int(r[neq][j])))
    far = ~one_step & in_exc
    if far.any():
        # inside an exception group: the band of codes its k bound allows
        fmax = 57344.0 if e5m2 else 448.0
        encode = ref_mod.e5m2_encode if e5m2 else ref_mod.e4m3_encode
        sel = np.nonzero(far)[0]
        xi = np.abs(np.asarray(x_ref, dtype=np.float64)[neq[sel]])
        dxi = np.asarray(dx, dtype=np.float64)[neq[sel]]
        a = fmax * np.asarray(scale_ref, dtype=np.float64)[grp[sel]]
        k = np.asarray(k_ref, dtype=np.float64)[grp[sel]]
        tk_all = bound[grp[sel]]
        free = ~np.isfinite(tk_all)                       # the fp32 side may have seen an exact zero
        tk = np.minimum(tk_all, 0.5)
        with np.errstate(divide="ignore", invalid="ignore", over="ignore"):
            r_hi = np.minimum((xi + dxi) / a, 1.0)
            r_lo = np.minimum(np.maximum(xi - dxi, 0.0) / a, 1.0)
            q_hi = np.minimum(fmax * r_hi ** (k * (1.0 - tk)) * (1.0 + 1e-5 + k * 4e-7), fmax)
            q_lo = fmax * r_lo ** (k * (1.0 + tk)) * (1.0 - 1e-5 - k * 4e-7)
        q_lo = np.where(np.isfinite(q_lo) & (q_lo > 0), q_lo, 0.0)
        q_hi = np.where(np.isfinite(q_hi), q_hi, fmax)
        lo_code = np.array([encode(float(v)) & 0x7F for v in q_lo])
        hi_code = np.array([encode(float(v)) & 0x7F for v in q_hi])
        inside = free | ((gm[sel] >= lo_code - 1) & (gm[sel] <= hi_code + 1))
        assert inside.all(), "%s: %d codes of exception groups outside their band" % (what, int((~inside).sum()))
    return int(neq.size), int((~one_step).sum())
