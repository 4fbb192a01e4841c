"""Seeded synthetic inputs for the FP8-state AdamW step: shapes, gradients, start states.

This module serves the tests, the smoke check and the bench.  It holds NONE of the
method's arithmetic (no quantizer, no expansion, no optimizer update): it only draws
random numbers with the value distributions of the workloads and formats them (fp32,
bf16 bit patterns, raw code bytes).  Neither the oracle nor the HIP path is imported here.

Workloads (parameter shapes are those of the Llama-2 models the paper trains; the value
distributions are stated per function):
  cfg1  one 1024 x 1024 matrix
  cfg2  the seven linear weights of one Llama-2-7B decoder layer
  cfg3  32 such layers plus embedding and LM head (the full 7B set)
  cfg5  the Llama-2-13B set
"""
from __future__ import annotations

import numpy as np

# ---------------------------------------------------------------------------------------
# shapes
# ---------------------------------------------------------------------------------------


def layer_shapes(hidden: int, ffn: int):
    """q, k, v, o projections and gate, up, down of one decoder layer."""
    return [(hidden, hidden)] * 4 + [(hidden, ffn)] * 3


def workload_shapes(name: str):
    if name == "cfg1":
        return [(1024, 1024)]
    if name == "cfg2":
        return layer_shapes(4096, 11008)
    if name == "cfg3":
        return layer_shapes(4096, 11008) * 32 + [(32000, 4096)] * 2
    if name == "cfg5":
        return layer_shapes(5120, 13824) * 40 + [(32000, 5120)] * 2
    raise ValueError(name)


def workload_numel(name: str) -> int:
    return int(sum(r * c for r, c in workload_shapes(name)))


# ---------------------------------------------------------------------------------------
# host (numpy) generators -- counter based: (seed, stream, step) keys a Philox stream, so
# any tensor of any step can be regenerated alone.
# ---------------------------------------------------------------------------------------

_STREAM_W, _STREAM_G, _STREAM_OUTLIER, _STREAM_STATE, _STREAM_ACT = 1, 2, 3, 4, 5


def _rng(seed: int, stream: int, step: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[(int(seed) << 8) | int(stream), int(step)]))


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (nearest, ties to even) and return the 16-bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    rounded = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
    return rounded.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def weights(n: int, seed: int, sigma: float = 0.02) -> np.ndarray:
    """Master weights ~ N(0, sigma^2), fp32."""
    return (_rng(seed, _STREAM_W).standard_normal(n, dtype=np.float32) * np.float32(sigma))


def outlier_group_mask(n_groups: int, seed: int, frac: float) -> np.ndarray:
    """A fixed subset of groups (the same at every step) that carries large gradients."""
    return _rng(seed, _STREAM_OUTLIER).random(n_groups) < frac


def grads_normal(n: int, seed: int, step: int, sigma: float = 1e-3, G: int = 128,
                 outlier_frac: float = 0.0, outlier_mult: float = 100.0) -> np.ndarray:
    """bf16 gradients ~ N(0, sigma^2); `outlier_frac` of the groups is scaled up."""
    g = _rng(seed, _STREAM_G, step).standard_normal(n, dtype=np.float32) * np.float32(sigma)
    if outlier_frac > 0.0:
        ng = (n + G - 1) // G
        mask = np.repeat(outlier_group_mask(ng, seed, outlier_frac), G)[:n]
        g[mask] *= np.float32(outlier_mult)
    return f32_to_bf16_bits(g)


def grads_lognormal(n: int, seed: int, step: int, base: float = 1e-3, sigma: float = 2.0) -> np.ndarray:
    """bf16 gradients with |g| = base * exp(sigma * z), z ~ N(0,1), and a random sign."""
    r = _rng(seed, _STREAM_G, step)
    z = r.standard_normal(n, dtype=np.float32)
    sign = np.where(r.random(n, dtype=np.float32) < 0.5, np.float32(-1), np.float32(1))
    return f32_to_bf16_bits(np.float32(base) * np.exp(np.float32(sigma) * z) * sign)


def activations(n: int, seed: int, hidden: int = 4096, sigma: float = 1.0, channel_frac: float = 1.0 / 512,
                channel_mult: float = 20.0, spike_frac: float = 1.0 / 4096, spike_mult: float = 60.0) -> np.ndarray:
    """bf16 activations of a [tokens, hidden] tensor, flattened row-major and cut to n elements:
    N(0, sigma^2) entries, a fixed set of outlier channels (columns) scaled by channel_mult and sparse
    single-element spikes scaled by spike_mult -- the heavy-tailed shape transformer activations have."""
    rng = _rng(seed, _STREAM_ACT)
    x = rng.standard_normal(n, dtype=np.float32) * np.float32(sigma)
    cols = np.arange(n, dtype=np.int64) % hidden
    hot = rng.random(hidden) < channel_frac
    x[hot[cols]] *= np.float32(channel_mult)
    x[rng.random(n) < spike_frac] *= np.float32(spike_mult)
    return f32_to_bf16_bits(x)


def zero_state(n: int, G: int):
    """The start state m0 = v0 = 0: all codes 0, scale 0, k 1."""
    ng = (n + G - 1) // G
    return dict(m_q=np.zeros(n, np.uint8), m_scale=np.zeros(ng, np.float32), m_k=np.ones(ng, np.float32),
                v_q=np.zeros(n, np.uint8), v_scale=np.zeros(ng, np.float32), v_k=np.ones(ng, np.float32))


def random_state(n: int, G: int, seed: int):
    """An arbitrary valid state: every finite code for m, non-negative codes for v,
    scales log-uniform over the magnitudes optimizer states take, k log-uniform in
    [0.5, 16).  A stress input: it does not come from any optimizer trajectory."""
    r = _rng(seed, _STREAM_STATE)
    ng = (n + G - 1) // G
    m_q = r.integers(0, 256, n, dtype=np.uint8)
    m_q[(m_q & 0x7F) == 0x7F] = 0x3C                      # no NaN codes
    v_q = r.integers(0, 127, n, dtype=np.uint8)           # sign clear, 0x7F excluded
    m_scale = np.exp(r.uniform(np.log(1e-7), np.log(1e-3), ng)).astype(np.float32)
    v_scale = np.exp(r.uniform(np.log(1e-13), np.log(1e-7), ng)).astype(np.float32)
    m_k = np.exp(r.uniform(np.log(0.5), np.log(16.0), ng)).astype(np.float32)
    v_k = np.exp(r.uniform(np.log(0.5), np.log(16.0), ng)).astype(np.float32)
    return dict(m_q=m_q, m_scale=m_scale, m_k=m_k, v_q=v_q, v_scale=v_scale, v_k=v_k)


# ---------------------------------------------------------------------------------------
# device (torch) generators for the full-size workloads: same distributions, drawn in
# place in device memory so that a 13B-parameter set needs no host copy.  Chunked so the
# temporaries stay small.
# ---------------------------------------------------------------------------------------

_CHUNK = 1 << 28


def torch_generator(device, seed: int):
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def torch_weights(n: int, device, gen, sigma: float = 0.02):
    import torch
    w = torch.empty(n, dtype=torch.float32, device=device)
    for lo in range(0, n, _CHUNK):
        w[lo:lo + _CHUNK].normal_(0.0, sigma, generator=gen)
    return w


def torch_outlier_group_mask(n_groups: int, device, gen, frac: float):
    import torch
    return torch.rand(n_groups, device=device, generator=gen) < frac


def torch_grads_normal(n: int, device, gen, sigma: float = 1e-3, G: int = 128,
                       outlier_mask=None, outlier_mult: float = 100.0, out=None):
    """bf16 gradients ~ N(0, sigma^2) (fp32 draw rounded to bf16); rows of `outlier_mask`
    (one bool per group, n divisible by G) are multiplied by `outlier_mult`."""
    import torch
    g = out if out is not None else torch.empty(n, dtype=torch.bfloat16, device=device)
    for lo in range(0, n, _CHUNK):
        hi = min(n, lo + _CHUNK)
        t = torch.empty(hi - lo, dtype=torch.float32, device=device).normal_(0.0, sigma, generator=gen)
        if outlier_mask is not None:
            assert lo % G == 0 and (hi - lo) % G == 0
            rows = outlier_mask[lo // G: hi // G]
            t.view(-1, G).mul_(torch.where(rows, outlier_mult, 1.0).to(torch.float32).unsqueeze(1))
        g[lo:hi].copy_(t)
    return g


def torch_grads_lognormal(n: int, device, gen, base: float = 1e-3, sigma: float = 2.0, out=None):
    import torch
    g = out if out is not None else torch.empty(n, dtype=torch.bfloat16, device=device)
    for lo in range(0, n, _CHUNK):
        hi = min(n, lo + _CHUNK)
        z = torch.empty(hi - lo, dtype=torch.float32, device=device).normal_(0.0, 1.0, generator=gen)
        z.mul_(sigma).exp_().mul_(base)
        s = torch.rand(hi - lo, device=device, generator=gen) < 0.5
        z.mul_(torch.where(s, -1.0, 1.0).to(torch.float32))
        g[lo:hi].copy_(z)
    return g


def torch_activations(n: int, device, gen, hidden: int = 4096, sigma: float = 1.0, channel_frac: float = 1.0 / 512,
                      channel_mult: float = 20.0, spike_frac: float = 1.0 / 4096, spike_mult: float = 60.0, out=None):
    """Device twin of activations() (same distribution, torch's own random stream); n % hidden == 0."""
    import torch
    assert n % hidden == 0
    x = out if out is not None else torch.empty(n, dtype=torch.bfloat16, device=device)
    hot = torch.rand(hidden, device=device, generator=gen) < channel_frac
    col_mult = torch.where(hot, channel_mult, 1.0).to(torch.float32)
    rows_per = max(1, _CHUNK // hidden)
    for lo in range(0, n // hidden, rows_per):
        hi = min(n // hidden, lo + rows_per)
        t = torch.empty((hi - lo, hidden), dtype=torch.float32, device=device).normal_(0.0, sigma, generator=gen)
        t.mul_(col_mult)
        spike = torch.rand((hi - lo, hidden), device=device, generator=gen) < spike_frac
        t.mul_(torch.where(spike, spike_mult, 1.0).to(torch.float32))
        x[lo * hidden: hi * hidden].copy_(t.view(-1))
    return x


def torch_moments(n: int, device, gen, G: int = 128, base: float = 1e-3, group_sigma: float = 1.0,
                  gamma_shape: float = 4.0):
    """fp32 first and second moments with the shape Sec. 4.1 describes: every group of G has its own
    gradient scale s_g = base * exp(group_sigma * z) (so scales differ widely ACROSS groups), while
    inside a group the dynamic range is small: m = s_g * N(0, 0.3^2), v = s_g^2 * Gamma(shape) / shape
    (what an exponential average of squared gradients of that scale looks like).  n % G == 0."""
    import torch
    assert n % G == 0
    z = torch.empty(n // G, dtype=torch.float32, device=device).normal_(0.0, 1.0, generator=gen)
    s = (z * group_sigma).exp_().mul_(base).unsqueeze(1)
    m = torch.empty((n // G, G), dtype=torch.float32, device=device).normal_(0.0, 0.3, generator=gen).mul_(s)
    acc = torch.zeros((n // G, G), dtype=torch.float32, device=device)
    for _ in range(int(gamma_shape)):                         # Gamma(k) for integer k = sum of k exponentials
        u = torch.rand((n // G, G), device=device, generator=gen).clamp_(min=1e-12)
        acc.sub_(u.log_())
    v = acc.div_(gamma_shape).mul_(s * s)
    return m.reshape(-1), v.reshape(-1)


def torch_zero_state(n: int, G: int, device):
    import torch
    ng = (n + G - 1) // G
    return dict(m_q=torch.zeros(n, dtype=torch.uint8, device=device),
                m_scale=torch.zeros(ng, dtype=torch.float32, device=device),
                m_k=torch.ones(ng, dtype=torch.float32, device=device),
                v_q=torch.zeros(n, dtype=torch.uint8, device=device),
                v_scale=torch.zeros(ng, dtype=torch.float32, device=device),
                v_k=torch.ones(ng, dtype=torch.float32, device=device))


def torch_random_state(n: int, G: int, device, gen):
    """Device twin of random_state (same distributions, torch's generator)."""
    import math
    import torch
    ng = (n + G - 1) // G
    m_q = torch.empty(n, dtype=torch.uint8, device=device)
    v_q = torch.empty(n, dtype=torch.uint8, device=device)
    for lo in range(0, n, _CHUNK):
        hi = min(n, lo + _CHUNK)
        t = torch.randint(0, 256, (hi - lo,), dtype=torch.uint8, device=device, generator=gen)
        t[(t & 0x7F) == 0x7F] = 0x3C
        m_q[lo:hi] = t
        v_q[lo:hi] = torch.randint(0, 127, (hi - lo,), dtype=torch.uint8, device=device, generator=gen)

    def logu(lo_, hi_):
        u = torch.rand(ng, device=device, generator=gen, dtype=torch.float64)
        return torch.exp(math.log(lo_) + u * (math.log(hi_) - math.log(lo_))).to(torch.float32)

    return dict(m_q=m_q, m_scale=logu(1e-7, 1e-3), m_k=logu(0.5, 16.0),
                v_q=v_q, v_scale=logu(1e-13, 1e-7), v_k=logu(0.5, 16.0))
