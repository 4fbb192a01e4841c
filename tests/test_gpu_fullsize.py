"""GPU parity at the full sizes of the workloads, in the launch configuration bench.py times:
one step over the whole flat buffer (202M, 6.7B and 13B parameters), checked on sampled groups
that the CPU oracle recomputes one by one.  Groups are independent, so a sampled group's result
must match the oracle run on that group alone.

The start state is the seeded synthetic state of synth_inputs (random codes, scales, exponents):
it is an input, not the product of earlier HIP steps, so nothing the oracle sees comes from the
HIP path."""
import numpy as np
import pytest
import torch

import synth_inputs as S
from test_gpu_parity import HP, check_step, coat, update_error_model  # noqa: F401  (coat is a fixture)

pytestmark = pytest.mark.gpu


def sample_groups(ng, count, seed):
    rng = np.random.default_rng(seed)
    idx = np.unique(np.concatenate([np.arange(8), np.arange(ng - 8, ng), rng.integers(0, ng, count)]))
    return idx


def gather(t, idx_dev, G):
    return t.view(-1, G).index_select(0, idx_dev).reshape(-1).cpu()


@pytest.mark.parametrize("workload,G,grads,flags", [
    ("cfg2", 128, "normal", {}), ("cfg2", 32, "lognormal", {}), ("cfg2", 512, "lognormal", {}),
    ("cfg3", 128, "normal", {}), ("cfg5", 128, "normal", {}),
    ("cfg3", 128, "normal", dict(bf16_scale=True)),                 # scales stored in BF16 (Sec. 3)
    ("cfg3", 128, "normal", dict(m_e5m2=True, v_e5m2=True)),        # a cell of Table 1 through the generic kernel
])
def test_full_size_sampled(coat, ref, workload, G, grads, flags):
    dev = torch.device("cuda:0")
    n = S.workload_numel(workload)
    need = n * 9 + (1 << 31)
    free, _ = torch.cuda.mem_get_info()
    if free < need:
        pytest.skip("needs %.0f GB of device memory" % (need / 1e9))
    ng = n // G
    gen = S.torch_generator(dev, 100 + G)
    w = S.torch_weights(n, dev, gen)
    st = S.torch_random_state(n, G, dev, gen)
    if flags.get("bf16_scale"):
        # an input like any other: the synthetic scales, made bf16 values (the oracle holds them as floats)
        for k in ("m_scale", "v_scale"):
            st[k] = st[k].to(torch.bfloat16)
    for name in ("m", "v"):
        if flags.get(name + "_e5m2"):
            # E5M2 has infinities and NaNs at 0x7C..0x7F: keep the synthetic codes finite
            q = st[name + "_q"]
            q.copy_((q & 0x80) | torch.clamp(q & 0x7F, max=0x7B))
    if grads == "normal":
        g = S.torch_grads_normal(n, dev, gen, G=G, outlier_mask=S.torch_outlier_group_mask(ng, dev, gen, 0.01))
    else:
        g = S.torch_grads_lognormal(n, dev, gen)
    idx = sample_groups(ng, 4096, seed=G)
    idx_dev = torch.from_numpy(idx).to(dev)

    # the sampled groups before the step, as contiguous host arrays (G divides every offset)
    w0 = gather(w, idx_dev, G).numpy()
    g_bits = gather(g.view(torch.int16), idx_dev, G).numpy().view(np.uint16)
    def host(v):
        v = gather(v, idx_dev, G) if v.numel() == n else v.index_select(0, idx_dev).cpu()
        return (v.float() if v.dtype == torch.bfloat16 else v).numpy()

    st0 = {k: host(v) for k, v in st.items()}

    t = 5
    hp = coat.make_hparams(step=t, group_size=G, **HP, **flags)
    coat.coat_fp8_adamw_step(w, g, st["m_q"], st["m_scale"], st["m_k"], st["v_q"], st["v_scale"], st["v_k"], hp)
    torch.cuda.synchronize()

    w_g = gather(w, idx_dev, G).numpy()
    st_g = {k: host(v) for k, v in st.items()}
    # gradients are read-only
    assert np.array_equal(gather(g.view(torch.int16), idx_dev, G).numpy().view(np.uint16), g_bits)
    del w, g, st
    torch.cuda.empty_cache()

    w_r = w0.copy()
    st_r = {k: v.copy() for k, v in st0.items()}
    rh = ref.make_hparams(step=t, group_size=G, **HP, **flags)
    assert ref.fp8_adamw_step(w_r, g_bits, st_r["m_q"], st_r["m_scale"], st_r["m_k"],
                              st_r["v_q"], st_r["v_scale"], st_r["v_k"], rh) == 0
    stats = check_step(ref, "%s G=%d sampled" % (workload, G), w_g, st_g, w_r, st_r, st0, g_bits, G,
                       extra_w_tol=update_error_model(ref, st0, g_bits, G, t, **flags), **flags)
    assert np.any(w_g != w0) and np.any(st_g["m_q"] != st0["m_q"])
    print(workload, G, stats)
