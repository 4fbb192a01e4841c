"""GPU tests of the multi-tensor step: one launch over many tensors must equal one single-tensor
call per tensor BIT FOR BIT (it runs the same device code on the same inputs), and therefore
inherits that entry point's parity with the oracle; a direct oracle comparison is kept as well."""
import numpy as np
import pytest
import torch

import synth_inputs as S
from test_gpu_parity import HP, check_step, ref_step

pytestmark = pytest.mark.gpu

# sizes: empty, sub-group, exactly one chunk, one chunk + 1, several chunks + ragged tail, large
SIZES = [1, 0, 100, 1024, 1025, 4096, 5000, 70 * 1024 + 3, 127, 128, 129, 300 * 1024]
DECAY = [0.1, 0.0, 0.0, 0.1, 0.05, 0.0, 0.1, 0.1, 0.0, 0.3, 0.0, 0.1]


@pytest.fixture(scope="module")
def coat():
    import paper_2410_19313_amd as C
    assert torch.cuda.is_available(), "these tests need the GPU"
    C.lib()
    return C


def make_tensors(G, seed, with_bf16=()):
    """Host-side state of every tensor: (w, state dict, weight decay)."""
    out = []
    for i, n in enumerate(SIZES):
        w = S.weights(n, seed + i)
        st = S.zero_state(n, G)
        out.append(dict(w=w, st=st, wd=DECAY[i], bf16=i in with_bf16))
    return out


def to_device(host, bf16_scale=False, bf16_k=False):
    dev = []
    for h in host:
        n = h["w"].size
        d = dict(w=torch.from_numpy(h["w"].copy()).cuda(), grad=torch.empty(n, dtype=torch.bfloat16, device="cuda"),
                 weight_decay=h["wd"])
        for k, v in h["st"].items():
            d[k] = torch.from_numpy(v.copy()).cuda()
            if (bf16_scale and k.endswith("_scale")) or (bf16_k and k.endswith("_k")):
                d[k] = d[k].to(torch.bfloat16)
        if h["bf16"]:
            d["w_bf16"] = torch.full((n,), 7.0, dtype=torch.bfloat16, device="cuda")
        dev.append(d)
    return dev


def set_grads(dev, grads):
    for d, g in zip(dev, grads):
        d["grad"].copy_(torch.from_numpy(g.view(np.int16)).view(torch.bfloat16))


def single_steps(coat, dev, G, t, **flags):
    for d in dev:
        hp = coat.make_hparams(step=t, group_size=G, **{**HP, "weight_decay": d["weight_decay"]}, **flags)
        args = (d["grad"], d["m_q"], d["m_scale"], d["m_k"], d["v_q"], d["v_scale"], d["v_k"], hp)
        if "w_bf16" in d:
            coat.coat_fp8_adamw_step_bf16w(d["w"], d["w_bf16"], *args)
        else:
            coat.coat_fp8_adamw_step(d["w"], *args)


KEYS = ("w", "m_q", "m_scale", "m_k", "v_q", "v_scale", "v_k", "w_bf16")


def raw(t):
    """The tensor's bytes (bit-for-bit comparison, NaN-safe)."""
    if t.numel() == 0:
        return b""
    return t.detach().reshape(-1).clone().view(torch.uint8).cpu().numpy().tobytes()


@pytest.mark.parametrize("G,flags", [(128, {}), (32, {}), (512, {}), (64, dict(m_e5m2=True, v_plain=True)),
                                     (128, dict(expand=False)), (128, dict(bf16_scale=True)),
                                     (32, dict(bf16_scale=True, bf16_k=True)), (512, dict(bf16_k=True)),
                                     (128, dict(precise_dq=True)), (64, dict(precise_dq=True, bf16_scale=True))])
def test_multi_equals_one_call_per_tensor(coat, G, flags):
    host = make_tensors(G, seed=11, with_bf16=(3, 7, 8))
    a = to_device(host, flags.get("bf16_scale", False), flags.get("bf16_k", False))
    b = to_device(host, flags.get("bf16_scale", False), flags.get("bf16_k", False))
    plan = coat.MultiPlan(a, G)
    for t in range(1, 4):
        grads = [S.grads_normal(h["w"].size, 50 + i, t, G=G) if i % 2 else S.grads_lognormal(h["w"].size, 50 + i, t)
                 for i, h in enumerate(host)]
        set_grads(a, grads)
        set_grads(b, grads)
        # hp.weight_decay is ignored by the multi-tensor step: give it a value no tensor uses
        coat.coat_fp8_adamw_step_multi(plan, coat.make_hparams(step=t, group_size=G, **{**HP, "weight_decay": 9.0}, **flags))
        single_steps(coat, b, G, t, **flags)
        torch.cuda.synchronize()
        for i, (da, db) in enumerate(zip(a, b)):
            for k in KEYS:
                if k in da:
                    assert raw(da[k]) == raw(db[k]), \
                        "G=%d step %d tensor %d (n=%d): %s differs" % (G, t, i, SIZES[i], k)


def shard_views(coat, dev, G, world):
    """Every tensor cut into `world` contiguous shards at multiples of G (coat_shard_range), as views
    of the same device memory: what the ranks of a ZeRO-style partition would each hand to the step."""
    out = []
    for d in dev:
        n = d["w"].numel()
        covered = 0
        for rank in range(world):
            b, e = coat.coat_shard_range(n, G, rank, world)
            assert b == covered and (b % (2 * G) == 0 or b == n) and (e % (2 * G) == 0 or e == n)
            covered = e
            gb, ge = (b // G, (e + G - 1) // G) if e > b else (0, 0)
            v = dict(weight_decay=d["weight_decay"])
            for k in ("w", "grad", "m_q", "v_q", "w_bf16"):
                if k in d:
                    v[k] = d[k][b:e]
            for k in ("m_scale", "m_k", "v_scale", "v_k"):
                v[k] = d[k][gb:ge]
            out.append(v)
        assert covered == n
    return out


@pytest.mark.parametrize("world", [2, 3, 8])
@pytest.mark.parametrize("G,bf16_scale,bf16_k", [(32, False, False), (128, False, False), (512, False, False),
                                                 (64, True, False), (32, True, True)])
def test_sharded_plan_equals_unsharded(coat, G, bf16_scale, bf16_k, world):
    """The optimizer state partitioned over `world` ranks (Sec. 2 places this step next to ZeRO-style
    sharding): all shards of all tensors as entries of ONE plan, one launch, against the unsharded
    plan, bit for bit, over three steps.  Groups never straddle a cut, so nothing else is acceptable."""
    host = make_tensors(G, seed=31, with_bf16=(4, 7))
    a, b = to_device(host, bf16_scale, bf16_k), to_device(host, bf16_scale, bf16_k)
    whole = coat.MultiPlan(a, G)
    shards = shard_views(coat, b, G, world)
    assert len(shards) == world * len(SIZES)
    cut = coat.MultiPlan(shards, G)
    for t in (1, 2, 3):
        grads = [S.grads_lognormal(h["w"].size, 90 + i, t) if i % 3 == 0 else S.grads_normal(h["w"].size, 90 + i, t, G=G)
                 for i, h in enumerate(host)]
        set_grads(a, grads)
        set_grads(b, grads)
        hp = coat.make_hparams(step=t, group_size=G, bf16_scale=bf16_scale, bf16_k=bf16_k, **HP)
        coat.coat_fp8_adamw_step_multi(whole, hp)
        coat.coat_fp8_adamw_step_multi(cut, hp)
        torch.cuda.synchronize()
        for i, (da, db) in enumerate(zip(a, b)):
            for k in KEYS:
                if k in da:
                    assert raw(da[k]) == raw(db[k]), "G=%d world=%d step %d tensor %d (n=%d): %s differs" % (
                        G, world, t, i, SIZES[i], k)


def test_multi_against_oracle(coat, ref):
    """Three lock-step steps from the zero state (both sides restart every step from the oracle's
    state), every tensor checked against the oracle with the rules of the single-tensor parity tests."""
    G = 128
    host = make_tensors(G, seed=23)
    for t in (1, 2, 3):
        dev = to_device(host)
        plan = coat.MultiPlan(dev, G)
        grads = [S.grads_normal(h["w"].size, 70 + i, t, G=G, outlier_frac=0.02) for i, h in enumerate(host)]
        set_grads(dev, grads)
        coat.coat_fp8_adamw_step_multi(plan, coat.make_hparams(step=t, group_size=G, **HP))
        torch.cuda.synchronize()
        for i, (h, d, g) in enumerate(zip(host, dev, grads)):
            n = h["w"].size
            if n == 0:
                continue
            w_r, st_r = ref_step(ref, h["w"], g, h["st"], G, t, weight_decay=h["wd"])
            st_g = {k: d[k].cpu().numpy() for k in h["st"]}
            check_step(ref, "multi tensor %d n=%d step %d" % (i, n, t), d["w"].cpu().numpy(), st_g, w_r, st_r, h["st"],
                       g, G, weight_decay=h["wd"])
            h["w"], h["st"] = w_r, st_r


def test_plan_survives_many_steps_and_only_touches_its_tensors(coat):
    """Guard bytes around every buffer stay intact, and tensors outside the plan are not touched."""
    G = 128
    sizes = [1000, 3 * 1024 + 5, 64]
    pad = 256
    bufs = []
    for i, n in enumerate(sizes):
        ng = (n + G - 1) // G
        def guarded(numel, dtype, fill):
            t = torch.full((numel + 2 * pad,), fill, dtype=dtype, device="cuda")
            return t, t[pad: pad + numel]
        d = {}
        raw = {}
        for k, numel, dtype, fill in (("w", n, torch.float32, 3.0), ("grad", n, torch.bfloat16, 5.0), ("m_q", n, torch.uint8, 0x55),
                                      ("m_scale", ng, torch.float32, 9.0), ("m_k", ng, torch.float32, 9.0),
                                      ("v_q", n, torch.uint8, 0x55), ("v_scale", ng, torch.float32, 9.0),
                                      ("v_k", ng, torch.float32, 9.0), ("w_bf16", n, torch.bfloat16, 5.0)):
            raw[k], d[k] = guarded(numel, dtype, fill)
        d["w"].copy_(torch.from_numpy(S.weights(n, i)))
        d["grad"].copy_(torch.from_numpy(S.grads_lognormal(n, i, 1).view(np.int16)).view(torch.bfloat16))
        for k in ("m_q", "v_q"):
            d[k].zero_()
        for k in ("m_scale", "v_scale"):
            d[k].zero_()
        for k in ("m_k", "v_k"):
            d[k].fill_(1.0)
        d["weight_decay"] = 0.1
        bufs.append((raw, d))
    plan = coat.MultiPlan([d for _, d in bufs], G)
    for t in range(1, 6):
        coat.coat_fp8_adamw_step_multi(plan, coat.make_hparams(step=t, group_size=G, **HP))
    torch.cuda.synchronize()
    fills = dict(w=3.0, grad=5.0, m_q=0x55, m_scale=9.0, m_k=9.0, v_q=0x55, v_scale=9.0, v_k=9.0, w_bf16=5.0)
    for raw, d in bufs:
        for k, t in raw.items():
            assert torch.all(t[:pad] == fills[k]) and torch.all(t[-pad:] == fills[k]), "guard bytes of %s changed" % k
        assert torch.all(torch.isfinite(d["w"])) and torch.all(d["m_scale"] > 0) and torch.all(d["v_scale"] > 0)


@pytest.mark.parametrize("workload", ["cfg2", "cfg3"])
def test_full_size_multi_equals_flat(coat, workload):
    """The bench's --multi configuration: the workload's weight matrices as separate tensors carved
    out of one flat buffer, stepped by one multi-tensor launch, must equal the flat single-tensor
    step bit for bit (two steps from the zero state)."""
    dev = torch.device("cuda:0")
    G = 128
    sizes = [r * c for r, c in S.workload_shapes(workload)]
    n = sum(sizes)
    free, _ = torch.cuda.mem_get_info()
    if free < n * 18 + (1 << 31):
        pytest.fail("needs %.0f GB of device memory, %.0f GB free" % (n * 18 / 1e9, free / 1e9))
    gen = S.torch_generator(dev, 3)
    w = S.torch_weights(n, dev, gen)
    g = S.torch_grads_normal(n, dev, gen, G=G, outlier_mask=S.torch_outlier_group_mask(n // G, dev, gen, 0.01))
    st = S.torch_zero_state(n, G, dev)
    w2, st2 = w.clone(), {k: v.clone() for k, v in st.items()}
    tens, off = [], 0
    for x in sizes:
        d = dict(w=w2[off:off + x], grad=g[off:off + x], weight_decay=HP["weight_decay"])
        for k in ("m_q", "v_q"):
            d[k] = st2[k][off:off + x]
        for k in ("m_scale", "m_k", "v_scale", "v_k"):
            d[k] = st2[k][off // G:(off + x) // G]
        tens.append(d)
        off += x
    plan = coat.MultiPlan(tens, G)
    for t in (1, 2):
        hp = coat.make_hparams(step=t, group_size=G, **HP)
        coat.coat_fp8_adamw_step(w, g, st["m_q"], st["m_scale"], st["m_k"], st["v_q"], st["v_scale"], st["v_k"], hp)
        coat.coat_fp8_adamw_step_multi(plan, hp)
        torch.cuda.synchronize()
        assert torch.equal(w.view(torch.int32), w2.view(torch.int32)), "%s step %d: w differs" % (workload, t)
        for k in st:
            a, b = st[k], st2[k]
            if a.dtype != torch.uint8:
                a, b = a.view(torch.int32), b.view(torch.int32)
            assert torch.equal(a, b), "%s step %d: %s differs" % (workload, t, k)
