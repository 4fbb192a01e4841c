"""GPU tests of how the entry points sit in HIP streams and graphs: they only enqueue on the
caller's stream, so they work on a non-default stream, and, as they allocate nothing and clear
nothing with memsets, they can be captured into a graph and replayed."""
import numpy as np
import pytest
import torch

import synth_inputs as S
from test_gpu_parity import HP

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def coat():
    import paper_2410_19313_amd as C
    assert torch.cuda.is_available(), "these tests need the GPU"
    C.lib()
    return C


def fresh(n, G, seed):
    dev = torch.device("cuda:0")
    w = torch.from_numpy(S.weights(n, seed)).to(dev)
    g = torch.from_numpy(S.grads_normal(n, seed, 1, G=G, outlier_frac=0.02).view(np.int16)).to(dev).view(torch.bfloat16)
    st = {k: torch.from_numpy(v).to(dev) for k, v in S.random_state(n, G, seed).items()}
    return w, g, st


def step(coat, w, g, st, G, t):
    coat.coat_fp8_adamw_step(w, g, st["m_q"], st["m_scale"], st["m_k"], st["v_q"], st["v_scale"], st["v_k"],
                             coat.make_hparams(step=t, group_size=G, **HP))


def same(a, b):
    return torch.equal(a.view(torch.uint8) if a.dtype == torch.uint8 else a.view(torch.int32),
                       b.view(torch.uint8) if b.dtype == torch.uint8 else b.view(torch.int32))


def test_step_on_a_side_stream_equals_default_stream(coat):
    n, G = 300 * 1024 + 517, 128
    w0, g, st0 = fresh(n, G, 1)
    w1, st1 = w0.clone(), {k: v.clone() for k, v in st0.items()}
    for t in (1, 2):
        step(coat, w0, g, st0, G, t)
    side = torch.cuda.Stream()                     # default priority
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        for t in (1, 2):
            step(coat, w1, g, st1, G, t)
    side.synchronize()
    torch.cuda.synchronize()
    assert same(w0, w1) and all(same(st0[k], st1[k]) for k in st0)


def test_graph_replays_match_eager(coat):
    """Capture step + activation quantizers (three kernels with a caller workspace) into one graph;
    replay it several times with eager work and synchronizations in between; every replay, started
    from the same restored state, must reproduce the eager results exactly."""
    n, G = 200 * 1024 + 33, 128
    w_init, g, st_init = fresh(n, G, 2)
    x = torch.from_numpy(S.activations(64 * 4096 + 100, 9).view(np.int16)).cuda().view(torch.bfloat16)
    # eager reference
    w_e, st_e = w_init.clone(), {k: v.clone() for k, v in st_init.items()}
    step(coat, w_e, g, st_e, G, 7)
    q_e, ts_e, ga_e, ta_e = coat.coat_act_quant_tensor(x, 16)
    qg_e, sg_e = coat.coat_act_quant_group(x, 16)
    torch.cuda.synchronize()
    # buffers the graph works on
    w, st = w_init.clone(), {k: v.clone() for k, v in st_init.items()}
    out_t = tuple(torch.empty_like(t) for t in (q_e, ts_e, ga_e, ta_e))
    out_g = (torch.empty_like(qg_e), torch.empty_like(sg_e))
    ws = coat.act_workspace("cuda")
    hp = coat.make_hparams(step=7, group_size=G, **HP)
    cap = torch.cuda.Stream()
    cap.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(cap):
        with torch.cuda.graph(graph, stream=cap):
            coat.coat_fp8_adamw_step(w, g, st["m_q"], st["m_scale"], st["m_k"], st["v_q"], st["v_scale"], st["v_k"], hp)
            coat.coat_act_quant_tensor(x, 16, out=out_t, workspace=ws)
            coat.coat_act_quant_group(x, 16, out=out_g)
    torch.cuda.synchronize()
    for rep in range(4):
        # restore the inputs the step overwrites, scribble over the outputs (eager work between replays)
        w.copy_(w_init)
        for k in st:
            st[k].copy_(st_init[k])
        for t in out_t + out_g:
            t.fill_(3)
        ws.fill_(1e30)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert same(w, w_e) and all(same(st[k], st_e[k]) for k in st), "replay %d: step differs" % rep
        assert same(out_t[0], q_e) and same(out_t[1], ts_e) and same(out_t[2], ga_e) and same(out_t[3], ta_e), rep
        assert same(out_g[0], qg_e) and same(out_g[1], sg_e), rep


def test_training_trajectory_tracks_fp32_adamw(coat):
    """The step in use, not in lock-step: 300 consecutive steps on a noisy quadratic whose curvatures
    spread over three decades inside every group, FP8 states (G = 128) against torch's fp32 AdamW fed
    the same noise.  With the dynamic range expansion the loss curve must never be more than 10 %
    above the fp32 one and must end within 2 % of it (the paper: nearly lossless); with the plain
    per-group quantizer the small second moments of such groups flush to zero and training goes
    wrong -- the under-used dynamic range that Sec. 4 sets out to fix.  (Measured: final ratio 1.003
    with expansion; without it the loss ends five orders of magnitude above the fp32 run.)"""
    n, G, steps = 256 * 1024, 128, 300
    dev = torch.device("cuda:0")
    hp = dict(lr=2e-3, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.01)
    gen = torch.Generator(device=dev)
    gen.manual_seed(0)
    target = torch.randn(n, device=dev, generator=gen) * 0.05
    curv = torch.exp(torch.randn(n, device=dev, generator=gen) * 1.5)

    def loss_and_grad(w, noise):
        d = w - target
        return 0.5 * float((curv * d * d).mean()), (curv * d + noise).to(torch.bfloat16)

    final = {}
    for expand in (True, False):
        gen.manual_seed(1)
        w_fp8 = torch.zeros(n, device=dev)
        w_ref = torch.zeros(n, device=dev, requires_grad=True)
        opt = torch.optim.AdamW([w_ref], lr=hp["lr"], betas=(hp["beta1"], hp["beta2"]), eps=hp["eps"],
                                weight_decay=hp["weight_decay"])
        st = S.torch_zero_state(n, G, dev)
        first = None
        for t in range(1, steps + 1):
            noise = torch.randn(n, device=dev, generator=gen) * 1e-3
            l_fp8, g_fp8 = loss_and_grad(w_fp8, noise)
            l_ref, g_ref = loss_and_grad(w_ref.detach(), noise)
            first = first or l_ref
            coat.coat_fp8_adamw_step(w_fp8, g_fp8, st["m_q"], st["m_scale"], st["m_k"], st["v_q"], st["v_scale"],
                                     st["v_k"], coat.make_hparams(step=t, group_size=G, expand=expand, **hp))
            w_ref.grad = g_ref.float()
            opt.step()
            if expand and t % 25 == 0:
                assert l_fp8 <= 1.10 * l_ref, "step %d: loss %.4g (FP8 states) against %.4g (fp32)" % (t, l_fp8, l_ref)
        final[expand] = (l_fp8, l_ref)
        assert l_ref < 1e-3 * first and torch.all(torch.isfinite(w_fp8))
    assert abs(final[True][0] / final[True][1] - 1.0) <= 0.02
    assert final[False][0] > 10.0 * final[True][0]


def test_one_captured_graph_replayed_across_steps(coat):
    """A training loop under a graph: the multi-tensor step is captured ONCE (with the step-dependent
    constants in a device block) and replayed for steps 1..5 with a changing learning rate, the host
    rewriting the 32-byte block and the gradients between replays.  Every step must equal the
    eager multi-tensor step with that step's hyper-parameters, bit for bit."""
    G = 128
    dev = torch.device("cuda:0")
    sizes = [70 * 1024 + 3, 4096, 129, 33 * 1024]

    def make():
        tens = []
        for i, n in enumerate(sizes):
            st = S.torch_zero_state(n, G, dev)
            d = dict(w=torch.from_numpy(S.weights(n, 40 + i)).to(dev), grad=torch.empty(n, dtype=torch.bfloat16, device=dev),
                     weight_decay=0.1 if i % 2 else 0.0)
            d.update(st)
            tens.append(d)
        return tens

    def set_grads(tens, t):
        for i, d in enumerate(tens):
            d["grad"].copy_(torch.from_numpy(S.grads_normal(sizes[i], 60 + i, t, G=G, outlier_frac=0.02).view(np.int16)).to(dev)
                            .view(torch.bfloat16))

    def hp_of(t):
        return coat.make_hparams(step=t, group_size=G, **{**HP, "lr": 3e-4 * (1.0 - 0.1 * t)})

    eager, graphed = make(), make()
    plan_e, plan_g = coat.MultiPlan(eager, G), coat.MultiPlan(graphed, G)
    consts = coat.step_consts_tensor(hp_of(1), dev)
    cap = torch.cuda.Stream()
    cap.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    set_grads(graphed, 1)
    snapshot = [{k: v.clone() for k, v in d.items() if torch.is_tensor(v)} for d in graphed]
    with torch.cuda.stream(cap):
        with torch.cuda.graph(graph, stream=cap):
            coat.coat_fp8_adamw_step_multi_consts(plan_g, hp_of(1), consts)
    torch.cuda.synchronize()
    for d, s in zip(graphed, snapshot):            # capture does not execute; make sure of the start state anyway
        for k, v in s.items():
            d[k].copy_(v)
    for t in range(1, 6):
        set_grads(eager, t)
        set_grads(graphed, t)
        coat.coat_fp8_adamw_step_multi(plan_e, hp_of(t))
        coat.step_consts_tensor(hp_of(t), dev, out=consts)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for i, (de, dg) in enumerate(zip(eager, graphed)):
            for k in ("w", "m_q", "m_scale", "m_k", "v_q", "v_scale", "v_k"):
                assert same(de[k], dg[k]), "step %d tensor %d: %s differs" % (t, i, k)
