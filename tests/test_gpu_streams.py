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
