"""coat_act_quant_tensor_static (the entry point that allocates nothing: its scratch is a static
device array of the library) against coat_act_quant_tensor (caller workspace), through the C ABI:
bit-identical outputs on two calls in a row, the second with a smaller input, so that what the
first call left in the shared scratch is seen not to leak into the second."""
import ctypes

import numpy as np
import pytest
import torch

import synth_inputs as S

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def coat():
    import paper_2410_19313_amd as C
    assert torch.cuda.is_available(), "these tests need the GPU"
    C.lib()
    return C


def run_both(coat, x_bits, G):
    dev = torch.device("cuda:0")
    n = x_bits.size
    ng = (n + G - 1) // G
    x = torch.from_numpy(x_bits.view(np.int16)).to(dev).view(torch.bfloat16)
    L = coat.lib()
    outs = []
    for static in (False, True):
        q = torch.full((n,), 0xAB, dtype=torch.uint8, device=dev)
        gamax = torch.full((ng,), -1.0, dtype=torch.float32, device=dev)
        tamax = torch.full((1,), -1.0, dtype=torch.float32, device=dev)
        tscale = torch.full((1,), -1.0, dtype=torch.float32, device=dev)
        stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
        if static:
            rc = L.coat_act_quant_tensor_static(x.data_ptr(), n, G, gamax.data_ptr(), tamax.data_ptr(), tscale.data_ptr(),
                                                q.data_ptr(), stream)
        else:
            ws = torch.full((coat.ACT_WORKSPACE_FLOATS,), 7.0, dtype=torch.float32, device=dev)
            rc = L.coat_act_quant_tensor(x.data_ptr(), n, G, gamax.data_ptr(), ws.data_ptr(), tamax.data_ptr(),
                                         tscale.data_ptr(), q.data_ptr(), stream)
        assert rc == 0, coat.strerror(rc)
        torch.cuda.synchronize()
        outs.append((q.cpu().numpy(), gamax.cpu().numpy(), tamax.cpu().numpy(), tscale.cpu().numpy()))
    return outs


def test_static_scratch_entry_matches_the_workspace_entry(coat, ref):
    G = 16
    # first call: large enough to use every slot of the scratch (one partial maximum per workgroup of
    # stage 1 plus the ragged tail's), with a big maximum; second call: a much smaller tensor (a few
    # slots) with a smaller maximum
    big = S.activations(5 * 1024 * 1024 + 1000 + 9, seed=31, hidden=4096)
    small = S.activations(5 * 1024 + 77, seed=32, hidden=512, channel_mult=1.0, spike_mult=1.0, sigma=0.01)
    for x_bits in (big, small):
        (q_w, ga_w, ta_w, ts_w), (q_s, ga_s, ta_s, ts_s) = run_both(coat, x_bits, G)
        assert np.array_equal(q_s, q_w) and np.array_equal(ga_s, ga_w)
        assert np.array_equal(ta_s, ta_w) and np.array_equal(ts_s, ts_w)
        # and both equal the oracle (bit-exact: every step is exact or one correctly rounded operation)
        q_r, ts_r, ga_r = ref.act_quant_tensor(x_bits, G)
        assert np.array_equal(q_s, q_r) and np.array_equal(ga_s, ga_r) and ts_s[0] == ts_r
    assert float(ta_s[0]) < 1.0          # the second maximum is the small tensor's own


def test_static_scratch_entry_argument_errors(coat):
    L = coat.lib()
    ok = ctypes.c_void_p(0x1000)
    assert L.coat_act_quant_tensor_static(ok, 1 << 47, 16, ok, ok, ok, ok, None) == -7          # beyond the size limit
    assert L.coat_act_quant_tensor_static(ok, 4096, 24, ok, ok, ok, ok, None) == -3             # group size
    assert L.coat_act_quant_tensor_static(None, 4096, 16, ok, ok, ok, ok, None) == -1           # NULL
    assert L.coat_act_quant_tensor_static(ctypes.c_void_p(0x1004), 4096, 16, ok, ok, ok, ok, None) == -2   # alignment
    assert L.coat_act_quant_tensor_static(ok, 0, 16, ok, ok, ok, ok, None) == 0                 # nothing to do
