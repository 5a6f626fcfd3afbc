"""The allocation-free backward entry point (dL/dY_k in the library's static device array) against
tac_conv_lif_backward, through the C ABI, on two calls in a row, the second with a smaller input."""
import gc

import numpy as np
import pytest
import torch

from paper_2603_13810_amd import api, synth
from parity_util import np_pack

pytestmark = pytest.mark.gpu
DEV = torch.device("cuda:0")


def _case(seed, T, B, Cin, Cout, H, W, mode, K, precision):
    r = np.random.Generator(np.random.PCG64(seed))
    s = (r.random((T, B, Cin, H, W)) < 0.2).astype(np.uint8)
    w = synth.kaiming_normal(seed, Cout, Cin) * np.float32(1.5)
    desc = api.make_desc(T, B, Cin, H, W, Cout, K=K, beta=0.9, theta=1.0, mode=mode, precision=precision)
    T_out, Ho, Wo = api.tac_out_shape(desc)
    sp, wd = torch.from_numpy(np_pack(s)).to(DEV), torch.from_numpy(w).to(DEV)
    vt = torch.empty((T_out, B, Cout, Ho, Wo), dtype=torch.float32, device=DEV)
    api.tac_conv_lif(desc, sp, api.tac_prepare_weights(desc, wd), None, None, None, vt)
    g_out = torch.from_numpy(r.standard_normal((T_out, B, Cout, Ho, Wo)).astype(np.float32)).to(DEV)
    kw = dict(surrogate=api.TAC_SG_ARCTAN, alpha=2.0, detach_reset=True)
    ref = api.tac_conv_lif_backward(desc, sp, wd, vt, g_out, **kw)
    # outputs of the allocation-free call, poisoned so that an element it does not write shows up
    gw = torch.full_like(ref["grad_w"], float("nan"))
    gb = torch.full_like(ref["grad_bias"], float("nan"))
    gi = torch.full_like(ref["grad_in"], float("nan"))
    torch.cuda.synchronize()
    gc.collect()                               # tensors of earlier tests must not be freed in between
    before = torch.cuda.memory_allocated()
    api.tac_conv_lif_backward_static(desc, sp, wd, vt, g_out, gw, gb, gi, **kw)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() <= before           # the binding allocated no tensor either
    # dL/dS has no sums over pixels: identical; dW and dbias are float atomics in both calls: equal up to the order of arrival
    assert torch.equal(gi, ref["grad_in"])
    for got, want in ((gw, ref["grad_w"]), (gb, ref["grad_bias"])):
        assert torch.isfinite(got).all()
        assert torch.allclose(got, want, rtol=1e-4, atol=1e-5 * float(want.abs().max()))
    assert float(ref["grad_w"].abs().max()) > 0 and float(ref["grad_in"].abs().max()) > 0


def test_static_scratch_backward_two_calls_in_a_row_the_second_smaller():
    _case(2101, 8, 3, 32, 128, 12, 32, api.TAC_COLLAPSE, 4, api.TAC_BF16)        # matrix-core gradients
    _case(2102, 4, 2, 32, 128, 6, 32, api.TAC_COLLAPSE, 2, api.TAC_BF16)         # smaller, same kernels
    _case(2103, 6, 2, 3, 10, 9, 20, api.TAC_PRESERVE, 2, api.TAC_FP32)           # vector kernels, smaller still


def test_static_scratch_rejects_what_does_not_fit():
    # dL/dY_k of this layer would take 16 * 64 * 128 * 64 * 64 * 4 bytes = 2 GiB
    desc = api.make_desc(16, 64, 128, 64, 64, 128, K=1, beta=0.9, theta=1.0, mode=api.TAC_PER_STEP, precision=api.TAC_BF16)
    one = torch.zeros(4, dtype=torch.float32, device=DEV)
    with pytest.raises(api.TacError) as e:
        api.tac_conv_lif_backward_static(desc, one, one, one, one, one, one, one)
    assert e.value.status == api.TAC_ERR_UNSUPPORTED


@pytest.mark.parametrize("shape", [(4, 2, 128, 32, 9, 32, api.TAC_COLLAPSE, 2, api.TAC_BF16),      # matrix-core gradients, wide tiles
                                   (6, 2, 3, 10, 9, 20, api.TAC_PRESERVE, 2, api.TAC_FP32)])        # vector kernels
def test_static_scratch_backward_recorded_into_a_graph(shape):
    # what the entry point is for: no allocation, memset or synchronisation inside the call, so it can be captured; the
    # graph is replayed several times, with eager work and synchronisations in between, every replay against the eager result
    T, B, Cin, Cout, H, W, mode, K, precision = shape
    r = np.random.Generator(np.random.PCG64(2200 + Cin))
    s = (r.random((T, B, Cin, H, W)) < 0.2).astype(np.uint8)
    w = synth.kaiming_normal(2201, Cout, Cin) * np.float32(1.5)
    desc = api.make_desc(T, B, Cin, H, W, Cout, K=K, beta=0.9, theta=1.0, mode=mode, precision=precision)
    T_out, Ho, Wo = api.tac_out_shape(desc)
    sp, wd = torch.from_numpy(np_pack(s)).to(DEV), torch.from_numpy(w).to(DEV)
    vt = torch.empty((T_out, B, Cout, Ho, Wo), dtype=torch.float32, device=DEV)
    api.tac_conv_lif(desc, sp, api.tac_prepare_weights(desc, wd), None, None, None, vt)
    g_out = torch.from_numpy(r.standard_normal((T_out, B, Cout, Ho, Wo)).astype(np.float32)).to(DEV)
    kw = dict(surrogate=api.TAC_SG_ARCTAN, alpha=2.0, detach_reset=True)
    ref = api.tac_conv_lif_backward(desc, sp, wd, vt, g_out, **kw)
    gw, gb, gi = torch.empty_like(ref["grad_w"]), torch.empty_like(ref["grad_bias"]), torch.empty_like(ref["grad_in"])
    api.tac_conv_lif_backward_static(desc, sp, wd, vt, g_out, gw, gb, gi, **kw)      # first use outside the capture
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.graph(graph, stream=side):
        api.tac_conv_lif_backward_static(desc, sp, wd, vt, g_out, gw, gb, gi, **kw)
    for rep in range(3):
        for t in (gw, gb, gi):
            t.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(gi, ref["grad_in"]), "replay %d" % rep
        for got, want in ((gw, ref["grad_w"]), (gb, ref["grad_bias"])):
            assert torch.allclose(got, want, rtol=1e-4, atol=1e-5 * float(want.abs().max())), "replay %d" % rep
        # another gradient in the same buffer: the graph reads it on the next replay
        keep = g_out.clone()
        g_out.mul_(-2.0)
        graph.replay()
        torch.cuda.synchronize()
        assert torch.allclose(gi, -2.0 * ref["grad_in"], rtol=1e-5, atol=1e-6 * float(ref["grad_in"].abs().max())), "replay %d, new gradient" % rep
        g_out.copy_(keep)
