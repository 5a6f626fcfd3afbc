"""Backward pass (surrogate-gradient BPTT of one conv-LIF layer, Sec. 5.1 "Training") through the C ABI against the
oracle: same inputs on both sides, the oracle on its own membranes in double, the library on the fp32 membranes its
forward pass recorded."""
import numpy as np
import pytest
import torch

import oracle
from paper_2603_13810_amd import api, synth
from gpu_util import ORACLE_MODE
from parity_util import np_pack

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
TOL = 1e-4          # relative to the largest magnitude of the tensor: fp32 sums of up to ~1e5 terms, atomics in any order


def _rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


def _close(name, got, ref, tol=TOL):
    scale = max(np.abs(ref).max(), 1e-30)
    err = np.abs(got - ref).max() / scale
    assert err <= tol, "%s: max error %.3g of the largest magnitude %.3g" % (name, err, scale)
    return err


# (Cin, Cout, H, W, stride)
SHAPES = [(3, 5, 7, 9, 1), (16, 24, 12, 33, 2), (2, 8, 20, 100, 1), (8, 16, 17, 40, 2)]
# (mode, K, T): whole groups, shorter last groups, a group longer than the sequence
TIMES = [(api.TAC_PER_STEP, 1, 5), (api.TAC_COLLAPSE, 2, 6), (api.TAC_COLLAPSE, 4, 7), (api.TAC_PRESERVE, 2, 6),
         (api.TAC_PRESERVE, 4, 10), (api.TAC_COLLAPSE, 8, 3)]
SURR = [(api.TAC_SG_FAST_SIGMOID, 25.0, False), (api.TAC_SG_ARCTAN, 2.0, True)]


@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("mode,K,T", TIMES)
@pytest.mark.parametrize("surrogate,alpha,detach", SURR)
def test_backward_against_the_oracle(shape, mode, K, T, surrogate, alpha, detach):
    Cin, Cout, H, W, stride = shape
    B = 3
    r = _rng(1200 + Cin + Cout + H + W + K + T)
    s = (r.random((T, B, Cin, H, W)) < 0.3).astype(np.uint8)
    w = synth.kaiming_normal(41, Cout, Cin) * np.float32(1.5)
    bias = (r.standard_normal(Cout) * 0.1).astype(np.float32)
    beta, theta = 0.9, 1.0
    desc = api.make_desc(T, B, Cin, H, W, Cout, K=K, beta=beta, theta=theta, mode=mode, stride=stride)
    T_out, Ho, Wo = api.tac_out_shape(desc)
    g_out = r.standard_normal((T_out, B, Cout, Ho, Wo)).astype(np.float32)
    # forward on the GPU, recording the membranes
    sp = torch.from_numpy(np_pack(s)).to(DEV)
    wd = torch.from_numpy(w).to(DEV)
    v = torch.zeros((B, Cout, Ho, Wo), dtype=torch.float32, device=DEV)
    vt = torch.empty((T_out, B, Cout, Ho, Wo), dtype=torch.float32, device=DEV)
    api.tac_conv_lif(desc, sp, api.tac_prepare_weights(desc, wd), torch.from_numpy(bias).to(DEV), v, None, vt)
    got = api.tac_conv_lif_backward(desc, sp, wd, vt, torch.from_numpy(g_out).to(DEV), surrogate=surrogate, alpha=alpha,
                                    detach_reset=detach)
    torch.cuda.synchronize()
    # the oracle, forward and backward, on the same host inputs
    kw = dict(K=K, beta=float(np.float32(beta)), theta=theta, mode=ORACLE_MODE[mode], stride=stride)
    out, v_pre, _ = oracle.conv_lif(s, w.astype(np.float64), bias.astype(np.float64), **kw)
    ref = oracle.conv_lif_backward(s, w.astype(np.float64), v_pre, g_out.astype(np.float64), surrogate=surrogate, alpha=alpha,
                                   detach_reset=detach, **kw)
    assert out.sum() > 0
    errs = [_close("dL/dY", got["grad_y"].cpu().numpy(), ref["dY"]), _close("dW", got["grad_w"].cpu().numpy(), ref["dW"]),
            _close("dbias", got["grad_bias"].cpu().numpy(), ref["dbias"]), _close("dL/dS", got["grad_in"].cpu().numpy(), ref["g_in"])]
    print("backward", shape, api.MODE_NAMES[mode], "K=%d T=%d" % (K, T), "max errors dY %.1e dW %.1e dbias %.1e dS %.1e" % tuple(errs))


def test_backward_first_layer_skips_the_input_gradient_and_is_repeatable_up_to_rounding():
    r = _rng(1300)
    s = (r.random((8, 2, 2, 16, 48)) < 0.3).astype(np.uint8)
    w = synth.kaiming_normal(42, 12, 2)
    desc = api.make_desc(8, 2, 2, 16, 48, 12, K=4, beta=0.5, theta=1.0, mode=api.TAC_PRESERVE, stride=2)
    T_out, Ho, Wo = api.tac_out_shape(desc)
    sp, wd = torch.from_numpy(np_pack(s)).to(DEV), torch.from_numpy(w).to(DEV)
    vt = torch.empty((T_out, 2, 12, Ho, Wo), dtype=torch.float32, device=DEV)
    api.tac_conv_lif(desc, sp, api.tac_prepare_weights(desc, wd), None, None, None, vt)
    g = torch.from_numpy(r.standard_normal((T_out, 2, 12, Ho, Wo)).astype(np.float32)).to(DEV)
    a = api.tac_conv_lif_backward(desc, sp, wd, vt, g, surrogate=api.TAC_SG_ARCTAN, alpha=2.0, detach_reset=True, want_input_grad=False)
    b = api.tac_conv_lif_backward(desc, sp, wd, vt, g, surrogate=api.TAC_SG_ARCTAN, alpha=2.0, detach_reset=True, want_input_grad=False)
    torch.cuda.synchronize()
    assert a["grad_in"] is None
    assert torch.equal(a["grad_y"], b["grad_y"])
    assert torch.allclose(a["grad_w"], b["grad_w"], rtol=1e-4, atol=1e-5 * float(a["grad_w"].abs().max()))


# weight gradients on the matrix cores (bf16 layers; Cin a multiple of 32, Cout of 128, width 16/32/64/128, stride 1)
# (Cin, Cout, H, W)
MFMA_SHAPES = [(32, 128, 12, 32), (64, 128, 9, 64), (32, 256, 20, 16), (32, 128, 5, 128), (32, 64, 15, 32),
               # input gradient on the wide tiles (Cin a multiple of 128): rows that do not fill the last tile, a Cout that is
               # only a multiple of 16 (its weight gradient then runs on the vector kernel), two tiles of input channels
               (128, 128, 9, 64), (128, 48, 11, 32), (256, 128, 5, 32)]
TOL_BF16 = 2e-2     # the bar of the bf16 path; dY and A_k enter the matrix cores rounded to bf16


@pytest.mark.parametrize("shape", MFMA_SHAPES)
@pytest.mark.parametrize("mode,K,T", [(api.TAC_PER_STEP, 1, 4), (api.TAC_COLLAPSE, 4, 8), (api.TAC_COLLAPSE, 4, 7), (api.TAC_PRESERVE, 2, 6),
                                      (api.TAC_COLLAPSE, 16, 16), (api.TAC_COLLAPSE, 8, 19), (api.TAC_PRESERVE, 8, 13)])
def test_backward_bf16_layer_weight_gradient_on_the_matrix_cores(shape, mode, K, T):
    from gpu_util import bf16_round_np
    Cin, Cout, H, W = shape
    B = 3
    r = _rng(1400 + Cin + Cout + H + W + K + T)
    s = (r.random((T, B, Cin, H, W)) < 0.15).astype(np.uint8)
    w = synth.kaiming_normal(43, Cout, Cin) * np.float32(1.5)
    bias = (r.standard_normal(Cout) * 0.1).astype(np.float32)
    beta, theta = 0.9, 1.0
    desc = api.make_desc(T, B, Cin, H, W, Cout, K=K, beta=beta, theta=theta, mode=mode, precision=api.TAC_BF16)
    T_out, Ho, Wo = api.tac_out_shape(desc)
    g_out = r.standard_normal((T_out, B, Cout, Ho, Wo)).astype(np.float32)
    sp, wd = torch.from_numpy(np_pack(s)).to(DEV), torch.from_numpy(w).to(DEV)
    v = torch.zeros((B, Cout, Ho, Wo), dtype=torch.float32, device=DEV)
    vt = torch.empty((T_out, B, Cout, Ho, Wo), dtype=torch.float32, device=DEV)
    api.tac_conv_lif(desc, sp, api.tac_prepare_weights(desc, wd), torch.from_numpy(bias).to(DEV), v, None, vt)
    torch.cuda.synchronize()
    # oracle: the bf16 forward pass (W and A_k rounded), then the backward pass with the rounded A_k in dW
    kw = dict(K=K, beta=float(np.float32(beta)), theta=theta, mode=ORACLE_MODE[mode])
    out, v_pre, _ = oracle.conv_lif(s, bf16_round_np(w).astype(np.float64), bias.astype(np.float64), round_a_bf16=True, **kw)
    # forward check, on its own: a membrane within rounding of the threshold may spike on one side only (every later
    # membrane of that neuron then differs by theta); such a flip must be that close to the threshold, and everywhere
    # before it the recorded membranes are the oracle's
    v_gpu = vt.cpu().numpy().astype(np.float64)
    flips = (v_gpu >= theta) != (v_pre >= theta)
    first = flips & (np.cumsum(flips, axis=0) == 1)
    assert flips.sum() <= 4 and (np.abs(v_pre[first] - theta) < 1e-3).all(), "spikes differ away from the threshold"
    clean = np.cumsum(flips, axis=0) == 0
    assert (np.abs(v_gpu - v_pre)[clean] <= 1e-3 * np.maximum(np.abs(v_pre[clean]), theta)).all()
    # backward check: both sides start from the ORACLE's membranes (uploaded as the v_trace argument), so that nothing
    # the library computed enters the oracle and a forward flip cannot leak into the gradient comparison
    vt_ref = torch.from_numpy(v_pre.astype(np.float32)).to(DEV)
    got = api.tac_conv_lif_backward(desc, sp, wd, vt_ref, torch.from_numpy(g_out).to(DEV), surrogate=api.TAC_SG_ARCTAN, alpha=2.0,
                                    detach_reset=True)
    torch.cuda.synchronize()
    ref = oracle.conv_lif_backward(s, w.astype(np.float64), v_pre, g_out.astype(np.float64),
                                   surrogate=oracle.ARCTAN, alpha=2.0, detach_reset=True, round_a_bf16=True, **kw)
    assert out.sum() > 0

    def err(name, a, b, tol):
        e = np.abs(a - b).max() / np.abs(b).max()
        assert e <= tol, "%s: %.3g" % (name, e)
        return e
    e = [err("dL/dY", got["grad_y"].cpu().numpy(), ref["dY"], 1e-3), err("dW", got["grad_w"].cpu().numpy(), ref["dW"], TOL_BF16),
         err("dbias", got["grad_bias"].cpu().numpy(), ref["dbias"], 1e-3), err("dL/dS", got["grad_in"].cpu().numpy(), ref["g_in"], TOL_BF16)]
    print("backward bf16", shape, api.MODE_NAMES[mode], "K=%d T=%d" % (K, T), "errors dY %.1e dW %.1e dbias %.1e dS %.1e" % tuple(e))


@pytest.mark.parametrize("modes", [[(api.TAC_COLLAPSE, 2), (api.TAC_COLLAPSE, 2), (api.TAC_COLLAPSE, 2)],
                                   [(api.TAC_PRESERVE, 4), (api.TAC_COLLAPSE, 3), (api.TAC_PER_STEP, 1)]])
def test_backward_through_a_stack(modes):
    # forward through the stack call, backward through tac_stack_backward; the oracle runs the same chain layer by
    # layer (forward on its own spikes, backward handing dL/dS of a layer to the layer before as dL/ds)
    r = _rng(1500 + len(modes) + modes[0][1])
    T, B, H, W = 8, 2, 10, 12
    chans = [3, 6, 8, 5]
    s = (r.random((T, B, chans[0], H, W)) < 0.4).astype(np.uint8)
    layers, ws, host = [], [], []
    Tl = T
    for l, (mode, K) in enumerate(modes):
        desc = api.make_desc(Tl, B, chans[l], H, W, chans[l + 1], K=K, beta=0.9, theta=1.0, mode=mode)
        w = (synth.kaiming_normal(50 + l, chans[l + 1], chans[l]) * np.float32(2.0)).astype(np.float32)
        wd = torch.from_numpy(w).to(DEV)
        T_out, Ho, Wo = api.tac_out_shape(desc)
        layers.append(dict(desc=desc, w_prepared=api.tac_prepare_weights(desc, wd),
                           v_inout=torch.zeros((B, chans[l + 1], Ho, Wo), dtype=torch.float32, device=DEV),
                           v_trace=torch.empty((T_out, B, chans[l + 1], Ho, Wo), dtype=torch.float32, device=DEV)))
        ws.append(wd)
        host.append((w, mode, K))
        Tl = T_out
    stack, outs = api.make_stack(layers)
    sp = torch.from_numpy(np_pack(s)).to(DEV)
    api.tac_stack_forward(stack, sp)
    g_last = r.standard_normal(tuple(layers[-1]["v_trace"].shape)).astype(np.float32)
    got = api.tac_stack_backward(stack, ws, sp, torch.from_numpy(g_last).to(DEV), surrogate=api.TAC_SG_ARCTAN, alpha=2.0,
                                 detach_reset=True, first_layer_input_grad=True)
    torch.cuda.synchronize()
    # oracle chain
    x, fwd = s, []
    for (w, mode, K) in host:
        out, v_pre, _ = oracle.conv_lif(x, w.astype(np.float64), K=K, beta=float(np.float32(0.9)), theta=1.0, mode=ORACLE_MODE[mode])
        fwd.append((x, v_pre))
        x = out
    from parity_util import np_unpack
    assert np.array_equal(np_unpack(outs[-1].cpu().numpy(), W), x) and x.sum() > 0      # same spikes on both sides
    g = g_last.astype(np.float64)
    for l in range(len(host) - 1, -1, -1):
        w, mode, K = host[l]
        ref = oracle.conv_lif_backward(fwd[l][0], w.astype(np.float64), fwd[l][1], g, K=K, beta=float(np.float32(0.9)), theta=1.0,
                                       mode=ORACLE_MODE[mode], surrogate=oracle.ARCTAN, alpha=2.0, detach_reset=True)
        _close("layer %d dW" % l, got[l]["grad_w"].cpu().numpy(), ref["dW"])
        _close("layer %d dbias" % l, got[l]["grad_bias"].cpu().numpy(), ref["dbias"])
        _close("layer %d dL/dS" % l, got[l]["grad_in"].cpu().numpy(), ref["g_in"])
        g = ref["g_in"]
    # the same pass with the input gradients handed over once per group of frames where a layer groups them: the same
    # products are formed on the reading side instead of the writing side, so dL/dY_k agrees bit for bit
    grp = api.tac_stack_backward(stack, ws, sp, torch.from_numpy(g_last).to(DEV), surrogate=api.TAC_SG_ARCTAN, alpha=2.0,
                                 detach_reset=True, first_layer_input_grad=True, grad_in_per_group=True)
    torch.cuda.synchronize()
    for l, (w, mode, K) in enumerate(host):
        d = layers[l]["desc"]
        grouped = l > 0 and mode != api.TAC_PER_STEP and K > 1
        assert grp[l]["grad_in"].shape[0] == (-(-d.T // min(K, d.T)) if grouped else d.T), l
        assert torch.equal(grp[l]["grad_y"], got[l]["grad_y"]), l
        assert torch.allclose(grp[l]["grad_w"], got[l]["grad_w"], rtol=1e-4, atol=1e-5 * float(got[l]["grad_w"].abs().max())), l


@pytest.mark.parametrize("mode,K,T", [(api.TAC_PER_STEP, 1, 4), (api.TAC_COLLAPSE, 4, 8), (api.TAC_PRESERVE, 2, 7)])
@pytest.mark.parametrize("precision", [api.TAC_FP32, api.TAC_BF16])
def test_backward_of_a_first_layer_on_real_valued_frames(mode, K, T, precision):
    # the continuous-valued first layer (Sec. 4.2): A_k is a weighted sum of real frames; its weight gradient uses them
    from gpu_util import bf16_round_np
    r = _rng(1600 + K + T)
    B, Cin, Cout, H, W, stride = 3, 2, 24, 12, 40, 2
    x = (r.random((T, B, Cin, H, W)) * (r.random((T, B, Cin, H, W)) < 0.4)).astype(np.float32)
    w = synth.kaiming_normal(60, Cout, Cin) * np.float32(2.0)
    desc = api.make_desc(T, B, Cin, H, W, Cout, K=K, beta=0.5, theta=1.0, mode=mode, stride=stride, precision=precision,
                         in_format=api.TAC_IN_F32)
    T_out, Ho, Wo = api.tac_out_shape(desc)
    g_out = r.standard_normal((T_out, B, Cout, Ho, Wo)).astype(np.float32)
    xd, wd = torch.from_numpy(x).to(DEV), torch.from_numpy(w).to(DEV)
    v = torch.zeros((B, Cout, Ho, Wo), dtype=torch.float32, device=DEV)
    vt = torch.empty((T_out, B, Cout, Ho, Wo), dtype=torch.float32, device=DEV)
    api.tac_conv_lif(desc, xd, api.tac_prepare_weights(desc, wd), None, v, None, vt)
    got = api.tac_conv_lif_backward(desc, xd, wd, vt, torch.from_numpy(g_out).to(DEV), surrogate=api.TAC_SG_ARCTAN, alpha=2.0,
                                    detach_reset=True)
    torch.cuda.synchronize()
    q = precision == api.TAC_BF16
    kw = dict(K=K, beta=0.5, theta=1.0, mode=ORACLE_MODE[mode], stride=stride)
    out, v_pre, _ = oracle.conv_lif(x.astype(np.float64), (bf16_round_np(w) if q else w).astype(np.float64), round_a_bf16=q, **kw)
    ref = oracle.conv_lif_backward(x.astype(np.float64), w.astype(np.float64), v_pre, g_out.astype(np.float64), surrogate=oracle.ARCTAN,
                                   alpha=2.0, detach_reset=True, **kw)
    assert out.sum() > 0
    _close("dL/dY", got["grad_y"].cpu().numpy(), ref["dY"])
    _close("dW", got["grad_w"].cpu().numpy(), ref["dW"])
    _close("dL/dx", got["grad_in"].cpu().numpy(), ref["g_in"])


@pytest.mark.parametrize("pool", [True, "max"])
@pytest.mark.parametrize("mode,K,T", [(api.TAC_PER_STEP, 1, 4), (api.TAC_COLLAPSE, 4, 8), (api.TAC_PRESERVE, 2, 7)])
@pytest.mark.parametrize("precision", [api.TAC_FP32, api.TAC_BF16])
def test_backward_through_the_pool_on_load(pool, mode, K, T, precision):
    # Pool(2) between the convolutions of the rate-coded network, MaxPool(2) behind every LIF layer of the event-data
    # network (Sec. 5.1): the gradient of the unpooled frames
    from gpu_util import bf16_round_np
    r = _rng(1700 + K + T + (pool == "max"))
    B, Cin, Cout, H, W = 2, 8, 16, 7, 20
    s = (r.random((T, B, Cin, 2 * H, 2 * W)) < 0.25).astype(np.uint8)
    w = synth.kaiming_normal(61, Cout, Cin) * np.float32(1.5)
    fmt = api.TAC_IN_BITS_MAXPOOL2 if pool == "max" else api.TAC_IN_BITS_POOL2
    desc = api.make_desc(T, B, Cin, H, W, Cout, K=K, beta=0.9, theta=1.0, mode=mode, precision=precision, in_format=fmt)
    T_out, Ho, Wo = api.tac_out_shape(desc)
    g_out = r.standard_normal((T_out, B, Cout, Ho, Wo)).astype(np.float32)
    sp, wd = torch.from_numpy(np_pack(s)).to(DEV), torch.from_numpy(w).to(DEV)
    v = torch.zeros((B, Cout, Ho, Wo), dtype=torch.float32, device=DEV)
    vt = torch.empty((T_out, B, Cout, Ho, Wo), dtype=torch.float32, device=DEV)
    api.tac_conv_lif(desc, sp, api.tac_prepare_weights(desc, wd), None, v, None, vt)
    got = api.tac_conv_lif_backward(desc, sp, wd, vt, torch.from_numpy(g_out).to(DEV), surrogate=api.TAC_SG_FAST_SIGMOID, alpha=25.0)
    torch.cuda.synchronize()
    q = precision == api.TAC_BF16
    kw = dict(K=K, beta=float(np.float32(0.9)), theta=1.0, mode=ORACLE_MODE[mode], pool2=pool)
    out, v_pre, _ = oracle.conv_lif(s, (bf16_round_np(w) if q else w).astype(np.float64), round_a_bf16=q, **kw)
    ref = oracle.conv_lif_backward(s, w.astype(np.float64), v_pre, g_out.astype(np.float64), surrogate=oracle.FAST_SIGMOID, alpha=25.0, **kw)
    assert out.sum() > 0 and got["grad_in"].shape == s.shape
    _close("dL/dY", got["grad_y"].cpu().numpy(), ref["dY"])
    _close("dW", got["grad_w"].cpu().numpy(), ref["dW"])
    _close("dL/dS", got["grad_in"].cpu().numpy(), ref["g_in"])


@pytest.mark.parametrize("pool", [True, "max"])
def test_backward_through_a_stack_with_a_pool_between_the_layers(pool):
    r = _rng(1800 + (pool == "max"))
    T, B, H, W = 8, 2, 12, 16
    s = (r.random((T, B, 3, H, W)) < 0.4).astype(np.uint8)
    fmt = api.TAC_IN_BITS_MAXPOOL2 if pool == "max" else api.TAC_IN_BITS_POOL2
    spec = [(3, 6, H, W, api.TAC_IN_BITS, api.TAC_PRESERVE, 2, False), (6, 8, H // 2, W // 2, fmt, api.TAC_COLLAPSE, 4, pool)]
    layers, ws, host = [], [], []
    for l, (ci, co, h, w_, f, mode, K, pl) in enumerate(spec):
        desc = api.make_desc(T, B, ci, h, w_, co, K=K, beta=0.9, theta=1.0, mode=mode, in_format=f)
        w = (synth.kaiming_normal(70 + l, co, ci) * np.float32(2.0)).astype(np.float32)
        wd = torch.from_numpy(w).to(DEV)
        T_out, Ho, Wo = api.tac_out_shape(desc)
        layers.append(dict(desc=desc, w_prepared=api.tac_prepare_weights(desc, wd),
                           v_inout=torch.zeros((B, co, Ho, Wo), dtype=torch.float32, device=DEV),
                           v_trace=torch.empty((T_out, B, co, Ho, Wo), dtype=torch.float32, device=DEV)))
        ws.append(wd)
        host.append((w, mode, K, pl))
    stack, outs = api.make_stack(layers)
    assert api.tac_stack_check(stack) == (api.TAC_OK, -1)
    sp = torch.from_numpy(np_pack(s)).to(DEV)
    api.tac_stack_forward(stack, sp)
    g_last = r.standard_normal(tuple(layers[-1]["v_trace"].shape)).astype(np.float32)
    got = api.tac_stack_backward(stack, ws, sp, torch.from_numpy(g_last).to(DEV), surrogate=api.TAC_SG_ARCTAN, alpha=2.0, detach_reset=True)
    torch.cuda.synchronize()
    x, fwd = s, []
    for (w, mode, K, pl) in host:
        out, v_pre, _ = oracle.conv_lif(x, w.astype(np.float64), K=K, beta=float(np.float32(0.9)), theta=1.0, mode=ORACLE_MODE[mode], pool2=pl)
        fwd.append((x, v_pre))
        x = out
    assert x.sum() > 0
    g = g_last.astype(np.float64)
    for l in (1, 0):
        w, mode, K, pl = host[l]
        ref = oracle.conv_lif_backward(fwd[l][0], w.astype(np.float64), fwd[l][1], g, K=K, beta=float(np.float32(0.9)), theta=1.0,
                                       mode=ORACLE_MODE[mode], surrogate=oracle.ARCTAN, alpha=2.0, detach_reset=True, pool2=pl)
        _close("layer %d dW" % l, got[l]["grad_w"].cpu().numpy(), ref["dW"])
        if l > 0:
            _close("layer %d dL/dS" % l, got[l]["grad_in"].cpu().numpy(), ref["g_in"])
        g = ref["g_in"]


@pytest.mark.parametrize("shape", [(32, 128, 6, 32), (32, 128, 5, 64), (64, 128, 9, 16)])
@pytest.mark.parametrize("mode,K,T", [(api.TAC_PER_STEP, 1, 3), (api.TAC_COLLAPSE, 4, 8), (api.TAC_PRESERVE, 2, 5)])
def test_backward_max_pool_on_load_on_the_matrix_cores(shape, mode, K, T):
    # the hidden layers of the event-data network (Conv-BN-LIF-MaxPool blocks, Sec. 5.1) at shapes the MFMA gradient
    # kernels take: the aggregates are pooled while they are rebuilt, the input gradient is routed to the stored frames
    from gpu_util import bf16_round_np
    Cin, Cout, H, W = shape
    B = 2
    r = _rng(1900 + Cin + H + W + K + T)
    s = (r.random((T, B, Cin, 2 * H, 2 * W)) < 0.08).astype(np.uint8)
    w = synth.kaiming_normal(62, Cout, Cin) * np.float32(1.5)
    desc = api.make_desc(T, B, Cin, H, W, Cout, K=K, beta=0.9, theta=1.0, mode=mode, precision=api.TAC_BF16,
                         in_format=api.TAC_IN_BITS_MAXPOOL2)
    T_out, Ho, Wo = api.tac_out_shape(desc)
    g_out = r.standard_normal((T_out, B, Cout, Ho, Wo)).astype(np.float32)
    sp, wd = torch.from_numpy(np_pack(s)).to(DEV), torch.from_numpy(w).to(DEV)
    v = torch.zeros((B, Cout, Ho, Wo), dtype=torch.float32, device=DEV)
    vt = torch.empty((T_out, B, Cout, Ho, Wo), dtype=torch.float32, device=DEV)
    api.tac_conv_lif(desc, sp, api.tac_prepare_weights(desc, wd), None, v, None, vt)
    got = api.tac_conv_lif_backward(desc, sp, wd, vt, torch.from_numpy(g_out).to(DEV), surrogate=api.TAC_SG_ARCTAN, alpha=2.0,
                                    detach_reset=True)
    torch.cuda.synchronize()
    kw = dict(K=K, beta=float(np.float32(0.9)), theta=1.0, mode=ORACLE_MODE[mode], pool2="max")
    out, v_pre, _ = oracle.conv_lif(s, bf16_round_np(w).astype(np.float64), round_a_bf16=True, **kw)
    ref = oracle.conv_lif_backward(s, w.astype(np.float64), v_pre, g_out.astype(np.float64), surrogate=oracle.ARCTAN, alpha=2.0,
                                   detach_reset=True, round_a_bf16=True, **kw)
    assert out.sum() > 0
    for name, a, b, tol in (("dL/dY", got["grad_y"], ref["dY"], 1e-3), ("dW", got["grad_w"], ref["dW"], TOL_BF16),
                            ("dL/dS", got["grad_in"], ref["g_in"], TOL_BF16)):
        e = np.abs(a.cpu().numpy() - b).max() / np.abs(b).max()
        assert e <= tol, "%s: %.3g" % (name, e)


# ---- the input gradient once per group of frames (dL/dS_{kK+j} = beta^(Kg-1-j) dL/dA_k, Eq. 2) ----------------------
def _group_factors(beta, K, T):
    """beta^(Kg-1-j) per frame, formed as the library forms them (double powers of the fp32 beta, rounded once)."""
    b = float(np.float32(beta))
    f = np.empty(T, dtype=np.float32)
    for t in range(T):
        k = t // K
        Kg = min(K, T - k * K)
        f[t] = np.float32(b ** (Kg - 1 - (t - k * K)))
    return f


# (Cin, Cout, H, W, stride, precision): the vector kernels and the matrix-core input gradient
GROUP_SHAPES = [(3, 5, 7, 9, 1, api.TAC_FP32), (16, 24, 12, 33, 2, api.TAC_FP32), (32, 128, 12, 32, 1, api.TAC_BF16),
                (64, 64, 9, 64, 1, api.TAC_BF16), (128, 32, 6, 64, 1, api.TAC_BF16)]


@pytest.mark.parametrize("shape", GROUP_SHAPES)
@pytest.mark.parametrize("mode,K,T", [(api.TAC_COLLAPSE, 4, 8), (api.TAC_COLLAPSE, 4, 7), (api.TAC_PRESERVE, 2, 6),
                                      (api.TAC_PRESERVE, 8, 13), (api.TAC_COLLAPSE, 8, 3), (api.TAC_PER_STEP, 1, 4)])
def test_input_gradient_once_per_group(shape, mode, K, T):
    Cin, Cout, H, W, stride, precision = shape
    B = 2
    r = _rng(1700 + Cin + Cout + H + W + K + T)
    s = (r.random((T, B, Cin, H, W)) < 0.2).astype(np.uint8)
    w = synth.kaiming_normal(47, Cout, Cin) * np.float32(1.5)
    beta, theta = 0.9, 1.0
    desc = api.make_desc(T, B, Cin, H, W, Cout, K=K, beta=beta, theta=theta, mode=mode, stride=stride, precision=precision)
    T_out, Ho, Wo = api.tac_out_shape(desc)
    Ke = 1 if mode == api.TAC_PER_STEP else min(K, T)
    G = -(-T // Ke)
    sp, wd = torch.from_numpy(np_pack(s)).to(DEV), torch.from_numpy(w).to(DEV)
    vt = torch.empty((T_out, B, Cout, Ho, Wo), dtype=torch.float32, device=DEV)
    v0 = torch.zeros((B, Cout, Ho, Wo), dtype=torch.float32, device=DEV)
    api.tac_conv_lif(desc, sp, api.tac_prepare_weights(desc, wd), None, v0, None, vt)
    r_g = r.standard_normal((T_out, B, Cout, Ho, Wo)).astype(np.float32)
    g = torch.from_numpy(r_g).to(DEV)
    frames = api.tac_conv_lif_backward(desc, sp, wd, vt, g)
    groups = api.tac_conv_lif_backward(desc, sp, wd, vt, g, grad_in_per_group=True)
    torch.cuda.synchronize()
    assert tuple(groups["grad_in"].shape) == (G, B, Cin, H, W)
    assert torch.equal(frames["grad_y"], groups["grad_y"])
    fr, gr = frames["grad_in"].cpu().numpy(), groups["grad_in"].cpu().numpy()
    f = _group_factors(beta, Ke, T)
    # the same fp32 product, formed by the library in one case and here in the other: identical bits
    expect = f[:, None, None, None, None] * gr[np.arange(T) // Ke]
    assert np.array_equal(fr, expect)
    # and against the oracle: the last frame of a group carries the factor 1, so its gradient is dL/dA_k itself
    kw = dict(K=K, beta=float(np.float32(beta)), theta=theta, mode=ORACLE_MODE[mode], stride=stride)
    v_pre = oracle.conv_lif(s, w.astype(np.float64), None, **kw)[1]
    ref = oracle.conv_lif_backward(s, w.astype(np.float64), v_pre, r_g.astype(np.float64), **kw)
    last = np.array([min((k + 1) * Ke, T) - 1 for k in range(G)])
    if precision == api.TAC_FP32:
        _close("dL/dA", gr, ref["g_in"][last])


@pytest.mark.parametrize("mode,K,T", [(api.TAC_COLLAPSE, 2, 6), (api.TAC_PRESERVE, 4, 10), (api.TAC_PER_STEP, 1, 9)])
@pytest.mark.parametrize("Kc,beta_c", [(2, 0.5), (4, 0.9), (8, 0.9)])
def test_output_gradient_read_once_per_group_of_the_next_layer(mode, K, T, Kc, beta_c):
    Cin, Cout, H, W, B = 6, 10, 9, 20, 2
    r = _rng(1800 + K + T + Kc)
    s = (r.random((T, B, Cin, H, W)) < 0.3).astype(np.uint8)
    w = synth.kaiming_normal(48, Cout, Cin) * np.float32(1.5)
    desc = api.make_desc(T, B, Cin, H, W, Cout, K=K, beta=0.9, theta=1.0, mode=mode)
    T_out, Ho, Wo = api.tac_out_shape(desc)
    Gc = -(-T_out // Kc)
    sp, wd = torch.from_numpy(np_pack(s)).to(DEV), torch.from_numpy(w).to(DEV)
    vt = torch.empty((T_out, B, Cout, Ho, Wo), dtype=torch.float32, device=DEV)
    v0 = torch.zeros((B, Cout, Ho, Wo), dtype=torch.float32, device=DEV)
    api.tac_conv_lif(desc, sp, api.tac_prepare_weights(desc, wd), None, v0, None, vt)
    dA = r.standard_normal((Gc, B, Cout, Ho, Wo)).astype(np.float32)
    f = _group_factors(beta_c, Kc, T_out)
    per_step = f[:, None, None, None, None] * dA[np.arange(T_out) // Kc]          # what the next layer would have written
    a = api.tac_conv_lif_backward(desc, sp, wd, vt, torch.from_numpy(per_step).to(DEV))
    b = api.tac_conv_lif_backward(desc, sp, wd, vt, torch.from_numpy(dA).to(DEV), grad_out_group_K=Kc, grad_out_group_beta=beta_c)
    torch.cuda.synchronize()
    assert torch.equal(a["grad_y"], b["grad_y"])
    assert torch.equal(a["grad_in"], b["grad_in"])
    assert torch.allclose(a["grad_w"], b["grad_w"], rtol=1e-4, atol=1e-5 * float(a["grad_w"].abs().max()))
    # the per-step form against the oracle (a shorter last group of the next layer included)
    kw = dict(K=K, beta=float(np.float32(0.9)), theta=1.0, mode=ORACLE_MODE[mode], stride=1)
    v_pre = oracle.conv_lif(s, w.astype(np.float64), None, **kw)[1]
    ref = oracle.conv_lif_backward(s, w.astype(np.float64), v_pre, per_step.astype(np.float64), **kw)
    # (the fast sigmoid's slope changes by up to 2 alpha = 50 per unit of V around the threshold, and the library reads
    # fp32 membranes of its own forward pass: a little more room than TOL over ten dependent steps)
    _close("dL/dY", b["grad_y"].cpu().numpy(), ref["dY"], 3e-4)
    _close("dW", b["grad_w"].cpu().numpy(), ref["dW"], 3e-4)


# ---- training through the max pool that the writer applies (out_format = TAC_OUT_BITS_MAXPOOL2) ---------------------
@pytest.mark.parametrize("mode,K,T", [(api.TAC_PER_STEP, 1, 4), (api.TAC_COLLAPSE, 2, 6), (api.TAC_PRESERVE, 2, 4)])
def test_backward_through_the_max_pool_in_the_writer(mode, K, T):
    # Layer A stores pooled spikes; the gradient it receives is that of the pooled tensor.  The oracle has no pooled
    # output: it runs the layer AFTER A with the max pool on load, whose input gradient is dL/d(A's unpooled spikes),
    # routed through the pool by the oracle's own rule, and the same layer on the pooled tensor, whose input gradient is
    # what the library is given.
    from gpu_util import bf16_round_np
    B, Cin, Ca, Cb, H, W = 2, 8, 16, 6, 12, 32
    r = _rng(1900 + K + T)
    s = (r.random((T, B, Cin, H, W)) < 0.3).astype(np.uint8)
    wA = bf16_round_np(synth.kaiming_normal(49, Ca, Cin) * np.float32(1.5))
    beta, theta = 0.9, 1.0
    desc = api.make_desc(T, B, Cin, H, W, Ca, K=K, beta=beta, theta=theta, mode=mode, precision=api.TAC_BF16,
                         out_format=api.TAC_OUT_BITS_MAXPOOL2)
    T_out, Ho, Wo = api.tac_out_shape(desc)
    sp, wd = torch.from_numpy(np_pack(s)).to(DEV), torch.from_numpy(wA).to(DEV)
    vt = torch.empty((T_out, B, Ca, Ho, Wo), dtype=torch.float32, device=DEV)
    pooled = api.tac_conv_lif(desc, sp, api.tac_prepare_weights(desc, wd), None, None, None, vt)
    kwA = dict(K=K, beta=float(np.float32(beta)), theta=theta, mode=ORACLE_MODE[mode])
    outA, v_preA, _ = oracle.conv_lif(s, wA.astype(np.float64), None, round_a_bf16=True, **kwA)
    assert np.array_equal(vt.cpu().numpy() >= np.float32(theta), outA.astype(bool)) and outA.sum() > 0     # same spikes on both sides
    from parity_util import np_unpack
    assert np.array_equal(np_unpack(pooled.cpu().numpy(), Wo // 2), oracle.maxpool2(outA).astype(np.uint8))
    # the layer after A, in the oracle only
    wB = r.standard_normal((Cb, Ca, 3, 3)) * 0.3
    kwB = dict(K=1, beta=0.8, theta=1.0, mode=oracle.PER_STEP)
    _, v_preB, _ = oracle.conv_lif(outA, wB, None, pool2="max", **kwB)
    gB = r.standard_normal(v_preB.shape)
    routed = oracle.conv_lif_backward(outA, wB, v_preB, gB, pool2="max", **kwB)["g_in"]                  # [T_out,B,Ca,Ho,Wo]
    at_pooled = oracle.conv_lif_backward(oracle.maxpool2(outA).astype(np.uint8), wB, v_preB, gB, **kwB)["g_in"]   # [T_out,B,Ca,Ho/2,Wo/2]
    assert np.allclose(routed.reshape(T_out, B, Ca, Ho // 2, 2, Wo // 2, 2).sum(axis=(4, 6)), at_pooled, rtol=1e-12, atol=1e-14)
    ref = oracle.conv_lif_backward(s, wA.astype(np.float64), v_preA, routed, **kwA)
    got = api.tac_conv_lif_backward(desc, sp, wd, vt, torch.from_numpy(at_pooled.astype(np.float32)).to(DEV))
    torch.cuda.synchronize()
    _close("dL/dY", got["grad_y"].cpu().numpy(), ref["dY"], 3e-4)
    _close("dW", got["grad_w"].cpu().numpy(), ref["dW"], TOL_BF16)
    _close("dL/dS", got["grad_in"].cpu().numpy(), ref["g_in"], TOL_BF16)
