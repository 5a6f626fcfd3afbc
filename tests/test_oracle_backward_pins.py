"""Pins of the oracle's backward pass (surrogate-gradient BPTT of the conv-LIF layer; Sec. 5.1 "Training").

The paper names its surrogates and "detach reset" but prints no formulas, so these tests fix the oracle to the
mathematics instead: (1) the backward pass is the exact gradient of the network in which the step function is
replaced by the surrogate's antiderivative, checked by central finite differences; (2) a scalar example worked
by hand; (3) automatic differentiation of a plain PyTorch forward pass with a custom spike function.
"""
import json
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle
from oracle import PER_STEP, TAC, TAC_TP, FAST_SIGMOID, ARCTAN

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


def sg(kind, alpha, x):
    """ds/dV in x = V - theta, from the published definitions of the two surrogates."""
    if kind == FAST_SIGMOID:
        return 1.0 / (1.0 + alpha * np.abs(x)) ** 2
    return 0.5 * alpha / (1.0 + (0.5 * np.pi * alpha * x) ** 2)


def soft_spike(kind, alpha, x):
    """An antiderivative of sg: the smooth function whose slope the surrogate is."""
    if kind == FAST_SIGMOID:
        return x / (1.0 + alpha * np.abs(x))
    return np.arctan(0.5 * np.pi * alpha * x) / np.pi


def groups(T, K):
    return [(t0, min(K, T - t0)) for t0 in range(0, T, K)]


def smooth_net(x, w, bias, g_out, *, K, beta, theta, mode, stride, kind, alpha, soft_reset):
    """The layer with the step function replaced by soft_spike (in the output, and in the reset when soft_reset):
    returns (loss = sum g_out * soft spikes, membranes before the reset).  numpy/torch double, written for this test."""
    T = x.shape[0]
    K = 1 if mode == PER_STEP else K
    V, vs, loss, n = None, [], 0.0, 0
    for t0, Kg in groups(T, K):
        A = sum(beta ** (Kg - 1 - j) * x[t0 + j] for j in range(Kg))
        Y = F.conv2d(torch.from_numpy(A), torch.from_numpy(w), torch.from_numpy(bias), stride=stride, padding=1).numpy()
        for _ in range(Kg if mode == TAC_TP else 1):
            d = beta ** Kg if mode == TAC else beta
            V = Y if V is None else d * V + Y
            s = soft_spike(kind, alpha, V - theta)
            vs.append(V.copy())
            loss += float((g_out[n] * s).sum())
            if soft_reset:
                V = V - theta * s
            n += 1
    return loss, np.stack(vs)


CASES = [(PER_STEP, 1, 5, 1), (TAC, 2, 6, 1), (TAC, 3, 7, 2), (TAC_TP, 2, 6, 1), (TAC_TP, 4, 7, 2), (TAC, 4, 5, 1)]


@pytest.mark.parametrize("mode,K,T,stride", CASES)
@pytest.mark.parametrize("kind,alpha", [(FAST_SIGMOID, 25.0), (ARCTAN, 2.0)])
@pytest.mark.parametrize("soft_reset", [False, True])
def test_backward_is_the_gradient_of_the_smoothed_network(mode, K, T, stride, kind, alpha, soft_reset):
    # soft_reset False <-> detach_reset True: the reset carries no gradient, the smooth network has none
    r = _rng(300 + 7 * K + T + stride + kind)
    B, Cin, Cout, H, W = 2, 2, 3, 5, 4
    x = r.random((T, B, Cin, H, W)) * (r.random((T, B, Cin, H, W)) < 0.6)         # real-valued frames (Sec. 4.2)
    w = r.standard_normal((Cout, Cin, 3, 3)) * 0.3
    bias = r.standard_normal(Cout) * 0.1
    Ho, Wo = (H - 1) // stride + 1, (W - 1) // stride + 1
    N = T if mode != TAC else -(-T // K)
    g_out = r.standard_normal((N, B, Cout, Ho, Wo))
    kw = dict(K=K, beta=0.8, theta=1.0, mode=mode, stride=stride, kind=kind, alpha=alpha, soft_reset=soft_reset)
    loss0, v = smooth_net(x, w, bias, g_out, **kw)
    got = oracle.conv_lif_backward(x, w, v, g_out, K=K, beta=0.8, theta=1.0, mode=mode, stride=stride, surrogate=kind,
                                   alpha=alpha, detach_reset=not soft_reset)
    h = 1e-6

    def fd(arr, idx):
        old = arr[idx]
        arr[idx] = old + h
        lp = smooth_net(x, w, bias, g_out, **kw)[0]
        arr[idx] = old - h
        lm = smooth_net(x, w, bias, g_out, **kw)[0]
        arr[idx] = old
        return (lp - lm) / (2 * h)

    scale = max(1.0, np.abs(got["dW"]).max())
    for _ in range(10):
        idx = tuple(r.integers(0, n) for n in w.shape)
        assert abs(fd(w, idx) - got["dW"][idx]) < 1e-6 * scale, ("dW", idx)
    for co in range(Cout):
        assert abs(fd(bias, (co,)) - got["dbias"][co]) < 1e-6 * max(1.0, np.abs(got["dbias"]).max()), ("dbias", co)
    for _ in range(10):
        idx = tuple(r.integers(0, n) for n in x.shape)
        assert abs(fd(x, idx) - got["g_in"][idx]) < 1e-6 * max(1.0, np.abs(got["g_in"]).max()), ("g_in", idx)


def test_hand_worked_scalar_example_backward():
    g = json.load(open(os.path.join(GOLDEN, "backward_scalar_example.json")))
    s = np.array(g["input"], dtype=np.uint8).reshape(-1, 1, 1, 1, 1)
    w = np.zeros((1, 1, 3, 3)); w[0, 0, 1, 1] = g["centre_tap"]
    out, v_pre, _ = oracle.conv_lif(s, w, beta=g["beta"], theta=g["theta"], mode=PER_STEP)
    assert out.ravel().tolist() == g["spikes"] and v_pre.ravel().tolist() == g["v_pre"]
    g_out = np.array(g["g_out"], dtype=np.float64).reshape(-1, 1, 1, 1, 1)
    for key, detach in (("not_detached", False), ("detached", True)):
        b = oracle.conv_lif_backward(s, w, v_pre, g_out, beta=g["beta"], theta=g["theta"], mode=PER_STEP,
                                     surrogate=FAST_SIGMOID, alpha=g["alpha"], detach_reset=detach)
        assert np.allclose(b["dY"].ravel(), g[key]["dY"], rtol=1e-12, atol=0), key
        assert np.isclose(b["dW"][0, 0, 1, 1], g[key]["dW_centre"], rtol=1e-12), key
        assert np.allclose(b["g_in"].ravel(), g[key]["g_in"], rtol=1e-12, atol=0), key


class _Spike(torch.autograd.Function):
    @staticmethod
    def forward(ctx, x, kind, alpha):
        ctx.save_for_backward(x)
        ctx.kind, ctx.alpha = kind, alpha
        return (x >= 0).to(x.dtype)

    @staticmethod
    def backward(ctx, g):
        (x,) = ctx.saved_tensors
        if ctx.kind == FAST_SIGMOID:
            d = 1.0 / (1.0 + ctx.alpha * x.abs()) ** 2
        else:
            d = 0.5 * ctx.alpha / (1.0 + (0.5 * np.pi * ctx.alpha * x) ** 2)
        return g * d, None, None


@pytest.mark.parametrize("mode,K,T,stride", CASES + [(TAC_TP, 8, 8, 1)])
@pytest.mark.parametrize("kind,alpha,detach", [(FAST_SIGMOID, 25.0, False), (ARCTAN, 2.0, True), (FAST_SIGMOID, 5.0, True)])
def test_backward_against_automatic_differentiation(mode, K, T, stride, kind, alpha, detach):
    r = _rng(500 + 11 * K + T + stride + kind)
    B, Cin, Cout, H, W = 2, 3, 4, 6, 5
    s = (r.random((T, B, Cin, H, W)) < 0.4).astype(np.uint8)
    w = r.standard_normal((Cout, Cin, 3, 3)) * 0.5
    bias = r.standard_normal(Cout) * 0.1
    beta, theta = 0.9, 1.0
    out, v_pre, _ = oracle.conv_lif(s, w, bias, K=K, beta=beta, theta=theta, mode=mode, stride=stride)
    g_out = r.standard_normal(out.shape)
    got = oracle.conv_lif_backward(s, w, v_pre, g_out, K=K, beta=beta, theta=theta, mode=mode, stride=stride, surrogate=kind,
                                   alpha=alpha, detach_reset=detach)
    # the same layer as a plain PyTorch graph
    xt = torch.tensor(s, dtype=torch.float64, requires_grad=True)
    wt = torch.tensor(w, requires_grad=True)
    bt = torch.tensor(bias, requires_grad=True)
    Kq = 1 if mode == PER_STEP else K
    V, spikes = torch.zeros(()), []
    for t0, Kg in groups(T, Kq):
        A = sum(beta ** (Kg - 1 - j) * xt[t0 + j] for j in range(Kg))
        Y = F.conv2d(A, wt, bt, stride=stride, padding=1)
        for _ in range(Kg if mode == TAC_TP else 1):
            V = (beta ** Kg if mode == TAC else beta) * V + Y
            sp = _Spike.apply(V - theta, kind, alpha)
            spikes.append(sp)
            V = V - theta * (sp.detach() if detach else sp)
    st = torch.stack(spikes)
    assert np.array_equal(st.detach().numpy().astype(np.uint8), out) and out.sum() > 0
    (st * torch.tensor(g_out)).sum().backward()
    for name, ref in (("dW", wt.grad), ("dbias", bt.grad), ("g_in", xt.grad)):
        ref = ref.numpy()
        assert np.allclose(got[name], ref, rtol=1e-9, atol=1e-10 * max(1.0, np.abs(ref).max())), name


@pytest.mark.parametrize("pool", [True, "max"])
@pytest.mark.parametrize("mode,K,T", [(PER_STEP, 1, 4), (TAC, 2, 6), (TAC_TP, 3, 7)])
def test_backward_through_the_pool_in_front_of_the_layer_against_automatic_differentiation(pool, mode, K, T):
    # mean pool: linear; max pool: the gradient goes to the first maximal input of the window in row-major order,
    # which is what the library pooling routine differentiated here does as well
    r = _rng(700 + 13 * K + T + (pool == "max"))
    B, Cin, Cout, H, W = 2, 3, 4, 5, 4
    s = (r.random((T, B, Cin, 2 * H, 2 * W)) < 0.4).astype(np.uint8)
    w = r.standard_normal((Cout, Cin, 3, 3)) * 0.6
    beta, theta = 0.9, 1.0
    out, v_pre, _ = oracle.conv_lif(s, w, K=K, beta=beta, theta=theta, mode=mode, pool2=pool)
    g_out = r.standard_normal(out.shape)
    got = oracle.conv_lif_backward(s, w, v_pre, g_out, K=K, beta=beta, theta=theta, mode=mode, surrogate=ARCTAN, alpha=2.0,
                                   detach_reset=True, pool2=pool)
    xt = torch.tensor(s, dtype=torch.float64, requires_grad=True)
    wt = torch.tensor(w, requires_grad=True)
    Kq = 1 if mode == PER_STEP else K
    V, spikes = torch.zeros(()), []
    for t0, Kg in groups(T, Kq):
        fr = [F.max_pool2d(xt[t0 + j], 2) if pool == "max" else F.avg_pool2d(xt[t0 + j], 2) for j in range(Kg)]
        A = sum(beta ** (Kg - 1 - j) * fr[j] for j in range(Kg))
        Y = F.conv2d(A, wt, None, padding=1)
        for _ in range(Kg if mode == TAC_TP else 1):
            V = (beta ** Kg if mode == TAC else beta) * V + Y
            sp = _Spike.apply(V - theta, ARCTAN, 2.0)
            spikes.append(sp)
            V = V - theta * sp.detach()
    st = torch.stack(spikes)
    assert np.array_equal(st.detach().numpy().astype(np.uint8), out) and out.sum() > 0
    (st * torch.tensor(g_out)).sum().backward()
    assert np.allclose(got["dW"], wt.grad.numpy(), rtol=1e-9, atol=1e-10)
    assert np.allclose(got["g_in"], xt.grad.numpy(), rtol=1e-9, atol=1e-12)
    assert got["g_in"].shape == s.shape


@pytest.mark.parametrize("mode,K,T", [(oracle.TAC, 4, 8), (oracle.TAC, 4, 7), (oracle.TAC_TP, 3, 8)])
def test_the_frames_of_a_group_receive_one_gradient_times_their_aggregate_weights(mode, K, T):
    # A_k = sum_j beta^(Kg-1-j) S_{kK+j} (Eq. 2) is the only place a frame enters, so dL/dS_{kK+j} = beta^(Kg-1-j) dL/dA_k:
    # within a group the input gradients are multiples of the last frame's, whose factor is 1
    r = np.random.Generator(np.random.PCG64(77 + K + T))
    B, Cin, Cout, H, W = 2, 3, 4, 6, 7
    s = (r.random((T, B, Cin, H, W)) < 0.4).astype(np.uint8)
    w = r.standard_normal((Cout, Cin, 3, 3))
    beta = 0.8
    kw = dict(K=K, beta=beta, theta=1.0, mode=mode)
    out, v_pre, _ = oracle.conv_lif(s, w, None, **kw)
    g_out = r.standard_normal(v_pre.shape)
    g_in = oracle.conv_lif_backward(s, w, v_pre, g_out, **kw)["g_in"]
    assert np.abs(g_in).max() > 0
    for k in range(-(-T // K)):
        Kg = min(K, T - k * K)
        last = g_in[k * K + Kg - 1]
        for j in range(Kg):
            np.testing.assert_allclose(g_in[k * K + j], beta ** (Kg - 1 - j) * last, rtol=1e-12, atol=1e-15)
