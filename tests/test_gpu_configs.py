"""GPU parity on the five benchmark configurations (synthetic stand-ins for the paper's
rate-coded and event-camera workloads), layer by layer against the CPU oracle.

Multi-layer configurations are checked with teacher forcing: every GPU layer is fed the
ORACLE's input spikes, because one tolerated near-threshold flip legitimately changes all later
layers.  The free-running end-to-end difference is printed next to it.  Batch sizes are cut
where the oracle would otherwise take minutes (samples are independent); the full-size
roofline configuration is checked on sampled neurons in the launch configuration the
benchmark times.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2603_13810_amd import api, synth

from gpu_util import check_layer, run_gpu, ORACLE_MODE, bf16_round_np
from parity_util import np_unpack, compare

pytestmark = pytest.mark.gpu


def _rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


# ---------------------------------------------------------------- cfg2: two-layer rate-coded net

@pytest.mark.parametrize("precision", [api.TAC_FP32, api.TAC_BF16])
@pytest.mark.parametrize("K", [2, 4, 8])
def test_cfg2_two_layer_rate_coded(K, precision):
    wl = synth.WORKLOADS["cfg2"]
    B = 32
    s = wl.make_spikes(B=B)
    w1, w2 = wl.make_weights(0), wl.make_weights(1)
    kw = dict(beta=wl.beta, theta=wl.theta, precision=precision, plain_stats=False)
    # layer 1: TAC with group size K, 28x28, 1 -> 32
    # bf16: the short-contraction MFMA kernel; fp32: the vector-FMA kernel
    first = api.TAC_KERNEL_MFMA if precision == api.TAC_BF16 else api.TAC_KERNEL_DIRECT
    p1, g1, r1 = check_layer(s, w1, K=K, mode=api.TAC_COLLAPSE, expect_kernel=first, **kw)
    assert r1[0].shape == (wl.T // K, B, 32, 28, 28) and r1[0].sum() > 0
    # layer 2 on the collapsed sequence: 2x2 mean pool while loading, 32 -> 64 at 14x14, K2 = 1
    p2, g2, r2 = check_layer(r1[0], w2, K=1, mode=api.TAC_COLLAPSE, pool2=True, expect_kernel=first, **kw)
    assert r2[0].shape == (wl.T // K, B, 64, 14, 14) and r2[0].sum() > 0
    # free running: the GPU's own layer-1 spikes into layer 2
    g2f = run_gpu(g1["spikes"], w2, K=1, mode=api.TAC_COLLAPSE, pool2=True, beta=wl.beta, theta=wl.theta,
                  precision=precision, trace=False)
    diff = float((g2f["spikes"] != r2[0]).mean())
    print("cfg2 K=%d %s | L1 %s | L2 %s | free-running L2 spike difference %.2e" %
          (K, "bf16" if precision else "fp32", p1, p2, diff))
    if K == 2:   # the collapsed sequence (T = 4) still divides by K: layer 2 with K2 = K as well
        check_layer(r1[0], w2, K=2, mode=api.TAC_COLLAPSE, pool2=True, **kw)


# ---------------------------------------------------------------- cfg3: event-camera single layer

@pytest.mark.parametrize("mode,K", [(api.TAC_PER_STEP, 1), (api.TAC_COLLAPSE, 2), (api.TAC_PRESERVE, 2)])
def test_cfg3_event_camera_layer(mode, K):
    wl = synth.WORKLOADS["cfg3"]
    s = wl.make_spikes(B=4)
    assert 0.02 < s.mean() < 0.05                      # sparse background plus the moving patch
    w = wl.make_weights(0)
    par, g, r = check_layer(s, w, K=K, mode=mode, stride=2, beta=wl.beta, theta=wl.theta, precision=api.TAC_BF16,
                            expect_kernel=api.TAC_KERNEL_MFMA)
    assert g["spikes"].shape[-2:] == (64, 64) and r[0].sum() > 0
    print("cfg3", api.MODE_NAMES[mode], K, par, "| vs unrounded oracle:", par.plain)


# ---------------------------------------------------------------- cfg4: five-layer event stack

@pytest.mark.parametrize("gain", [1.0, 3.0])
@pytest.mark.parametrize("mode,K,calls", [(api.TAC_PER_STEP, 1, 80), (api.TAC_PRESERVE, 2, 40), (api.TAC_PRESERVE, 4, 20)])
def test_cfg4_five_layer_stack(mode, K, calls, gain):
    # gain 1 is the configuration as stated (Kaiming weights: with beta = 0.5 and theta = 1 the
    # deep layers then hardly fire); gain 3 scales the weights so that all five layers are active
    wl = synth.WORKLOADS["cfg4"]
    x_ref = wl.make_spikes(B=1)
    x_gpu = x_ref
    api.tac_reset_counters()
    report = []
    for li, L in enumerate(wl.layers):
        w = wl.make_weights(li) * np.float32(gain)
        kw = dict(K=K, mode=mode, stride=L.stride, beta=wl.beta, theta=wl.theta, precision=api.TAC_BF16)
        par, g, r = check_layer(x_ref, w, plain_stats=False, **kw)          # teacher forced
        assert r[0].shape[0] == wl.T                                         # TAC-TP keeps T at every layer
        gf = run_gpu(x_gpu, w, trace=False, **kw) if li else g               # free running
        report.append("L%d[%s] flips=%d rate=%.3f free-diff=%.1e" %
                      (li + 1, "mfma" if g["kernel"] == api.TAC_KERNEL_MFMA else "direct", par.flips,
                       r[0].mean(), float((gf["spikes"] != r[0]).mean())))
        x_ref, x_gpu = r[0], gf["spikes"]
    assert x_ref.shape == (wl.T, 1, 256, 16, 16)
    if gain > 1:
        assert x_ref.mean() > 0.01                                           # the last layer does fire
    stages, lif = api.tac_get_counters()
    # teacher-forced and free-running calls both count (layer 1 is shared): 9 layer calls
    assert stages == calls * 9 // 5 and lif == 16 * 9
    print("cfg4 gain %g" % gain, api.MODE_NAMES[mode], K, " | ".join(report))


# ---------------------------------------------------------------- cfg5: full size, sampled neurons

@pytest.fixture(scope="module")
def cfg5_inputs():
    wl = synth.WORKLOADS["cfg5"]
    dev = torch.device("cuda:0")
    out = {}
    for rate in (0.1, 0.3):
        packed = torch.empty((wl.T, wl.B, wl.C, wl.H, 2), dtype=torch.int32, device=dev)
        dense = np.empty((wl.T, 2, wl.C, wl.H, wl.W), dtype=np.uint8)        # samples 0 and B-1, before packing
        for t in range(wl.T):
            fr = synth.bernoulli_device(wl.seed + 100 * int(rate * 10) + t, wl.B, wl.C, wl.H, wl.W, rate, dev)
            api.tac_pack_spikes(fr, packed[t])
            dense[t, 0] = fr[0].cpu().numpy()
            dense[t, 1] = fr[wl.B - 1].cpu().numpy()
            del fr
        out[rate] = (packed, dense)
    torch.cuda.synchronize()
    return out


@pytest.mark.parametrize("rate,mode,K", [(0.1, api.TAC_PER_STEP, 1), (0.1, api.TAC_COLLAPSE, 4), (0.1, api.TAC_PRESERVE, 2),
                                         (0.3, api.TAC_COLLAPSE, 16), (0.3, api.TAC_PRESERVE, 8), (0.1, api.TAC_COLLAPSE, 2),
                                         (0.3, api.TAC_COLLAPSE, 8)])
def test_cfg5_full_size_sampled_neurons(cfg5_inputs, rate, mode, K):
    wl = synth.WORKLOADS["cfg5"]
    dev = torch.device("cuda:0")
    packed, dense = cfg5_inputs[rate]
    w = wl.make_weights(0)
    d = api.make_desc(wl.T, wl.B, 128, 64, 64, 128, K=K, beta=wl.beta, theta=wl.theta, mode=mode, precision=api.TAC_BF16)
    assert api.tac_select_kernel(d) == api.TAC_KERNEL_MFMA
    wp = api.tac_prepare_weights(d, torch.from_numpy(w).to(dev))
    T_out = api.tac_out_shape(d)[0]
    v = torch.zeros((wl.B, 128, 64, 64), dtype=torch.float32, device=dev)
    out = torch.full((T_out, wl.B, 128, 64, 2), -1, dtype=torch.int32, device=dev)
    api.tac_conv_lif(d, packed, wp, None, v, out)                     # the call the benchmark times (plus v_inout)
    torch.cuda.synchronize()
    r = _rng(int(rate * 100) + 7 * K + mode)
    n = 4000
    idx = np.stack([r.integers(0, 2, n), r.integers(0, 128, n), r.integers(0, 64, n), r.integers(0, 64, n)], 1).astype(np.int32)
    idx[:64, 2] = r.choice([0, 63], 64); idx[64:128, 3] = r.choice([0, 63], 64)      # image borders too
    ref = oracle.conv_lif_neurons(dense, bf16_round_np(w).astype(np.float64), idx=idx, K=K, beta=float(np.float32(wl.beta)),
                                  theta=1.0, mode=ORACLE_MODE[mode], round_a_bf16=True, nthreads=16)
    bsel = np.where(idx[:, 0] == 0, 0, wl.B - 1)
    sel = out[:, torch.from_numpy(bsel).to(dev), torch.from_numpy(idx[:, 1]).to(dev).long(),
              torch.from_numpy(idx[:, 2]).to(dev).long()].cpu().numpy()            # [T_out, n, 2] packed words
    gpu_spk = (sel[np.arange(T_out)[:, None], np.arange(n)[None, :], idx[:, 3] // 32] >> (idx[:, 3] % 32)) & 1
    par = compare(ref[0], ref[1], gpu_spk.astype(np.uint8), None, 1.0, 1e-3)
    assert par.mismatches == 0, str(par)
    v_gpu = v[torch.from_numpy(bsel).to(dev), torch.from_numpy(idx[:, 1]).to(dev).long(),
              torch.from_numpy(idx[:, 2]).to(dev).long(), torch.from_numpy(idx[:, 3]).to(dev).long()].cpu().numpy()
    clean = (ref[0] == gpu_spk).all(axis=0)
    err = np.abs(v_gpu - ref[2]) / np.maximum(np.abs(ref[2]), 1.0)
    assert err[clean].max() < 1e-3
    assert ref[0].mean() > 0.01
    print("cfg5 rate %.1f %s K=%d: %s final-V err %.2e output rate %.3f" %
          (rate, api.MODE_NAMES[mode], K, par, err[clean].max(), ref[0].mean()))


# ---------------------------------------------------------------- cfg5 backward: full size, sampled windows

_CENTRES = [0, 5, 11, 17, 23, 29, 35, 41, 47, 53, 58, 63]            # 5 x 5 input windows around them do not overlap


@pytest.mark.parametrize("mode,K", [(api.TAC_COLLAPSE, 4), (api.TAC_PER_STEP, 1), (api.TAC_PRESERVE, 8)])
def test_cfg5_full_size_backward_sampled_windows(cfg5_inputs, mode, K):
    """Backward pass in the launch configuration `bench.py --backward` times.  dL/d(output spikes) is zero except on
    sampled 3 x 3 windows of output pixels (all channels, all steps; image corners and edges among them), so every
    gradient is a sum over those windows only and the oracle can form it from 5 x 5 crops of the input: dW and dbias
    are compared whole, dL/dS on the crops, and dL/dS must be exactly zero everywhere else."""
    wl = synth.WORKLOADS["cfg5"]
    dev = torch.device("cuda:0")
    packed, dense = cfg5_inputs[0.1]
    w = wl.make_weights(0)
    beta = float(np.float32(wl.beta))
    d = api.make_desc(wl.T, wl.B, 128, 64, 64, 128, K=K, beta=wl.beta, theta=wl.theta, mode=mode, precision=api.TAC_BF16)
    wd = torch.from_numpy(w).to(dev)
    T_out = api.tac_out_shape(d)[0]
    v = torch.zeros((wl.B, 128, 64, 64), dtype=torch.float32, device=dev)
    vt = torch.empty((T_out, wl.B, 128, 64, 64), dtype=torch.float32, device=dev)
    api.tac_conv_lif(d, packed, api.tac_prepare_weights(d, wd), None, v, None, vt)
    torch.cuda.synchronize()
    del v

    r = _rng(5000 + 7 * K + mode)
    cells = [(s, y, x) for s in (0, 1) for y in _CENTRES for x in _CENTRES]
    corners = [c for c in cells if c[1] in (0, 63) or c[2] in (0, 63)]
    pick = [corners[i] for i in r.choice(len(corners), 24, replace=False)]
    inner = [c for c in cells if c not in corners]
    pick += [inner[i] for i in r.choice(len(inner), 40, replace=False)]
    n = len(pick)
    # crops: input rows/columns y-2 .. y+2 (zero outside the image, which is the layer's own padding), output
    # pixels of the crop = the same 5 x 5 positions, of which the inner 3 x 3 see their whole receptive field
    crop = np.zeros((wl.T, n, 128, 5, 5), dtype=np.uint8)
    inside = np.zeros((n, 5, 5), dtype=bool)
    for i, (s, y, x) in enumerate(pick):
        for dy in range(5):
            for dx in range(5):
                yy, xx = y - 2 + dy, x - 2 + dx
                if 0 <= yy < 64 and 0 <= xx < 64:
                    crop[:, i, :, dy, dx] = dense[:, s, :, yy, xx]
                    inside[i, dy, dx] = True
    kw = dict(K=K, beta=beta, theta=1.0, mode=ORACLE_MODE[mode])
    spk_ref, v_ref, _ = oracle.conv_lif(crop, bf16_round_np(w).astype(np.float64), None, round_a_bf16=True, **kw)
    win = inside.copy()                                                  # the 3 x 3 window, where it lies in the image
    win[:, 0, :] = win[:, 4, :] = False
    win[:, :, 0] = win[:, :, 4] = False
    # the library's recorded membranes on the windows; windows with a spike that differs from the oracle's (a
    # membrane within rounding of the threshold) are left out of the loss, on both sides
    keep = np.ones(n, dtype=bool)
    v_err = 0.0
    for i, (s, y, x) in enumerate(pick):
        b = 0 if s == 0 else wl.B - 1
        for dy in range(1, 4):
            for dx in range(1, 4):
                if not win[i, dy, dx]:
                    continue
                vg = vt[:, b, :, y - 2 + dy, x - 2 + dx].cpu().numpy().astype(np.float64)
                vr = v_ref[:, i, :, dy, dx]
                if ((vg >= 1.0) != (vr >= 1.0)).any():
                    keep[i] = False
                else:
                    v_err = max(v_err, (np.abs(vg - vr) / np.maximum(np.abs(vr), 1.0)).max())
    assert keep.sum() >= n - 4, "too many windows with a threshold flip: %d of %d" % (n - keep.sum(), n)
    assert v_err < 1e-3
    g_crop = r.standard_normal((T_out, n, 128, 5, 5)) * (win & keep[:, None, None])[None, :, None]
    g_crop = g_crop.astype(np.float32)
    g_out = torch.zeros((T_out, wl.B, 128, 64, 64), dtype=torch.float32, device=dev)
    for i, (s, y, x) in enumerate(pick):
        b = 0 if s == 0 else wl.B - 1
        for dy in range(1, 4):
            for dx in range(1, 4):
                if win[i, dy, dx]:
                    g_out[:, b, :, y - 2 + dy, x - 2 + dx] = torch.from_numpy(g_crop[:, i, :, dy, dx]).to(dev)
    got = api.tac_conv_lif_backward(d, packed, wd, vt, g_out, surrogate=api.TAC_SG_ARCTAN, alpha=2.0, detach_reset=True)
    torch.cuda.synchronize()
    ref = oracle.conv_lif_backward(crop, w.astype(np.float64), v_ref, g_crop.astype(np.float64), surrogate=oracle.ARCTAN,
                                   alpha=2.0, detach_reset=True, round_a_bf16=True, **kw)

    def err(name, a, b, tol):
        e = np.abs(a - b).max() / np.abs(b).max()
        assert e <= tol, "%s: %.3g" % (name, e)
        return e
    e_w = err("dW", got["grad_w"].cpu().numpy(), ref["dW"], 2e-2)
    e_b = err("dbias", got["grad_bias"].cpu().numpy(), ref["dbias"], 1e-3)
    gi = got["grad_in"]
    scale = np.abs(ref["g_in"]).max()
    e_s = 0.0
    for i, (s, y, x) in enumerate(pick):
        b = 0 if s == 0 else wl.B - 1
        y0, y1, x0, x1 = max(y - 2, 0), min(y + 3, 64), max(x - 2, 0), min(x + 3, 64)
        g = gi[:, b, :, y0:y1, x0:x1].cpu().numpy()
        rr = ref["g_in"][:, i, :, y0 - (y - 2):y1 - (y - 2), x0 - (x - 2):x1 - (x - 2)]
        e_s = max(e_s, np.abs(g - rr).max() / scale)
        gi[:, b, :, y0:y1, x0:x1] = 0
    assert e_s <= 2e-2, "dL/dS: %.3g" % e_s
    assert scale > 0 and np.abs(ref["dW"]).max() > 0
    assert float(gi.abs().max()) == 0.0, "input gradient outside the windows"
    print("cfg5 backward %s K=%d: %d windows (%d left out), membrane err %.1e, dW %.1e dbias %.1e dS %.1e" %
          (api.MODE_NAMES[mode], K, n, n - keep.sum(), v_err, e_w, e_b, e_s))
