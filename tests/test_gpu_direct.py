"""GPU parity of the vector-FMA kernel family against the CPU oracle, through the C ABI."""
import numpy as np
import pytest
import torch

from paper_2603_13810_amd import api, synth

from gpu_util import check_layer, run_gpu, run_oracle
from parity_util import np_pack, np_unpack, compare

pytestmark = pytest.mark.gpu

MODES = [(api.TAC_PER_STEP, 1), (api.TAC_COLLAPSE, 2), (api.TAC_COLLAPSE, 4), (api.TAC_PRESERVE, 2), (api.TAC_PRESERVE, 4)]


def _rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


def test_pack_unpack_roundtrip_and_layout():
    dev = torch.device("cuda:0")
    for W in (1, 28, 32, 33, 64, 70, 128, 200):
        d = (_rng(W).random((3, 5, 7, W)) < 0.3).astype(np.uint8)
        p = api.tac_pack_spikes(torch.from_numpy(d).to(dev))
        torch.cuda.synchronize()
        assert np.array_equal(p.cpu().numpy(), np_pack(d)), W          # layout and zero pad bits
        u = api.tac_unpack_spikes(p, W)
        assert np.array_equal(u.cpu().numpy(), d), W
    # non-zero bytes other than 1 pack as 1
    d = torch.tensor([[0, 2, 255, 0, 1]], dtype=torch.uint8, device=dev)
    assert api.tac_pack_spikes(d).item() == 0b10110


def test_packed_word_sparsity_matches_simd_bound():
    # Prop. 1: a 32-wide group of Bernoulli(0.1) lanes is all-zero with probability 0.9^32 = 0.034
    d = synth.bernoulli(7, 1, 4, 8, 64, 64, 0.1)
    p = api.tac_pack_spikes(torch.from_numpy(d).cuda()).cpu().numpy()
    frac = float((p == 0).mean())
    assert abs(frac - 0.9 ** 32) < 0.005


@pytest.mark.parametrize("mode,K", MODES)
def test_cfg1_small_layer_fp32(mode, K):
    wl = synth.WORKLOADS["cfg1"]
    s = wl.make_spikes()
    w = (_rng(1).standard_normal((8, 1, 3, 3)) * np.sqrt(2.0 / 9.0)).astype(np.float32)
    par, g, r = check_layer(s, w, K=K, beta=wl.beta, theta=wl.theta, mode=mode, expect_kernel=api.TAC_KERNEL_DIRECT)
    assert r[0].sum() > 0
    print("cfg1", api.MODE_NAMES[mode], K, par)


@pytest.mark.parametrize("mode,K", MODES)
@pytest.mark.parametrize("shape", [
    dict(B=2, Cin=3, H=7, W=20, Cout=5, stride=1),
    dict(B=1, Cin=2, H=9, W=70, Cout=20, stride=2),
    dict(B=3, Cin=17, H=12, W=33, Cout=33, stride=1),
    dict(B=1, Cin=4, H=37, W=130, Cout=8, stride=2),
])
def test_ragged_shapes_fp32(mode, K, shape):
    r = _rng(hash((mode, K, shape["W"])) % 2 ** 31)
    T = 8
    s = (r.random((T, shape["B"], shape["Cin"], shape["H"], shape["W"])) < 0.25).astype(np.uint8)
    w = synth.kaiming_normal(3, shape["Cout"], shape["Cin"])
    bias = (r.standard_normal(shape["Cout"]) * 0.1).astype(np.float32)
    Ho = (shape["H"] - 1) // shape["stride"] + 1
    Wo = (shape["W"] - 1) // shape["stride"] + 1
    v0 = (r.standard_normal((shape["B"], shape["Cout"], Ho, Wo)) * 0.3).astype(np.float32)
    par, g, ref = check_layer(s, w, K=K, beta=0.9, theta=1.0, mode=mode, stride=shape["stride"], bias=bias, v0=v0)
    assert ref[0].sum() > 0


@pytest.mark.parametrize("mode,K", MODES)
def test_pool_on_load(mode, K):
    r = _rng(31 + K)
    s = (r.random((8, 2, 6, 28, 28)) < 0.3).astype(np.uint8)
    w = synth.kaiming_normal(5, 12, 6)
    par, g, ref = check_layer(s, w, K=K, beta=0.9, theta=1.0, mode=mode, pool2=True)
    assert g["spikes"].shape[-2:] == (14, 14) and ref[0].sum() > 0


@pytest.mark.parametrize("mode,K", MODES)
def test_bf16_operands_on_direct_kernel(mode, K):
    r = _rng(41 + K)
    s = (r.random((8, 2, 16, 10, 40)) < 0.2).astype(np.uint8)
    w = synth.kaiming_normal(6, 24, 16)
    par, g, ref = check_layer(s, w, K=K, beta=0.9, theta=1.0, mode=mode, precision=api.TAC_BF16,
                              kernel=api.TAC_KERNEL_DIRECT)
    print("bf16 direct", api.MODE_NAMES[mode], K, par)


def test_threshold_tie_and_integer_exactness():
    # integer-valued weights, beta = 1, theta = 2: V lands exactly on theta and must fire
    r = _rng(51)
    s = (r.random((6, 1, 2, 8, 8)) < 0.4).astype(np.uint8)
    w = r.integers(-1, 2, size=(4, 2, 3, 3)).astype(np.float32)
    for mode, K in [(api.TAC_PER_STEP, 1), (api.TAC_COLLAPSE, 2), (api.TAC_PRESERVE, 3)]:
        g = run_gpu(s, w, K=K, beta=1.0, theta=2.0, mode=mode)
        ref = run_oracle(s, w, K=K, beta=1.0, theta=2.0, mode=mode)
        assert (ref[1] == 2.0).any()                      # the tie does occur
        assert np.array_equal(g["spikes"], ref[0])
        assert np.array_equal(g["v_trace"].astype(np.float64), ref[1])


def test_K1_equals_per_step_bitwise_on_gpu():
    r = _rng(61)
    s = (r.random((8, 2, 3, 9, 40)) < 0.3).astype(np.uint8)
    w = synth.kaiming_normal(7, 8, 3)
    a = run_gpu(s, w, K=1, beta=0.9, theta=1.0, mode=api.TAC_PER_STEP)
    for mode in (api.TAC_COLLAPSE, api.TAC_PRESERVE):
        b = run_gpu(s, w, K=1, beta=0.9, theta=1.0, mode=mode)
        assert np.array_equal(a["packed"], b["packed"]) and np.array_equal(a["v_trace"], b["v_trace"])


def test_state_carry_across_calls():
    # the membrane is the only state: T = 8 in one call equals two calls of T = 4 carrying v_inout
    r = _rng(71)
    s = (r.random((8, 2, 3, 9, 40)) < 0.3).astype(np.uint8)
    w = synth.kaiming_normal(8, 8, 3)
    for mode, K in [(api.TAC_PER_STEP, 1), (api.TAC_COLLAPSE, 2), (api.TAC_PRESERVE, 4)]:
        whole = run_gpu(s, w, K=K, beta=0.9, theta=1.0, mode=mode)
        a = run_gpu(s[:4], w, K=K, beta=0.9, theta=1.0, mode=mode)
        b = run_gpu(s[4:], w, K=K, beta=0.9, theta=1.0, mode=mode, v0=a["v_final"])
        assert np.array_equal(np.concatenate([a["packed"], b["packed"]]), whole["packed"])
        assert np.array_equal(b["v_final"], whole["v_final"])


def test_null_state_and_no_trace():
    r = _rng(81)
    s = (r.random((4, 1, 2, 8, 30)) < 0.3).astype(np.uint8)
    w = synth.kaiming_normal(9, 8, 2)
    a = run_gpu(s, w, K=2, beta=0.9, theta=1.0, mode=api.TAC_COLLAPSE, trace=True)
    b = run_gpu(s, w, K=2, beta=0.9, theta=1.0, mode=api.TAC_COLLAPSE, trace=False)
    assert b["v_final"] is None and np.array_equal(a["packed"], b["packed"])


def test_conv_call_counts_five_layers():
    # Table 3: 5 conv layers at T = 16 make 80 / 40 / 20 / 10 conv calls for K = 1 / 2 / 4 / 8
    dev = torch.device("cuda:0")
    chans = [2, 4, 4, 4, 4, 4]
    for K, expect in [(1, 80), (2, 40), (4, 20), (8, 10)]:
        api.tac_reset_counters()
        x = torch.from_numpy(np_pack((_rng(K).random((16, 1, 2, 8, 8)) < 0.3).astype(np.uint8))).to(dev)
        for l in range(5):
            d = api.make_desc(16, 1, chans[l], 8, 8, chans[l + 1], K=K, beta=0.5, theta=1.0,
                              mode=api.TAC_PRESERVE if K > 1 else api.TAC_PER_STEP)
            wp = api.tac_prepare_weights(d, torch.from_numpy(synth.kaiming_normal(l, chans[l + 1], chans[l])).to(dev))
            x = api.tac_conv_lif(d, x, wp)
        torch.cuda.synchronize()
        assert api.tac_get_counters() == (expect, 80)


@pytest.mark.parametrize("mode,K", [(api.TAC_PER_STEP, 1), (api.TAC_COLLAPSE, 2), (api.TAC_PRESERVE, 4)])
@pytest.mark.parametrize("precision", [api.TAC_FP32, api.TAC_BF16])
def test_max_pool_on_load(mode, K, precision):
    # the previous layer's spikes arrive unpooled; MaxPool(2) = OR of the 2x2 bits while loading
    r = np.random.Generator(np.random.PCG64(31 + K))
    s = (r.random((8, 2, 6, 2 * 9, 2 * 20)) < 0.15).astype(np.uint8)
    w = synth.kaiming_normal(41, 16, 6)
    par, g, ref = check_layer(s, w, K=K, beta=0.9, theta=1.0, mode=mode, pool2="max", precision=precision,
                              kernel=api.TAC_KERNEL_DIRECT)
    assert ref[0].sum() > 0 and g["spikes"].shape[-2:] == (9, 20)
    # and it is not the mean pool
    gm = run_gpu(s, w, K=K, beta=0.9, theta=1.0, mode=mode, pool2=True, precision=precision, kernel=api.TAC_KERNEL_DIRECT)
    assert (gm["spikes"] != g["spikes"]).any()


def test_fold_batchnorm_on_device():
    import oracle
    r = np.random.Generator(np.random.PCG64(51))
    w = (r.standard_normal((24, 5, 3, 3)) * 0.3).astype(np.float32)
    bias = (r.standard_normal(24) * 0.2).astype(np.float32)
    g, b = r.uniform(0.5, 1.5, 24).astype(np.float32), (r.standard_normal(24) * 0.1).astype(np.float32)
    mean, var = (r.standard_normal(24) * 0.3).astype(np.float32), r.uniform(0.2, 2.0, 24).astype(np.float32)
    dev = torch.device("cuda:0")
    t = lambda a: torch.from_numpy(a).to(dev)
    for bb in (bias, None):
        wf, bf = api.tac_fold_batchnorm(t(w), None if bb is None else t(bb), t(g), t(b), t(mean), t(var), eps=1e-5)
        rw, rb = oracle.fold_batchnorm(w, bb, g, b, mean, var, eps=float(np.float32(1e-5)))
        assert np.abs(wf.cpu().numpy() - rw).max() <= 1e-7 * np.abs(rw).max() + 1e-12
        assert np.abs(bf.cpu().numpy() - rb).max() <= 1e-6
    # folded layer = BN after the convolution, checked on the membrane trace of a spiking layer
    s = (r.random((4, 1, 5, 8, 32)) < 0.3).astype(np.uint8)
    wf, bf = api.tac_fold_batchnorm(t(w), t(bias), t(g), t(b), t(mean), t(var), eps=1e-5)
    rw, rb = oracle.fold_batchnorm(w, bias, g, b, mean, var, eps=float(np.float32(1e-5)))
    gpu = run_gpu(s, wf.cpu().numpy(), K=2, beta=0.9, theta=1.0, mode=api.TAC_COLLAPSE, bias=bf.cpu().numpy())
    ref = oracle.conv_lif(s, rw, rb, K=2, beta=0.9, theta=1.0, mode=oracle.TAC)
    assert np.abs(gpu["v_trace"] - ref[1]).max() < 1e-4


@pytest.mark.parametrize("mode,K", [(api.TAC_PER_STEP, 1), (api.TAC_COLLAPSE, 4), (api.TAC_PRESERVE, 2)])
@pytest.mark.parametrize("precision", [api.TAC_FP32, api.TAC_BF16])
def test_real_valued_input_frames(mode, K, precision):
    # the continuous-valued first layer: float32 frames instead of packed spikes
    r = np.random.Generator(np.random.PCG64(61 + K))
    x = (r.random((8, 2, 3, 11, 37)) * (r.random((8, 2, 3, 11, 37)) < 0.4)).astype(np.float32)
    w = synth.kaiming_normal(42, 16, 3) * np.float32(1.5)
    par, g, ref = check_layer(x, w, K=K, beta=0.9, theta=1.0, mode=mode, precision=precision, kernel=api.TAC_KERNEL_DIRECT)
    assert ref[0].sum() > 0
    # frames of zeros and ones given as reals are the spike layer
    s = (r.random((8, 2, 3, 11, 37)) < 0.3).astype(np.uint8)
    a = run_gpu(s, w, K=K, beta=0.9, theta=1.0, mode=mode, precision=precision, kernel=api.TAC_KERNEL_DIRECT)
    b = run_gpu(s.astype(np.float32), w, K=K, beta=0.9, theta=1.0, mode=mode, precision=precision, kernel=api.TAC_KERNEL_DIRECT)
    assert np.array_equal(a["packed"], b["packed"]) and np.abs(a["v_trace"] - b["v_trace"]).max() < 1e-5


def test_bf16_aggregates_of_sixteen_frames_are_summed_exactly():
    # With bf16 operands every A_k is rounded once, after the sum over the frames (Eq. 2).  A chain of fp32 additions
    # over 16 frames can land on the other side of a bf16 rounding boundary than the exact sum does; the membranes
    # of the 9 x Cout neurons around such an element are then off by one bf16 step of A_k times a weight (this very
    # input did that: 1399 membranes of the first group off by up to 8e-3).  The kernel therefore sums in the 2^-23
    # fixed point of the matrix-core kernels and rounds once.  128-pixel rows: the vector kernel takes this shape.
    r = _rng(1400 + 32 + 128 + 14 + 128 + 16 + 23)
    s = (r.random((23, 3, 32, 14, 128)) < 0.15).astype(np.uint8)[:16]
    w = synth.kaiming_normal(43, 128, 32) * np.float32(1.5)
    bias = (r.standard_normal(128) * 0.1).astype(np.float32)
    par, g, ref = check_layer(s, w, K=16, beta=0.9, theta=1.0, mode=api.TAC_COLLAPSE, precision=api.TAC_BF16, bias=bias,
                              v0=np.zeros((3, 128, 14, 128), np.float32), expect_kernel=api.TAC_KERNEL_DIRECT)
    assert par.max_err < 1e-4, par
