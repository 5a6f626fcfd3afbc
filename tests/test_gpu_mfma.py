"""GPU parity of the bf16 MFMA implicit-GEMM kernel family against the CPU oracle."""
import numpy as np
import pytest
import torch

from paper_2603_13810_amd import api, synth

from gpu_util import check_layer, run_gpu, run_oracle
from parity_util import compare

pytestmark = pytest.mark.gpu

MODES = [(api.TAC_PER_STEP, 1), (api.TAC_COLLAPSE, 2), (api.TAC_COLLAPSE, 4), (api.TAC_PRESERVE, 2),
         (api.TAC_PRESERVE, 4), (api.TAC_COLLAPSE, 8), (api.TAC_PRESERVE, 16), (api.TAC_COLLAPSE, 3)]


def _rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


@pytest.mark.parametrize("mode,K", MODES)
def test_w64_tiles_and_ragged_rows(mode, K):
    # 10 rows = two full 4-row tiles and a ragged one; 32 input channels = two k-chunks
    r = _rng(100 + K)
    T = 48 if K in (16, 3) else 8
    s = (r.random((T, 2, 32, 10, 64)) < 0.15).astype(np.uint8)
    w = synth.kaiming_normal(11, 128, 32)
    bias = (r.standard_normal(128) * 0.1).astype(np.float32)
    v0 = (r.standard_normal((2, 128, 10, 64)) * 0.3).astype(np.float32)
    par, g, ref = check_layer(s, w, K=K, beta=0.9, theta=1.0, mode=mode, precision=api.TAC_BF16,
                              bias=bias, v0=v0, expect_kernel=api.TAC_KERNEL_MFMA)
    assert ref[0].sum() > 0
    print("mfma", api.MODE_NAMES[mode], K, par)


def test_two_cout_tiles_no_bias_no_state():
    r = _rng(7)
    s = (r.random((4, 1, 16, 4, 64)) < 0.2).astype(np.uint8)
    w = synth.kaiming_normal(12, 256, 16)
    par, g, ref = check_layer(s, w, K=2, beta=0.5, theta=1.0, mode=api.TAC_PRESERVE, precision=api.TAC_BF16,
                              expect_kernel=api.TAC_KERNEL_MFMA)
    g2 = run_gpu(s, w, K=2, beta=0.5, theta=1.0, mode=api.TAC_PRESERVE, precision=api.TAC_BF16, trace=False)
    assert np.array_equal(g["packed"], g2["packed"])


def test_mfma_matches_direct_kernel_on_same_operands():
    # both kernel families round W and A_k to bf16 the same way; their spikes should agree
    # except at near-threshold neurons (different fp32 summation order)
    r = _rng(8)
    s = (r.random((8, 1, 64, 8, 64)) < 0.1).astype(np.uint8)
    w = synth.kaiming_normal(13, 128, 64)
    kw = dict(K=4, beta=0.9, theta=1.0, mode=api.TAC_COLLAPSE, precision=api.TAC_BF16)
    a = run_gpu(s, w, kernel=api.TAC_KERNEL_MFMA, **kw)
    b = run_gpu(s, w, kernel=api.TAC_KERNEL_DIRECT, **kw)
    assert a["kernel"] == api.TAC_KERNEL_MFMA and b["kernel"] == api.TAC_KERNEL_DIRECT
    assert np.abs(a["v_trace"][0] - b["v_trace"][0]).max() < 1e-4
    assert (a["spikes"] != b["spikes"]).mean() < 1e-3


def test_state_carry_and_K1_equivalence():
    r = _rng(9)
    s = (r.random((8, 1, 16, 8, 64)) < 0.2).astype(np.uint8)
    w = synth.kaiming_normal(14, 128, 16)
    kw = dict(beta=0.9, theta=1.0, precision=api.TAC_BF16)
    ps = run_gpu(s, w, K=1, mode=api.TAC_PER_STEP, **kw)
    for mode in (api.TAC_COLLAPSE, api.TAC_PRESERVE):
        k1 = run_gpu(s, w, K=1, mode=mode, **kw)
        assert np.array_equal(ps["packed"], k1["packed"]) and np.array_equal(ps["v_trace"], k1["v_trace"])
    whole = run_gpu(s, w, K=2, mode=api.TAC_PRESERVE, **kw)
    a = run_gpu(s[:4], w, K=2, mode=api.TAC_PRESERVE, **kw)
    b = run_gpu(s[4:], w, K=2, mode=api.TAC_PRESERVE, v0=a["v_final"], **kw)
    assert np.array_equal(np.concatenate([a["packed"], b["packed"]]), whole["packed"])
    assert np.array_equal(b["v_final"], whole["v_final"])


# (input width, stride, input rows): the rows give at least one full tile and a ragged one
# (tiles are 8 output rows for output width 32, 16 rows for output width 16), odd and even
GEOMETRIES = [(32, 1, 11), (64, 2, 21), (64, 2, 18), (32, 2, 35), (32, 2, 38)]
GEO_MODES = [(api.TAC_PER_STEP, 1), (api.TAC_COLLAPSE, 2), (api.TAC_PRESERVE, 4), (api.TAC_COLLAPSE, 4)]


@pytest.mark.parametrize("W,stride,H", GEOMETRIES)
@pytest.mark.parametrize("mode,K", GEO_MODES)
def test_other_geometries(W, stride, H, mode, K):
    # width 32 and stride 2: a wave's 64 pixels fold into 2 or 4 output rows
    r = _rng(1000 + 10 * W + stride + H + K)
    s = (r.random((8, 2, 32, H, W)) < 0.15).astype(np.uint8)
    w = synth.kaiming_normal(21, 128, 32)
    bias = (r.standard_normal(128) * 0.1).astype(np.float32)
    Ho, Wo = (H - 1) // stride + 1, W // stride
    v0 = (r.standard_normal((2, 128, Ho, Wo)) * 0.3).astype(np.float32)
    par, g, ref = check_layer(s, w, K=K, beta=0.9, theta=1.0, mode=mode, stride=stride, precision=api.TAC_BF16,
                              bias=bias, v0=v0, expect_kernel=api.TAC_KERNEL_MFMA)
    assert ref[0].sum() > 0
    print("mfma W=%d stride=%d H=%d" % (W, stride, H), api.MODE_NAMES[mode], K, par)


@pytest.mark.parametrize("K", [8, 16, 5])
def test_width_32_larger_K(K):
    r = _rng(1200 + K)
    s = (r.random((80 if K == 5 else 32, 1, 16, 9, 32)) < 0.1).astype(np.uint8)
    w = synth.kaiming_normal(22, 256, 16)
    check_layer(s, w, K=K, beta=0.9, theta=1.0, mode=api.TAC_PRESERVE, precision=api.TAC_BF16,
                expect_kernel=api.TAC_KERNEL_MFMA)


def test_stride_2_large_K_leaves_the_large_kernel():
    # the stride-2 tiles of the large kernel have LDS room for 4 frames; larger groups go to the
    # kernel for the shapes in between (still on the matrix cores) and stay correct
    r = _rng(1300)
    s = (r.random((16, 1, 16, 12, 64)) < 0.2).astype(np.uint8)
    w = synth.kaiming_normal(23, 128, 16)
    check_layer(s, w, K=8, beta=0.9, theta=1.0, mode=api.TAC_COLLAPSE, stride=2, precision=api.TAC_BF16,
                expect_kernel=api.TAC_KERNEL_MFMA)
    d = api.make_desc(16, 1, 256, 16, 64, 128, K=8, beta=0.9, theta=1.0, mode=api.TAC_COLLAPSE, stride=2,
                      precision=api.TAC_BF16)
    assert api.tac_select_kernel(d) == api.TAC_KERNEL_DIRECT      # 256 input channels: neither of them


# ---- the short-contraction member of the family (Cin = 1 or 2: first layers)
# (Cin, Cout, H, W, stride): ragged rows and widths, one and two 32-channel blocks, partial blocks, several
# channel tiles (Cout > 64), output rows of more than 64 pixels (two waves per row, odd row counts)
SMALL_SHAPES = [(1, 8, 28, 28, 1), (1, 32, 13, 28, 1), (2, 64, 22, 128, 2), (2, 40, 9, 64, 1), (1, 64, 11, 50, 2),
                (2, 24, 7, 33, 1), (2, 64, 6, 127, 2), (2, 128, 9, 128, 1), (2, 96, 7, 100, 1), (1, 160, 5, 70, 2),
                (1, 16, 6, 65, 1)]
SMALL_MODES = [(api.TAC_PER_STEP, 1), (api.TAC_COLLAPSE, 2), (api.TAC_PRESERVE, 4), (api.TAC_COLLAPSE, 3)]


@pytest.mark.parametrize("shape", SMALL_SHAPES)
@pytest.mark.parametrize("mode,K", SMALL_MODES)
def test_short_contraction_kernel(shape, mode, K):
    Cin, Cout, H, W, stride = shape
    r = _rng(2000 + Cin + Cout + H + W + stride + K)
    s = (r.random((12, 2, Cin, H, W)) < 0.3).astype(np.uint8)
    w = synth.kaiming_normal(31, Cout, Cin)
    bias = (r.standard_normal(Cout) * 0.1).astype(np.float32)
    Ho, Wo = (H - 1) // stride + 1, (W - 1) // stride + 1
    v0 = (r.standard_normal((2, Cout, Ho, Wo)) * 0.3).astype(np.float32)
    par, g, ref = check_layer(s, w, K=K, beta=0.9, theta=1.0, mode=mode, stride=stride, precision=api.TAC_BF16,
                              bias=bias, v0=v0, expect_kernel=api.TAC_KERNEL_MFMA)
    assert ref[0].sum() > 0
    print("short contraction", shape, api.MODE_NAMES[mode], K, par)


def test_short_contraction_limits():
    mk = lambda **kw: api.make_desc(8, 1, kw.pop("Cin", 2), 16, kw.pop("W", 128), kw.pop("Cout", 64), K=kw.pop("K", 2), beta=0.9,
                                    theta=1.0, mode=api.TAC_COLLAPSE, stride=kw.pop("stride", 2), precision=api.TAC_BF16)
    assert api.tac_select_kernel(mk()) == api.TAC_KERNEL_MFMA
    assert api.tac_select_kernel(mk(stride=1)) == api.TAC_KERNEL_MFMA            # 128 output pixels per row
    assert api.tac_select_kernel(mk(Cout=96)) == api.TAC_KERNEL_MFMA             # more than one channel tile
    assert api.tac_select_kernel(mk(Cin=3)) == api.TAC_KERNEL_DIRECT
    assert api.tac_select_kernel(mk(W=160, stride=2)) == api.TAC_KERNEL_DIRECT


def test_short_contraction_state_carry_and_no_trace():
    r = _rng(77)
    s = (r.random((8, 1, 2, 12, 96)) < 0.2).astype(np.uint8)
    w = synth.kaiming_normal(32, 48, 2)
    kw = dict(beta=0.5, theta=1.0, stride=2, precision=api.TAC_BF16)
    whole = run_gpu(s, w, K=2, mode=api.TAC_PRESERVE, **kw)
    plain = run_gpu(s, w, K=2, mode=api.TAC_PRESERVE, trace=False, **kw)
    assert whole["kernel"] == api.TAC_KERNEL_MFMA and np.array_equal(whole["packed"], plain["packed"])
    a = run_gpu(s[:4], w, K=2, mode=api.TAC_PRESERVE, **kw)
    b = run_gpu(s[4:], w, K=2, mode=api.TAC_PRESERVE, v0=a["v_final"], **kw)
    assert np.array_equal(np.concatenate([a["packed"], b["packed"]]), whole["packed"])
    assert np.array_equal(b["v_final"], whole["v_final"])


# ---- max pool on load (the MaxPool(2) between the blocks of the event-data network)

@pytest.mark.parametrize("W,H", [(64, 10), (32, 19)])
@pytest.mark.parametrize("mode,K", [(api.TAC_PER_STEP, 1), (api.TAC_COLLAPSE, 2), (api.TAC_PRESERVE, 4), (api.TAC_COLLAPSE, 4)])
def test_max_pool_on_load_mfma(W, H, mode, K):
    r = _rng(3000 + W + H + K)
    s = (r.random((8, 2, 32, 2 * H, 2 * W)) < 0.06).astype(np.uint8)          # unpooled spikes of the layer before
    w = synth.kaiming_normal(51, 128, 32)
    bias = (r.standard_normal(128) * 0.1).astype(np.float32)
    par, g, ref = check_layer(s, w, K=K, beta=0.9, theta=1.0, mode=mode, pool2="max", precision=api.TAC_BF16, bias=bias,
                              expect_kernel=api.TAC_KERNEL_MFMA)
    assert ref[0].sum() > 0 and g["spikes"].shape[-2:] == (H, W)
    d = run_gpu(s, w, K=K, beta=0.9, theta=1.0, mode=mode, pool2="max", precision=api.TAC_BF16, bias=bias,
                kernel=api.TAC_KERNEL_DIRECT, trace=False)
    assert (d["spikes"] != g["spikes"]).mean() < 1e-3                           # the two kernel families agree
    print("max pool on load W=%d H=%d" % (W, H), api.MODE_NAMES[mode], K, par)


def test_max_pool_on_load_limits():
    mk = lambda **kw: api.make_desc(8, 1, 32, 16, 64, 128, K=kw.pop("K", 2), beta=0.9, theta=1.0, mode=api.TAC_COLLAPSE,
                                    stride=kw.pop("stride", 1), precision=api.TAC_BF16, in_format=api.TAC_IN_BITS_MAXPOOL2)
    assert api.tac_select_kernel(mk()) == api.TAC_KERNEL_MFMA
    # 32 input channels: the kernel for the shapes in between takes what the large one does not
    assert api.tac_select_kernel(mk(K=8)) == api.TAC_KERNEL_MFMA
    assert api.tac_select_kernel(mk(stride=2)) == api.TAC_KERNEL_MFMA


def test_conv_bn_lif_maxpool_blocks_stay_packed():
    # three blocks Conv -> BN -> LIF -> MaxPool(2) of the event-data network shape (Sec. 5.1) at a
    # reduced width: batch norm folded on the device, every inter-layer tensor packed bits, the pool
    # applied by the next layer's loader; teacher-forced against the oracle layer by layer
    import oracle
    r = _rng(3100)
    dev = torch.device("cuda:0")
    x = (r.random((4, 1, 2, 64, 128)) < 0.1).astype(np.uint8)
    chans = [(2, 32), (32, 128), (128, 128)]
    fmt = [False, "max", "max"]
    for li, (ci, co) in enumerate(chans):
        w = synth.kaiming_normal(60 + li, co, ci) * np.float32(2.0)
        g_, b_ = r.uniform(0.8, 1.2, co).astype(np.float32), (r.standard_normal(co) * 0.05).astype(np.float32)
        mean, var = (r.standard_normal(co) * 0.05).astype(np.float32), r.uniform(0.8, 1.2, co).astype(np.float32)
        t = lambda a: torch.from_numpy(a).to(dev)
        wf, bf = api.tac_fold_batchnorm(t(w), None, t(g_), t(b_), t(mean), t(var), eps=1e-5)
        rw, rb = oracle.fold_batchnorm(w, None, g_, b_, mean, var, eps=float(np.float32(1e-5)))
        assert np.abs(wf.cpu().numpy() - rw).max() < 1e-6
        # both sides take the device's folded fp32 weights from here on
        wq, bq = wf.cpu().numpy(), bf.cpu().numpy()
        par, g, ref = check_layer(x, wq, K=2, beta=0.5, theta=1.0, mode=api.TAC_PRESERVE, pool2=fmt[li], bias=bq,
                                  precision=api.TAC_BF16)
        assert ref[0].mean() > 0.002, "layer %d is silent" % (li + 1)
        print("block %d %s: %s rate %.3f" % (li + 1, "mfma" if g["kernel"] == api.TAC_KERNEL_MFMA else "direct", par, ref[0].mean()))
        x = ref[0]                                                               # unpooled spikes, pooled by the next loader
    assert x.shape == (4, 1, 128, 16, 32)


# ---- real-valued input frames (the continuous-valued first layer, Sec. 4.2)

@pytest.mark.parametrize("shape", [(2, 64, 22, 128, 2), (1, 32, 13, 28, 1), (2, 40, 9, 64, 1), (2, 128, 6, 128, 1)])
@pytest.mark.parametrize("mode,K", [(api.TAC_PER_STEP, 1), (api.TAC_COLLAPSE, 2), (api.TAC_PRESERVE, 4), (api.TAC_COLLAPSE, 3)])
def test_real_valued_frames_short_contraction_kernel(shape, mode, K):
    Cin, Cout, H, W, stride = shape
    r = _rng(4000 + Cin + Cout + H + W + K)
    # normalised event counts: mostly zero, some values in (0, 1]
    x = (r.random((12, 2, Cin, H, W)) * (r.random((12, 2, Cin, H, W)) < 0.3)).astype(np.float32)
    w = synth.kaiming_normal(71, Cout, Cin) * np.float32(1.5)
    bias = (r.standard_normal(Cout) * 0.1).astype(np.float32)
    par, g, ref = check_layer(x, w, K=K, beta=0.9, theta=1.0, mode=mode, stride=stride, precision=api.TAC_BF16, bias=bias,
                              expect_kernel=api.TAC_KERNEL_MFMA)
    assert ref[0].sum() > 0
    print("real-valued frames", shape, api.MODE_NAMES[mode], K, par)


# ---- tile choice: 64 output channels per workgroup on small grids, 128 on grids that fill the chip

@pytest.mark.parametrize("W,stride,H,reps", [(64, 1, 10, 48), (32, 1, 11, 72), (64, 2, 21, 72), (32, 2, 35, 136)])
@pytest.mark.parametrize("mode,K", [(api.TAC_PER_STEP, 1), (api.TAC_COLLAPSE, 4), (api.TAC_PRESERVE, 2)])
def test_full_grid_uses_128_channel_tiles(W, stride, H, reps, mode, K):
    # the other tests have a handful of workgroups and get 64-channel tiles; here the same two
    # samples are repeated until the 128-channel grid has at least 256 workgroups
    r = _rng(5000 + W + stride + H + K)
    s = (r.random((8, 2, 32, H, W)) < 0.15).astype(np.uint8)
    w = synth.kaiming_normal(81, 128, 32)
    bias = (r.standard_normal(128) * 0.1).astype(np.float32)
    kw = dict(K=K, beta=0.9, theta=1.0, mode=mode, stride=stride, bias=bias)
    small = run_gpu(s, w, precision=api.TAC_BF16, **kw)           # 64-channel tiles
    ref = run_oracle(s, w, quantised=True, **kw)
    par = compare(ref[0], ref[1], small["spikes"], small["v_trace"], 1.0, 1e-3)
    assert par.ok, par
    big = run_gpu(np.tile(s, (1, reps, 1, 1, 1)), w, precision=api.TAC_BF16, **kw)        # 128-channel tiles
    rows = {64: 4, 32: 8, 16: 16}[W // stride]
    assert (-(-small["spikes"].shape[-2] // rows)) * 2 * reps >= 256
    for i in range(0, 2 * reps, 2):
        # same operands, same summation order within a tile: the two tile sizes agree bit for bit
        assert np.array_equal(big["packed"][:, i:i + 2], small["packed"]), i
    assert np.array_equal(big["v_trace"][:, :2], small["v_trace"])


@pytest.mark.parametrize("Cin,Cout,W,stride,H,reps", [(128, 128, 64, 1, 10, 48), (256, 256, 32, 2, 35, 34), (128, 256, 32, 1, 11, 36)])
@pytest.mark.parametrize("mode,K", [(api.TAC_PER_STEP, 1), (api.TAC_PRESERVE, 2), (api.TAC_PRESERVE, 4)])
def test_tile_sizes_agree_on_deep_layers(Cin, Cout, W, stride, H, reps, mode, K):
    # the channel counts of the five-layer event stack (128 -> 128 at stride 2 and 1, 256 -> 256 at stride 2): the
    # 64-channel and half-height tiles of a small batch against the 128-channel tiles of a grid that fills the chip
    r = _rng(5100 + Cin + Cout + W + stride + K)
    s = (r.random((8, 2, Cin, H, W)) < 0.1).astype(np.uint8)
    w = synth.kaiming_normal(82, Cout, Cin) * np.float32(1.5)
    bias = (r.standard_normal(Cout) * 0.1).astype(np.float32)
    kw = dict(K=K, beta=0.5, theta=1.0, mode=mode, stride=stride, bias=bias)
    par, small, ref = check_layer(s, w, precision=api.TAC_BF16, expect_kernel=api.TAC_KERNEL_MFMA, **kw)     # small tiles
    assert ref[0].mean() > 0.01
    big = run_gpu(np.tile(s, (1, reps, 1, 1, 1)), w, precision=api.TAC_BF16, **kw)        # 128-channel tiles
    rows = {64: 4, 32: 8, 16: 16}[W // stride]
    assert (-(-small["spikes"].shape[-2] // rows)) * (Cout // 128) * 2 * reps >= 256
    for i in range(0, 2 * reps, 2):
        assert np.array_equal(big["packed"][:, i:i + 2], small["packed"]), i
    assert np.array_equal(big["v_trace"][:, :2], small["v_trace"])
    print("tile sizes, deep layers", (Cin, Cout, W, stride, H), api.MODE_NAMES[mode], K, par)


# ---- the kernel for the shapes in between (Cin a multiple of 8 up to 64, any pool on load)
# (Cin, Cout, H, W, stride, pool)
MID_SHAPES = [(32, 64, 14, 14, 1, True), (8, 32, 9, 50, 1, False), (16, 96, 11, 64, 2, False), (64, 24, 7, 20, 1, "max"),
              (24, 64, 10, 128, 2, False), (40, 160, 6, 33, 1, True), (128, 128, 16, 16, 1, "max"), (128, 64, 8, 8, 1, False)]
MID_MODES = [(api.TAC_PER_STEP, 1), (api.TAC_COLLAPSE, 2), (api.TAC_PRESERVE, 4), (api.TAC_COLLAPSE, 3), (api.TAC_PRESERVE, 8)]


@pytest.mark.parametrize("shape", MID_SHAPES)
@pytest.mark.parametrize("mode,K", MID_MODES)
def test_in_between_kernel(shape, mode, K):
    Cin, Cout, H, W, stride, pool = shape
    r = _rng(6000 + Cin + Cout + H + W + stride + K)
    f = 2 if pool else 1
    s = (r.random((24, 2, Cin, f * H, f * W)) < 0.12).astype(np.uint8)
    w = synth.kaiming_normal(91, Cout, Cin) * np.float32(1.5)
    bias = (r.standard_normal(Cout) * 0.1).astype(np.float32)
    Ho, Wo = (H - 1) // stride + 1, (W - 1) // stride + 1
    v0 = (r.standard_normal((2, Cout, Ho, Wo)) * 0.3).astype(np.float32)
    par, g, ref = check_layer(s, w, K=K, beta=0.9, theta=1.0, mode=mode, stride=stride, pool2=pool, precision=api.TAC_BF16,
                              bias=bias, v0=v0, expect_kernel=api.TAC_KERNEL_MFMA)
    assert ref[0].sum() > 0
    print("in-between kernel", shape, api.MODE_NAMES[mode], K, par)


# ---- the in-between kernel in fp32 (float32 operands on the matrix cores), held to the fp32 bar of 1e-5
# (Cin, Cout, H, W, stride, pool)
MID_F32_SHAPES = [(32, 64, 14, 14, 1, True), (8, 32, 9, 50, 1, False), (16, 96, 11, 64, 2, False), (24, 20, 7, 20, 1, "max"),
                  (40, 64, 6, 33, 1, True), (32, 64, 10, 40, 1, False)]


@pytest.mark.parametrize("shape", MID_F32_SHAPES)
@pytest.mark.parametrize("mode,K", [(api.TAC_PER_STEP, 1), (api.TAC_COLLAPSE, 2), (api.TAC_PRESERVE, 4), (api.TAC_COLLAPSE, 3), (api.TAC_COLLAPSE, 8)])
def test_in_between_kernel_fp32(shape, mode, K):
    Cin, Cout, H, W, stride, pool = shape
    r = _rng(6500 + Cin + Cout + H + W + stride + K)
    f = 2 if pool else 1
    s = (r.random((16, 2, Cin, f * H, f * W)) < 0.15).astype(np.uint8)
    w = synth.kaiming_normal(92, Cout, Cin) * np.float32(1.5)
    bias = (r.standard_normal(Cout) * 0.1).astype(np.float32)
    Ho, Wo = (H - 1) // stride + 1, (W - 1) // stride + 1
    v0 = (r.standard_normal((2, Cout, Ho, Wo)) * 0.3).astype(np.float32)
    par, g, ref = check_layer(s, w, K=K, beta=0.9, theta=1.0, mode=mode, stride=stride, pool2=pool, precision=api.TAC_FP32,
                              bias=bias, v0=v0, expect_kernel=api.TAC_KERNEL_MFMA)
    assert ref[0].sum() > 0 and par.max_err < 1e-5
    print("in-between kernel fp32", shape, api.MODE_NAMES[mode], K, par)


def test_fp32_layers_outside_the_in_between_shapes_stay_on_the_vector_kernel():
    mk = lambda **kw: api.make_desc(8, 2, kw.pop("Cin", 32), 16, kw.pop("W", 16), kw.pop("Cout", 64), K=2, beta=0.9, theta=1.0,
                                    mode=api.TAC_COLLAPSE, precision=api.TAC_FP32, **kw)
    assert api.tac_select_kernel(mk()) == api.TAC_KERNEL_MFMA
    assert api.tac_select_kernel(mk(Cin=1)) == api.TAC_KERNEL_DIRECT            # first layers
    assert api.tac_select_kernel(mk(Cin=12)) == api.TAC_KERNEL_DIRECT           # not a multiple of 8
    assert api.tac_select_kernel(mk(Cin=128, Cout=128)) == api.TAC_KERNEL_DIRECT   # float32 weights of the tile exceed the LDS
    assert api.tac_select_kernel(mk(kernel=api.TAC_KERNEL_DIRECT)) == api.TAC_KERNEL_DIRECT
