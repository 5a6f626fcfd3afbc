"""MaxPool(2) of the output spikes in the layer that writes them (the Conv -> BN -> LIF -> MaxPool(2) blocks of the
event-data network, Sec. 5.1): every matrix-core kernel, then the whole five-block stack, against the oracle."""
import numpy as np
import pytest
import torch

import oracle
from paper_2603_13810_amd import api, synth

from gpu_util import check_layer, run_gpu, run_oracle, ORACLE_MODE
from parity_util import np_pack, np_unpack

pytestmark = pytest.mark.gpu
DEV = torch.device("cuda:0")
MODES = [(api.TAC_PER_STEP, 1), (api.TAC_COLLAPSE, 2), (api.TAC_PRESERVE, 4), (api.TAC_COLLAPSE, 8), (api.TAC_PRESERVE, 3)]

# (Cin, Cout, H, W): which kernel takes it
SHAPES = [(32, 128, 10, 64, "large, rows of 64"), (32, 256, 12, 32, "large, two rows per wave"), (128, 128, 16, 32, "large, half tiles"),
          (2, 128, 64, 64, "short contraction"), (2, 40, 6, 128, "short contraction, rows of 128"), (1, 32, 28, 28, "short contraction, ragged"),
          (128, 128, 16, 16, "in between"), (128, 128, 4, 4, "in between, 4 x 4"), (64, 96, 8, 8, "in between, 96 channels"),
          (24, 64, 10, 50, "in between, ragged")]


@pytest.mark.parametrize("shape", SHAPES, ids=[s[4] for s in SHAPES])
@pytest.mark.parametrize("mode,K", MODES)
def test_pooled_output_of_every_matrix_core_kernel(shape, mode, K):
    Cin, Cout, H, W, _ = shape
    r = np.random.Generator(np.random.PCG64(8000 + Cin + Cout + H + W + K))
    T = 6 if K == 3 else 8
    if mode == api.TAC_PRESERVE and K == 3:
        T = 7                                                   # a shorter last group as well
    s = (r.random((T, 2, Cin, H, W)) < (0.3 if Cin <= 2 else 0.12)).astype(np.uint8)
    w = synth.kaiming_normal(93, Cout, Cin) * np.float32(1.5)
    bias = (r.standard_normal(Cout) * 0.1).astype(np.float32)
    v0 = (r.standard_normal((2, Cout, H, W)) * 0.3).astype(np.float32)
    par, g, ref = check_layer(s, w, K=K, beta=0.9, theta=1.0, mode=mode, precision=api.TAC_BF16, bias=bias, v0=v0,
                              expect_kernel=api.TAC_KERNEL_MFMA, out_pool=True)
    pooled_ref = oracle.maxpool2(ref[0]).astype(np.uint8)
    assert pooled_ref.mean() > 0.02
    diff = int((pooled_ref != g["pooled"]).sum())
    assert diff <= 4 * par.flips, "pooled spikes differ from the oracle's at %d places with %d tolerated flips" % (diff, par.flips)
    print("pooled output", shape[4], api.MODE_NAMES[mode], K, par)


def test_five_block_event_stack_conv_bn_lif_maxpool():
    """The event-data network of Sec. 5.1: five Conv -> BN -> LIF -> MaxPool(2) blocks, 2 -> 128 -> 128 -> 128 -> 128
    -> 128 channels, 64 -> 32 -> 16 -> 8 -> 4 -> 2 pixels, T = 16, TAC-TP with K = 2 in every block.  The batch norm is
    folded into weights and bias by the library; every block pools its own output.  Teacher forcing: block l is fed the
    ORACLE's pooled spikes of block l - 1; next to it the same five blocks run as one stack call on the library's own
    spikes."""
    r = np.random.Generator(np.random.PCG64(8100))
    T, B, K = 16, 2, 2
    chans = [2, 128, 128, 128, 128, 128]
    x_ref = synth.event_camera(8101, T, B, 64, 64, 2, base_rate=0.05)
    x0 = x_ref
    layers = []
    H = 64
    for l in range(5):
        Cin, Cout = chans[l], chans[l + 1]
        w = synth.kaiming_normal(8110 + l, Cout, Cin) * np.float32(2.0)
        gamma = (1.0 + 0.2 * r.standard_normal(Cout)).astype(np.float32)
        beta_bn = (0.1 * r.standard_normal(Cout)).astype(np.float32)
        mean = (0.05 * r.standard_normal(Cout)).astype(np.float32)
        var = (0.8 + 0.4 * r.random(Cout)).astype(np.float32)
        # the library folds the batch norm (device), the oracle folds it in double (host)
        wf_d, bf_d = api.tac_fold_batchnorm(torch.from_numpy(w).to(DEV), None, torch.from_numpy(gamma).to(DEV),
                                            torch.from_numpy(beta_bn).to(DEV), torch.from_numpy(mean).to(DEV),
                                            torch.from_numpy(var).to(DEV), eps=1e-5)
        wf_o, bf_o = oracle.fold_batchnorm(w, None, gamma, beta_bn, mean, var, eps=1e-5)
        wf, bf = wf_d.cpu().numpy(), bf_d.cpu().numpy()
        assert np.allclose(wf, wf_o, rtol=1e-6, atol=1e-7) and np.allclose(bf, bf_o, rtol=1e-6, atol=1e-7)
        par, g, ref = check_layer(x_ref, wf, K=K, beta=0.5, theta=1.0, mode=api.TAC_PRESERVE, precision=api.TAC_BF16, bias=bf,
                                  expect_kernel=api.TAC_KERNEL_MFMA, out_pool=True)
        x_ref = oracle.maxpool2(ref[0]).astype(np.uint8)               # the oracle's own pool: the next block's input
        assert x_ref.shape == (T, B, Cout, H // 2, H // 2) and x_ref.mean() > 0.02, (l, x_ref.mean())
        print("five-block stack, block %d (%d -> %d at %d x %d):" % (l + 1, Cin, Cout, H, H), par, "pooled rate %.3f" % x_ref.mean())
        d = api.make_desc(T, B, Cin, H, H, Cout, K=K, beta=0.5, theta=1.0, mode=api.TAC_PRESERVE, precision=api.TAC_BF16,
                          out_format=api.TAC_OUT_BITS_MAXPOOL2)
        layers.append(dict(desc=d, w_prepared=api.tac_prepare_weights(d, wf_d), bias=bf_d))
        H //= 2
    assert x_ref.shape[-2:] == (2, 2)
    # free running: one stack call, every tensor between the blocks a quarter of the unpooled size
    stack, outs = api.make_stack(layers)
    assert api.tac_stack_check(stack) == (api.TAC_OK, -1)
    api.tac_reset_counters()
    api.tac_stack_forward(stack, torch.from_numpy(np_pack(x0)).to(DEV))
    torch.cuda.synchronize()
    assert api.tac_get_counters() == (5 * T // K, 5 * T)                 # 40 convolution stages at K = 2 (Table 3)
    assert [tuple(o.shape) for o in outs] == [(T, B, 128, 32, 1), (T, B, 128, 16, 1), (T, B, 128, 8, 1), (T, B, 128, 4, 1),
                                              (T, B, 128, 2, 1)]
    free = np_unpack(outs[-1].cpu().numpy(), 2)
    print("five-block stack, free running: last block differs from the teacher-forced oracle at %.2e of its bits" %
          float((free != x_ref).mean()))
