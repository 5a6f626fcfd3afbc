"""Sequences whose length is not a multiple of K (Sec. 5 runs T = 25 with K = 4, 8, 16; App. A assumes K | T):
the frames left over form a shorter last group.  Every kernel family against the oracle, through the C ABI."""
import numpy as np
import pytest
import torch


from paper_2603_13810_amd import api, synth
from gpu_util import check_layer, run_gpu, run_oracle

pytestmark = pytest.mark.gpu

B16, F32 = api.TAC_BF16, api.TAC_FP32
MFMA, DIRECT = api.TAC_KERNEL_MFMA, api.TAC_KERNEL_DIRECT
# (name, Cin, Cout, H, W, stride, pool, precision, kernel family expected)
SHAPES = [
    ("long contraction", 32, 128, 12, 32, 1, False, B16, MFMA),
    ("long contraction, 64 wide", 16, 128, 9, 64, 1, False, B16, MFMA),
    ("max pool on load", 16, 128, 8, 32, 1, "max", B16, MFMA),
    ("stride 2", 16, 128, 10, 64, 2, False, B16, MFMA),
    ("short contraction", 2, 64, 9, 40, 1, False, B16, MFMA),
    ("in between, mean pool", 8, 32, 9, 50, 1, True, B16, MFMA),
    ("vector kernel fp32", 3, 5, 7, 9, 1, False, F32, DIRECT),
    ("vector kernel bf16", 3, 40, 7, 33, 2, False, B16, DIRECT),
]
# (T, K): one frame left over, several left over, T = 25 as in the paper's runs, a group longer than the sequence
TK = [(7, 2), (11, 4), (7, 3), (25, 8), (25, 16), (3, 8)]


def _rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


@pytest.mark.parametrize("shape", SHAPES, ids=[s[0] for s in SHAPES])
@pytest.mark.parametrize("T,K", TK)
@pytest.mark.parametrize("mode", [api.TAC_COLLAPSE, api.TAC_PRESERVE])
def test_shorter_last_group(shape, T, K, mode):
    name, Cin, Cout, H, W, stride, pool, precision, family = shape
    r = _rng(9000 + Cin + Cout + H + W + T + K)
    f = 2 if pool else 1
    s = (r.random((T, 2, Cin, f * H, f * W)) < (0.12 if Cin > 2 else 0.3)).astype(np.uint8)
    w = synth.kaiming_normal(17, Cout, Cin) * np.float32(1.5)
    bias = (r.standard_normal(Cout) * 0.1).astype(np.float32)
    Ho, Wo = (H - 1) // stride + 1, (W - 1) // stride + 1
    v0 = (r.standard_normal((2, Cout, Ho, Wo)) * 0.3).astype(np.float32)
    api.tac_reset_counters()
    par, g, ref = check_layer(s, w, K=K, beta=0.9, theta=1.0, mode=mode, stride=stride, pool2=pool, precision=precision,
                              bias=bias, v0=v0, expect_kernel=family)
    n_groups = -(-T // min(K, T))
    assert g["spikes"].shape[0] == (n_groups if mode == api.TAC_COLLAPSE else T)
    # two calls: with and without the membrane trace
    assert api.tac_get_counters() == (2 * n_groups, 2 * (n_groups if mode == api.TAC_COLLAPSE else T))
    assert ref[0].sum() > 0 and ref[0][-1].sum() > 0          # the last group's step fires somewhere
    print("shorter last group:", name, "T=%d K=%d" % (T, K), api.MODE_NAMES[mode], par)


@pytest.mark.parametrize("T,K", [(7, 2), (11, 4), (9, 8)])
@pytest.mark.parametrize("mode", [api.TAC_COLLAPSE, api.TAC_PRESERVE])
def test_shorter_last_group_real_valued_frames(T, K, mode):
    r = _rng(9500 + T + K)
    x = (r.random((T, 2, 2, 9, 40)) * (r.random((T, 2, 2, 9, 40)) < 0.3)).astype(np.float32)
    w = synth.kaiming_normal(18, 48, 2) * np.float32(1.5)
    for precision, family in ((B16, MFMA), (F32, DIRECT)):
        par, g, ref = check_layer(x, w, K=K, beta=0.9, theta=1.0, mode=mode, precision=precision, expect_kernel=family,
                                  )
        assert ref[0][-1].sum() > 0
        print("shorter last group, real-valued frames T=%d K=%d" % (T, K), api.MODE_NAMES[mode], par)


def test_group_longer_than_the_sequence_is_one_group_of_T_frames():
    r = _rng(9600)
    s = (r.random((3, 2, 16, 8, 32)) < 0.15).astype(np.uint8)
    w = synth.kaiming_normal(19, 128, 16) * np.float32(1.5)
    kw = dict(beta=0.9, theta=1.0, mode=api.TAC_COLLAPSE, precision=B16)
    a, b = run_gpu(s, w, K=8, **kw), run_gpu(s, w, K=3, **kw)
    assert np.array_equal(a["packed"], b["packed"]) and np.array_equal(a["v_trace"], b["v_trace"])
    assert np.array_equal(a["v_final"], b["v_final"])


def test_shorter_last_group_needs_the_state_buffer():
    # the last group is a launch of its own; without v_inout the membrane could not reach it
    r = _rng(9700)
    s = (r.random((7, 1, 2, 8, 32)) < 0.3).astype(np.uint8)
    w = synth.kaiming_normal(20, 8, 2)
    with pytest.raises(Exception) as e:
        run_gpu(s, w, K=2, beta=0.9, theta=1.0, mode=api.TAC_COLLAPSE, trace=False)
    assert "v_inout" in str(e.value)
    ok = run_gpu(s, w, K=2, beta=0.9, theta=1.0, mode=api.TAC_COLLAPSE, trace=False, v0=np.zeros((1, 8, 8, 32), np.float32))
    ref = run_oracle(s, w, K=2, beta=0.9, theta=1.0, mode=api.TAC_COLLAPSE)
    assert np.array_equal(ok["spikes"], ref[0])
