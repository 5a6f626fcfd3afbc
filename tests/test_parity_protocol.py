"""CPU checks of the comparison protocol itself (tests/parity_util.py): the three-way comparison of the
bf16 path must accept a result that is the rounded oracle's own, and must catch a spike or a membrane
that leaves the plain oracle by more than the operand rounding does."""
import numpy as np
import torch

import oracle
from parity_util import compare, compare3


def _two_oracles(mode, K):
    r = np.random.Generator(np.random.PCG64(77))
    s = (r.random((8, 2, 16, 6, 6)) < 0.3).astype(np.uint8)
    w = (r.standard_normal((8, 16, 3, 3)) * np.sqrt(2.0 / 144) * 1.5).astype(np.float32)
    wq = torch.from_numpy(w).to(torch.bfloat16).to(torch.float32).numpy()
    kw = dict(K=K, beta=float(np.float32(0.9)), theta=1.0, mode=mode)
    plain = oracle.conv_lif(s, w.astype(np.float64), **kw)
    rounded = oracle.conv_lif(s, wq.astype(np.float64), round_a_bf16=True, **kw)
    return plain, rounded


def test_rounded_oracle_itself_is_within_the_rounding():
    for mode, K in ((oracle.TAC, 4), (oracle.TAC_TP, 4)):
        plain, rounded = _two_oracles(mode, K)
        p3 = compare3(plain[:2], rounded[:2], rounded[0], rounded[1], 1.0, 1e-3)
        assert p3.vs_rounded.ok and p3.vs_rounded.max_err == 0 and p3.bounded and p3.extra_mismatches == 0
        # what the library is charged with against the plain oracle is exactly the rounding's own
        assert (p3.vs_plain.mismatches, p3.vs_plain.flips) == (p3.quant.mismatches, p3.quant.flips)


def test_planted_spike_far_from_threshold_is_caught():
    plain, rounded = _two_oracles(oracle.TAC_TP, 2)
    spk = rounded[0].copy()
    v = rounded[1]
    far = np.argwhere((np.abs(v - 1.0) > 0.2) & (spk == plain[0]))
    t, b, c, y, x = far[len(far) // 2]
    spk[t, b, c, y, x] ^= 1
    p3 = compare3(plain[:2], rounded[:2], spk, rounded[1], 1.0, 1e-3)
    assert p3.vs_rounded.mismatches == 1 and not p3.vs_rounded.ok


def test_planted_membrane_error_is_caught():
    plain, rounded = _two_oracles(oracle.TAC, 2)
    v = rounded[1].copy()
    v[1, 0, 3, 2, 2] += 5e-3 * max(abs(plain[1][1, 0, 3, 2, 2]), 1.0) * (1 if rounded[1][1, 0, 3, 2, 2] >= plain[1][1, 0, 3, 2, 2] else -1)
    p3 = compare3(plain[:2], rounded[:2], rounded[0], v, 1.0, 1e-3)
    assert p3.vs_rounded.v_violations == 1
    assert p3.excess > 1e-3 and not p3.bounded


def test_spike_that_leaves_the_plain_oracle_alone_is_counted():
    """A library spike that differs from both oracles where they agree is an extra mismatch, even when the rounded
    oracle's membrane is near the threshold (a tolerated flip against the rounded oracle still explains it)."""
    plain, rounded = _two_oracles(oracle.TAC, 2)
    agree = (plain[0] == rounded[0]).all(axis=0)
    b, c, y, x = np.argwhere(agree)[5]
    spk = rounded[0].copy()
    spk[0, b, c, y, x] ^= 1
    p3 = compare3(plain[:2], rounded[:2], spk, None, 1.0, 1e-3)
    near = abs(rounded[1][0, b, c, y, x] - 1.0) <= 1e-3 * max(abs(rounded[1][0, b, c, y, x]), 1.0)
    assert p3.vs_rounded.mismatches + p3.vs_rounded.flips == 1
    assert p3.vs_rounded.ok == bool(near)
    assert p3.extra_mismatches == 0        # explained by (and charged to) the comparison with the rounded oracle


def test_tolerated_flip_taints_the_neuron_only():
    spk = np.zeros((3, 4), dtype=np.uint8)
    v = np.full((3, 4), 0.5)
    v[0, 1] = 1.0 - 1e-7
    g = spk.copy()
    g[0, 1] = 1
    gv = v.copy()
    gv[1:, 1] -= 1.0                       # the flipped neuron's membrane legitimately differs afterwards
    par = compare(spk, v, g, gv, 1.0, 1e-5)
    assert par.ok and par.flips == 1 and par.tainted == 1
