"""The aggregation stage alone (tac_aggregate_sums) against the oracle's aggregate (Eq. 2): the 64-bit sums of
A-tile words are exact integers, so the comparison is bit for bit."""
import numpy as np
import pytest
import torch

import oracle
from paper_2603_13810_amd import api, synth
from parity_util import np_pack

pytestmark = pytest.mark.gpu
DEV = torch.device("cuda:0")


def _expected(s, K, beta, cout):
    """sum over (group, sample, cin, y, x) of pattern16(bf16(2^23 A_k)) * (cin odd ? 65536 : 1), times cout / 128."""
    T = s.shape[0]
    total = 0
    for k in range(T // K):
        A = oracle.aggregate(s, k, K=K, beta=float(np.float32(beta)), round_a_bf16=True)      # exact in bf16
        pat = (np.ascontiguousarray(A * 2.0 ** 23, dtype=np.float32).view(np.uint32) >> 16).astype(np.uint64)
        total += int(pat[:, 0::2].sum()) + 65536 * int(pat[:, 1::2].sum())
    return total * (cout // 128)


@pytest.mark.parametrize("W,H,B", [(64, 10, 3), (32, 19, 2), (64, 64, 2)])
@pytest.mark.parametrize("K", [1, 2, 4, 8, 16])
@pytest.mark.parametrize("beta", [0.9, 0.5])
def test_aggregate_sums_match_the_oracle(W, H, B, K, beta):
    r = np.random.Generator(np.random.PCG64(700 + W + H + K))
    Cin, Cout, T = 32, 256, 32
    s = (r.random((T, B, Cin, H, W)) < 0.2).astype(np.uint8)
    d = api.make_desc(T, B, Cin, H, W, Cout, K=K, beta=beta, theta=1.0, mode=api.TAC_COLLAPSE, precision=api.TAC_BF16)
    n = api.tac_aggregate_tiles(d)
    rows = 4 if W == 64 else 8
    assert n == -(-H // rows) * (Cout // 128) * B
    sums = torch.full((n,), -1, dtype=torch.int64, device=DEV)
    api.tac_aggregate_sums(d, torch.from_numpy(np_pack(s)).to(DEV), sums)
    torch.cuda.synchronize()
    got = int(sums.cpu().numpy().astype(object).sum())
    assert got == _expected(s, K, beta, Cout), (got, _expected(s, K, beta, Cout))


def test_aggregate_sums_reject_what_the_large_kernel_does_not_take():
    for kw in (dict(stride=2), dict(precision=api.TAC_FP32), dict(K=3), dict(in_format=api.TAC_IN_BITS_MAXPOOL2)):
        base = dict(K=4, beta=0.9, theta=1.0, mode=api.TAC_COLLAPSE, precision=api.TAC_BF16)
        base.update(kw)
        d = api.make_desc(12, 2, 32, 16, 64, 128, **base)
        assert api.tac_aggregate_tiles(d) == 0
        with pytest.raises(api.TacError) as e:
            api.tac_aggregate_sums(d, torch.zeros(12 * 2 * 32 * 16 * 2 * (4 if kw.get("in_format") else 1), dtype=torch.int32, device=DEV))
        assert e.value.status == api.TAC_ERR_UNSUPPORTED


def test_matrix_core_probe_runs_and_every_workgroup_computes_the_same():
    # the measurement aid behind the bench line's "mfma_loop" figures: nothing but MFMAs on fixed operands
    sums, flop = api.tac_mfma_probe(50)
    sums2, _ = api.tac_mfma_probe(50)
    torch.cuda.synchronize()
    wg = sums.shape[0]
    assert flop == wg * 4 * 50 * 8 * 32768
    s = sums.cpu().numpy()
    assert np.isfinite(s).all() and np.abs(s).max() > 0
    assert (s == s[0]).all()                       # same operands in every workgroup
    assert np.array_equal(s, sums2.cpu().numpy())  # and in every launch
    more, _ = api.tac_mfma_probe(100)
    torch.cuda.synchronize()
    assert np.allclose(more.cpu().numpy(), 2 * s, rtol=1e-3)    # twice the iterations accumulate twice the products
