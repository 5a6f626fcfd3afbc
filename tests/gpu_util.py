"""Test-side plumbing for running one layer on the GPU library and on the oracle."""
import numpy as np
import torch

import oracle
from paper_2603_13810_amd import api

from parity_util import np_pack, np_unpack, pad_bits_zero, compare, compare3, TOL_FP32, TOL_BF16

ORACLE_MODE = {api.TAC_PER_STEP: oracle.PER_STEP, api.TAC_COLLAPSE: oracle.TAC, api.TAC_PRESERVE: oracle.TAC_TP}


def bf16_round_np(w32: np.ndarray) -> np.ndarray:
    """float32 array -> nearest-even bf16 values as float32 (library cast, not the oracle's)."""
    return torch.from_numpy(np.ascontiguousarray(w32, dtype=np.float32)).to(torch.bfloat16).to(torch.float32).numpy()


def run_gpu(spikes, w32, *, K, beta, theta, mode, stride=1, bias=None, v0=None, pool2=False,
            precision=api.TAC_FP32, kernel=api.TAC_KERNEL_AUTO, trace=True, out_pool=False):
    """spikes uint8 [T,B,Cin,Hs,Ws] host array (float32: real-valued frames, TAC_IN_F32).
    Returns dict with unpacked spikes, v_trace, v_final, kernel id.  out_pool: the layer max-pools its output
    spikes 2 x 2 before it stores them; `spikes` is then the pooled tensor [T_out,B,Cout,Ho/2,Wo/2]."""
    dev = torch.device("cuda:0")
    dense = np.issubdtype(np.asarray(spikes).dtype, np.floating)
    T, B, Cin, Hs, Ws = spikes.shape
    H, W = (Hs // 2, Ws // 2) if pool2 else (Hs, Ws)
    Cout = w32.shape[0]
    desc = api.make_desc(T, B, Cin, H, W, Cout, K=K, beta=beta, theta=theta, mode=mode, stride=stride,
                         precision=precision, kernel=kernel,
                         out_format=api.TAC_OUT_BITS_MAXPOOL2 if out_pool else api.TAC_OUT_BITS,
                         in_format=api.TAC_IN_F32 if dense else
                         (api.TAC_IN_BITS_MAXPOOL2 if pool2 == "max" else api.TAC_IN_BITS_POOL2) if pool2 else api.TAC_IN_BITS)
    T_out, Ho, Wo = api.tac_out_shape(desc)
    sp = torch.from_numpy(np.ascontiguousarray(spikes, dtype=np.float32) if dense else np_pack(spikes)).to(dev)
    wp = api.tac_prepare_weights(desc, torch.from_numpy(np.ascontiguousarray(w32, dtype=np.float32)).to(dev))
    bias_d = None if bias is None else torch.from_numpy(np.asarray(bias, dtype=np.float32)).to(dev)
    v = None
    if v0 is not None or trace:
        v = torch.zeros((B, Cout, Ho, Wo), dtype=torch.float32, device=dev)
        if v0 is not None:
            v.copy_(torch.from_numpy(np.asarray(v0, dtype=np.float32)))
    vt = torch.full((T_out, B, Cout, Ho, Wo), float("nan"), dtype=torch.float32, device=dev) if trace else None
    # poison the output so unwritten words show up
    _, Hst, Wst = api.stored_out_shape(desc)
    out = torch.full((T_out, B, Cout, Hst, (Wst + 31) // 32), -1, dtype=torch.int32, device=dev)
    api.tac_conv_lif(desc, sp, wp, bias_d, v, out, vt)
    torch.cuda.synchronize()
    out_h = out.cpu().numpy()
    return dict(spikes=np_unpack(out_h, Wst), pad_ok=pad_bits_zero(out_h, Wst), packed=out_h,
                v_trace=None if vt is None else vt.cpu().numpy(), v_final=None if v is None else v.cpu().numpy(),
                kernel=api.tac_select_kernel(desc), desc=desc)


def run_oracle(spikes, w32, *, K, beta, theta, mode, stride=1, bias=None, v0=None, pool2=False,
               quantised=False, nthreads=None):
    """Plain oracle (double arithmetic on the fp32 inputs the GPU received) or, with quantised=True,
    the same with W and A_k first rounded to bf16."""
    w = bf16_round_np(w32) if quantised else np.asarray(w32, dtype=np.float32)
    return oracle.conv_lif(spikes, w.astype(np.float64), None if bias is None else np.asarray(bias, np.float32).astype(np.float64),
                           K=K, beta=float(np.float32(beta)), theta=float(np.float32(theta)), mode=ORACLE_MODE[mode],
                           stride=stride, pad=1, v0=None if v0 is None else np.asarray(v0, np.float32).astype(np.float64),
                           pool2=pool2, round_a_bf16=quantised, nthreads=nthreads or oracle.max_threads())


TOL_BF16_SAME_OPERANDS = 1e-3


def check_layer(spikes, w32, *, precision=api.TAC_FP32, kernel=api.TAC_KERNEL_AUTO, expect_kernel=None,
                oracle_samples=None, **kw):
    """Run both sides and assert parity.

    oracle_samples: list of sample indices.  The library runs on the whole batch (the launch geometry
    under test); the oracle runs on those samples only and the comparison covers all of their neurons
    (samples are independent).  The returned oracle arrays then have len(oracle_samples) samples.

    fp32 path: against the plain double-precision oracle at 1e-5.
    bf16 path: the oracle runs twice, plain and with W and every A_k rounded to bfloat16 (its own
    rounding code).  Asserted: (i) the library against the rounded oracle at 1e-3 (what is left is
    fp32-vs-double accumulation and, rarely, one bf16 ulp in an A_k whose fp32 sum sits on a rounding
    tie); (ii) the library adds nothing to what the operand rounding does by itself on the CPU: its
    distance to the plain oracle is at most the rounded oracle's plus 1e-3 of the scale, and a neuron
    leaves the plain oracle's spike train only where the rounded oracle's does (Parity3.bounded).
    The comparison against the plain oracle at the stated 2e-2 is computed, returned as `.plain`
    (all three as `.p3`) and printed by the callers; it is not asserted to be clean, because the rounded
    oracle itself is not (TAC-TP with K >= 4: see test_bf16_operand_rounding_alone_exceeds_the_bar in
    the CPU tests).
    """
    g = run_gpu(spikes, w32, precision=precision, kernel=kernel, **kw)
    if expect_kernel is not None:
        assert g["kernel"] == expect_kernel
    assert g["pad_ok"], "pad bits of the packed output must be zero"
    theta = float(np.float32(kw["theta"]))
    if not kw.get("out_pool"):
        # the kernel without the membrane trace is the one that is timed (on the large matrix-core kernel it is a
        # variant of its own, with the LIF step under the MFMAs): same spikes and same final membrane, bit for bit
        g2 = run_gpu(spikes, w32, precision=precision, kernel=kernel, **dict(kw, trace=False, v0=kw.get("v0") if kw.get("v0") is not None else np.zeros_like(g["v_final"])))
        assert np.array_equal(g2["packed"], g["packed"]), "kernels with and without the membrane trace store different spikes"
        assert np.array_equal(g2["v_final"], g["v_final"]), "kernels with and without the membrane trace leave different membranes"
    if kw.get("out_pool"):
        # The stored spikes are pooled.  The library's unpooled spikes follow from the membranes it recorded
        # (spike iff V >= theta, the comparison the kernel makes, in fp32): (i) they and the membranes are held
        # against the oracle below like any other layer's; (ii) the stored tensor must be their 2 x 2 maximum,
        # bit for bit; (iii) the kernel without the membrane trace (the timed one) stores the same bits.
        kw = {k: v for k, v in kw.items() if k != "out_pool"}
        unpooled = (g["v_trace"] >= np.float32(theta)).astype(np.uint8)
        T_, B_, C_, Ho_, Wo_ = unpooled.shape
        want = unpooled.reshape(T_, B_, C_, Ho_ // 2, 2, Wo_ // 2, 2).max(axis=(4, 6))
        assert np.array_equal(g["spikes"], want), "stored spikes are not the 2 x 2 maximum of the layer's spikes"
        g2 = run_gpu(spikes, w32, precision=precision, kernel=kernel, trace=False, out_pool=True, **kw)
        assert np.array_equal(g2["packed"], g["packed"]), "kernels with and without the membrane trace differ"
        g = dict(g, pooled=g["spikes"], spikes=unpooled)
    if oracle_samples is not None:
        sel = list(oracle_samples)
        spikes = np.ascontiguousarray(np.asarray(spikes)[:, sel])
        if kw.get("v0") is not None:
            kw = dict(kw, v0=np.asarray(kw["v0"])[sel])
        g = dict(g, spikes=g["spikes"][:, sel], v_trace=None if g["v_trace"] is None else g["v_trace"][:, sel],
                 v_final=None if g["v_final"] is None else g["v_final"][sel], spikes_all=g["spikes"])
    if precision == api.TAC_BF16:
        rp = run_oracle(spikes, w32, **kw)
        r = run_oracle(spikes, w32, quantised=True, **kw)
        tol = TOL_BF16_SAME_OPERANDS
        p3 = compare3(rp[:2], r[:2], g["spikes"], g["v_trace"], theta, tol, TOL_BF16)
        par = p3.vs_rounded
        par.plain, par.p3 = p3.vs_plain, p3
        assert par.ok, "vs rounded oracle: %s" % par
        assert p3.bounded, "beyond the operand rounding: %s" % p3
    else:
        r = run_oracle(spikes, w32, **kw)
        tol = TOL_FP32
        par = compare(r[0], r[1], g["spikes"], g["v_trace"], theta, tol)
        par.plain, par.p3 = None, None
        assert par.ok, "vs oracle: %s" % par
    if par.flips == 0 and g["v_final"] is not None:
        err = np.abs(g["v_final"] - r[2]) / np.maximum(np.abs(r[2]), theta)
        assert err.max() <= tol, "final V err %.3g" % err.max()
    return par, g, r
