"""CPU oracle for the conv-LIF layer (per-step, TAC, TAC-TP).

TEST INFRASTRUCTURE ONLY: imported by the tests, by the smoke check and by the
CPU-baseline leg of the benchmark.  The GPU library never imports or calls it.

The arithmetic lives in ``tac_oracle.c`` (plain C, double precision, seven-loop
convolution, explicit LIF recurrences as in Algorithms 1 and 2 of the paper);
this module only marshals numpy arrays into it.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "tac_oracle.c")
_LIB = os.path.join(_HERE, "libtac_oracle.so")

PER_STEP, TAC, TAC_TP = 0, 1, 2
FAST_SIGMOID, ARCTAN = 0, 1      # surrogate gradients (Sec. 5.1, Training)


def build(force: bool = False) -> str:
    """Compile tac_oracle.c with gcc (no fast-math; OpenMP only over the batch loop)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
             "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


class _Desc(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("T", "B", "Cin", "H", "W", "Cout", "kh", "kw", "stride", "pad", "K",
                 "pool2", "round_a_bf16", "nthreads", "dense")] + \
               [("beta", ctypes.c_double), ("theta", ctypes.c_double)]


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        dp = ctypes.POINTER(_Desc)
        vp = ctypes.c_void_p
        for name in ("oracle_per_step", "oracle_tac", "oracle_tac_tp"):
            f = getattr(lib, name)
            f.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp]
            f.restype = ctypes.c_int
        lib.oracle_neurons.argtypes = [dp, ctypes.c_int, vp, vp, vp, vp, ctypes.c_int64, vp, vp, vp, vp]
        lib.oracle_neurons.restype = ctypes.c_int
        lib.oracle_conv2d.argtypes = [vp, vp, vp, vp] + [ctypes.c_int] * 10
        lib.oracle_conv2d.restype = None
        lib.oracle_round_bf16.argtypes = [ctypes.c_double]
        lib.oracle_round_bf16.restype = ctypes.c_double
        lib.oracle_decay_weights.argtypes = [ctypes.c_double, ctypes.c_int, vp]
        lib.oracle_decay_weights.restype = None
        lib.oracle_aggregate.argtypes = [dp, vp, ctypes.c_int, vp, vp, vp]
        lib.oracle_aggregate.restype = None
        lib.oracle_avgpool2.argtypes = [vp, vp, ctypes.c_int64, ctypes.c_int, ctypes.c_int]
        lib.oracle_avgpool2.restype = None
        lib.oracle_maxpool2.argtypes = [vp, vp, ctypes.c_int64, ctypes.c_int, ctypes.c_int]
        lib.oracle_maxpool2.restype = None
        lib.oracle_fold_batchnorm.argtypes = [vp, vp, vp, vp, vp, vp, ctypes.c_double, ctypes.c_int, ctypes.c_int, vp, vp]
        lib.oracle_fold_batchnorm.restype = None
        lib.oracle_backward.argtypes = [dp, ctypes.c_int, ctypes.c_int, ctypes.c_double, ctypes.c_int, vp, vp, vp, vp, vp, vp, vp, vp]
        lib.oracle_backward.restype = ctypes.c_int
        lib.oracle_max_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def max_threads() -> int:
    return int(_load().oracle_max_threads())


def round_bf16(x):
    """Nearest-even rounding to bfloat16, elementwise, returned as float64."""
    lib = _load()
    a = np.asarray(x, dtype=np.float64)
    return np.vectorize(lambda v: lib.oracle_round_bf16(float(v)), otypes=[np.float64])(a)


def decay_weights(beta: float, K: int) -> np.ndarray:
    """w[j] = beta^(K-1-j) (Eq. 2)."""
    w = np.zeros(K, dtype=np.float64)
    _load().oracle_decay_weights(float(beta), int(K), _ptr(w))
    return w


def aggregate(spikes, k: int, *, K: int, beta: float, round_a_bf16: bool = False) -> np.ndarray:
    """A_k = sum_j beta^(Kg-1-j) S_{kK+j} (Eq. 2) of group k of spikes uint8 [T,B,Cin,H,W]; float64 [B,Cin,H,W]."""
    spikes = np.ascontiguousarray(spikes, dtype=np.uint8)
    T, B, Cin, H, W = spikes.shape
    d = _Desc(T=T, B=B, Cin=Cin, H=H, W=W, Cout=1, kh=3, kw=3, stride=1, pad=1, K=K, pool2=0,
              round_a_bf16=int(bool(round_a_bf16)), nthreads=1, dense=0, beta=float(beta), theta=1.0)
    A = np.zeros((B, Cin, H, W), dtype=np.float64)
    X = np.zeros_like(A)
    tmp = np.zeros_like(A)
    _load().oracle_aggregate(ctypes.byref(d), _ptr(spikes), int(k), _ptr(A), _ptr(X), _ptr(tmp))
    return A


def avgpool2(x: np.ndarray) -> np.ndarray:
    """2x2 mean pool, stride 2, over the last two axes."""
    x = np.ascontiguousarray(x, dtype=np.float64)
    H2, W2 = x.shape[-2:]
    assert H2 % 2 == 0 and W2 % 2 == 0
    out = np.zeros(x.shape[:-2] + (H2 // 2, W2 // 2), dtype=np.float64)
    _load().oracle_avgpool2(_ptr(x), _ptr(out), int(np.prod(x.shape[:-2], dtype=np.int64)), H2 // 2, W2 // 2)
    return out


def maxpool2(x: np.ndarray) -> np.ndarray:
    """2x2 max pool, stride 2, over the last two axes (Sec. 5.1: MaxPool(2) after each LIF layer)."""
    x = np.ascontiguousarray(x, dtype=np.float64)
    H2, W2 = x.shape[-2:]
    assert H2 % 2 == 0 and W2 % 2 == 0
    out = np.zeros(x.shape[:-2] + (H2 // 2, W2 // 2), dtype=np.float64)
    _load().oracle_maxpool2(_ptr(x), _ptr(out), int(np.prod(x.shape[:-2], dtype=np.int64)), H2 // 2, W2 // 2)
    return out


def fold_batchnorm(w, bias, gamma, beta_bn, mean, var, eps=1e-5):
    """Inference batch norm after the convolution folded into (weights, bias) (Sec. 5.1:
    Conv -> BN -> LIF).  Returns (w_folded [Cout,Cin,kh,kw], bias_folded [Cout]) in float64."""
    w = np.ascontiguousarray(w, dtype=np.float64)
    Cout = w.shape[0]
    arrs = [None if bias is None else np.ascontiguousarray(bias, dtype=np.float64)]
    arrs += [np.ascontiguousarray(a, dtype=np.float64) for a in (gamma, beta_bn, mean, var)]
    for a in arrs:
        assert a is None or a.shape == (Cout,)
    w_out = np.zeros_like(w)
    b_out = np.zeros(Cout, dtype=np.float64)
    _load().oracle_fold_batchnorm(_ptr(w), _ptr(arrs[0]), _ptr(arrs[1]), _ptr(arrs[2]), _ptr(arrs[3]), _ptr(arrs[4]),
                                  float(eps), Cout, int(w.size // Cout), _ptr(w_out), _ptr(b_out))
    return w_out, b_out


def conv2d(x: np.ndarray, w: np.ndarray, bias=None, stride: int = 1, pad: int = 1, nthreads: int = 1) -> np.ndarray:
    """Zero-padded cross-correlation, x[B,Cin,H,W], w[Cout,Cin,kh,kw] -> [B,Cout,Ho,Wo] (float64)."""
    x = np.ascontiguousarray(x, dtype=np.float64)
    w = np.ascontiguousarray(w, dtype=np.float64)
    B, Cin, H, W = x.shape
    Cout, Cin2, kh, kw = w.shape
    assert Cin == Cin2
    if bias is not None:
        bias = np.ascontiguousarray(bias, dtype=np.float64)
        assert bias.shape == (Cout,)
    Ho = (H + 2 * pad - kh) // stride + 1
    Wo = (W + 2 * pad - kw) // stride + 1
    y = np.zeros((B, Cout, Ho, Wo), dtype=np.float64)
    _load().oracle_conv2d(_ptr(x), _ptr(w), _ptr(bias), _ptr(y), B, Cin, H, W, Cout, kh, kw, stride, pad, nthreads)
    return y


def _as_input(spikes):
    """uint8 0/1 spikes stay bytes; anything real-valued is handed over as float64 frames."""
    spikes = np.asarray(spikes)
    if np.issubdtype(spikes.dtype, np.floating):
        return np.ascontiguousarray(spikes, dtype=np.float64)
    return np.ascontiguousarray(spikes, dtype=np.uint8)


def _desc(spikes, weight, K, beta, theta, stride, pad, pool2, round_a_bf16, nthreads):
    T, B, Cin, Hs, Ws = spikes.shape
    Cout, Cin2, kh, kw = weight.shape
    if Cin != Cin2:
        raise ValueError("channel mismatch")
    if pool2:
        if Hs % 2 or Ws % 2:
            raise ValueError("pool2 needs even input size")
        H, W = Hs // 2, Ws // 2
    else:
        H, W = Hs, Ws
    d = _Desc(T=T, B=B, Cin=Cin, H=H, W=W, Cout=Cout, kh=kh, kw=kw, stride=stride, pad=pad, K=K,
              pool2=(2 if pool2 in (2, "max") else int(bool(pool2))), round_a_bf16=int(bool(round_a_bf16)), nthreads=int(nthreads),
              dense=int(spikes.dtype == np.float64), beta=float(beta), theta=float(theta))
    Ho = (H + 2 * pad - kh) // stride + 1
    Wo = (W + 2 * pad - kw) // stride + 1
    return d, Ho, Wo


def conv_lif(spikes, weight, bias=None, *, K=1, beta, theta, mode, stride=1, pad=1, v0=None,
             pool2=False, round_a_bf16=False, nthreads=1):
    """One conv-LIF layer over all T input frames.

    spikes uint8 [T,B,Cin,H,W] of 0/1 (unpooled size when pool2); weight [Cout,Cin,kh,kw];
    mode PER_STEP / TAC / TAC_TP.  Returns (out_spikes uint8 [T_out,B,Cout,Ho,Wo],
    v_pre float64 same shape (membrane before reset at every LIF step),
    v_final float64 [B,Cout,Ho,Wo]).
    """
    lib = _load()
    spikes = _as_input(spikes)
    if spikes.max(initial=0) > 1:
        raise ValueError("spikes must be 0/1")
    weight = np.ascontiguousarray(weight, dtype=np.float64)
    d, Ho, Wo = _desc(spikes, weight, K, beta, theta, stride, pad, pool2, round_a_bf16, nthreads)
    if bias is not None:
        bias = np.ascontiguousarray(bias, dtype=np.float64)
    if v0 is not None:
        v0 = np.ascontiguousarray(v0, dtype=np.float64)
        assert v0.shape == (d.B, d.Cout, Ho, Wo)
    T_out = -(-d.T // K) if mode == TAC else d.T       # a shorter last group when K does not divide T
    out_s = np.zeros((T_out, d.B, d.Cout, Ho, Wo), dtype=np.uint8)
    v_pre = np.zeros((T_out, d.B, d.Cout, Ho, Wo), dtype=np.float64)
    v_fin = np.zeros((d.B, d.Cout, Ho, Wo), dtype=np.float64)
    fn = {PER_STEP: lib.oracle_per_step, TAC: lib.oracle_tac, TAC_TP: lib.oracle_tac_tp}[mode]
    rc = fn(ctypes.byref(d), _ptr(spikes), _ptr(weight), _ptr(bias), _ptr(v0), _ptr(out_s), _ptr(v_pre), _ptr(v_fin))
    if rc:
        raise ValueError("oracle rejected the layer description (code %d)" % rc)
    return out_s, v_pre, v_fin


def conv_lif_neurons(spikes, weight, bias=None, *, idx, K=1, beta, theta, mode, stride=1, pad=1,
                     v0=None, pool2=False, round_a_bf16=False, nthreads=1):
    """The same layer followed at single output neurons idx[n,4] = (b, co, oy, ox).

    Returns (out_spikes uint8 [T_out,n], v_pre float64 [T_out,n], v_final float64 [n]).
    """
    lib = _load()
    spikes = _as_input(spikes)
    weight = np.ascontiguousarray(weight, dtype=np.float64)
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    assert idx.ndim == 2 and idx.shape[1] == 4
    n = idx.shape[0]
    d, Ho, Wo = _desc(spikes, weight, K, beta, theta, stride, pad, pool2, round_a_bf16, nthreads)
    if bias is not None:
        bias = np.ascontiguousarray(bias, dtype=np.float64)
    if v0 is not None:
        v0 = np.ascontiguousarray(v0, dtype=np.float64)
        assert v0.shape == (n,)
    T_out = -(-d.T // K) if mode == TAC else d.T
    out_s = np.zeros((T_out, n), dtype=np.uint8)
    v_pre = np.zeros((T_out, n), dtype=np.float64)
    v_fin = np.zeros((n,), dtype=np.float64)
    rc = lib.oracle_neurons(ctypes.byref(d), int(mode), _ptr(spikes), _ptr(weight), _ptr(bias), _ptr(v0),
                            n, _ptr(idx), _ptr(out_s), _ptr(v_pre), _ptr(v_fin))
    if rc:
        raise ValueError("oracle rejected the request (code %d)" % rc)
    return out_s, v_pre, v_fin


def conv_lif_backward(spikes, weight, v_pre, g_out, *, K=1, beta, theta, mode, stride=1, pad=1,
                      surrogate=FAST_SIGMOID, alpha=25.0, detach_reset=False, want_input_grad=True, round_a_bf16=False, pool2=False):
    """Backward pass of one conv-LIF layer with a surrogate gradient (Sec. 5.1, Training).

    spikes as in conv_lif (no pooled input); v_pre [T_out,B,Cout,Ho,Wo] is the membrane before the
    reset that conv_lif returned; g_out, same shape, is dL/d(output spikes).  Returns a dict with
    dY [G,B,Cout,Ho,Wo] (dL/dY_k), dW [Cout,Cin,kh,kw], dbias [Cout] and g_in [T,B,Cin,H,W]
    (dL/d(input frames); None when not wanted).  round_a_bf16: the aggregates A_k enter dW rounded to bfloat16,
    as they entered a bf16 forward pass.  pool2 as in conv_lif: g_in is then the gradient of the unpooled frames."""
    lib = _load()
    spikes = _as_input(spikes)
    weight = np.ascontiguousarray(weight, dtype=np.float64)
    d, Ho, Wo = _desc(spikes, weight, K, beta, theta, stride, pad, pool2, round_a_bf16, 1)
    Kg = 1 if mode == PER_STEP else K
    G = -(-d.T // Kg)
    T_out = d.T if mode != TAC else G
    v_pre = np.ascontiguousarray(v_pre, dtype=np.float64)
    g_out = np.ascontiguousarray(g_out, dtype=np.float64)
    assert v_pre.shape == (T_out, d.B, d.Cout, Ho, Wo) and g_out.shape == v_pre.shape
    dY = np.zeros((G, d.B, d.Cout, Ho, Wo))
    dW = np.zeros(weight.shape)
    dbias = np.zeros(d.Cout)
    g_in = np.zeros(spikes.shape) if want_input_grad else None
    rc = lib.oracle_backward(ctypes.byref(d), int(mode), int(surrogate), float(alpha), int(bool(detach_reset)),
                             _ptr(spikes), _ptr(weight), _ptr(v_pre), _ptr(g_out), _ptr(dY), _ptr(dW), _ptr(dbias), _ptr(g_in))
    if rc:
        raise ValueError("oracle rejected the request (code %d)" % rc)
    return dict(dY=dY, dW=dW, dbias=dbias, g_in=g_in)
