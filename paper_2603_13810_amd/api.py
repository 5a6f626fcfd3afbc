"""Thin ctypes binding over libtac.so: same names as include/tac.h, argument marshalling only.

Every step of the layer (spike loading, aggregation, convolution, LIF, packing) runs inside
the library's HIP kernels.  PyTorch is used for device memory and the current stream only.
There is no fallback: if the library has not been built, the first call raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libtac.so")

TAC_PER_STEP, TAC_COLLAPSE, TAC_PRESERVE = 0, 1, 2
TAC_FP32, TAC_BF16 = 0, 1
TAC_IN_BITS, TAC_IN_BITS_POOL2, TAC_IN_BITS_MAXPOOL2, TAC_IN_F32 = 0, 1, 2, 3
TAC_KERNEL_AUTO, TAC_KERNEL_DIRECT, TAC_KERNEL_MFMA = 0, 1, 2
TAC_OUT_BITS, TAC_OUT_BITS_MAXPOOL2 = 0, 1
TAC_OK, TAC_ERR_NULL, TAC_ERR_BAD_SHAPE, TAC_ERR_BAD_K = 0, -1, -2, -3
TAC_ERR_BAD_PARAM, TAC_ERR_UNSUPPORTED, TAC_ERR_HIP, TAC_ERR_ALIGN, TAC_ERR_NEED_STATE = -4, -5, -6, -7, -8
TAC_MAX_K = 32

MODE_NAMES = {TAC_PER_STEP: "per_step", TAC_COLLAPSE: "TAC", TAC_PRESERVE: "TAC_TP"}

EXPORTS = ("tac_out_shape", "tac_packed_bytes", "tac_select_kernel", "tac_prepared_weight_bytes",
           "tac_prepare_weights", "tac_conv_lif", "tac_aggregate_tiles", "tac_aggregate_sums", "tac_mfma_probe_workgroups", "tac_mfma_probe", "tac_pack_spikes", "tac_unpack_spikes", "tac_fold_batchnorm",
           "tac_stack_check", "tac_stack_forward", "tac_conv_lif_backward", "tac_conv_lif_backward_static", "tac_stack_backward", "tac_get_counters", "tac_reset_counters", "tac_status_string",
           "tac_last_error")


class tac_layer_desc_t(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("T", "B", "Cin", "H", "W", "Cout", "kh", "kw", "stride", "pad", "K",
                 "mode", "precision", "in_format", "kernel", "out_format")] + \
               [("beta", ctypes.c_float), ("theta", ctypes.c_float)]


class TacError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__("libtac status %d: %s" % (status, text))
        self.status = status


_lib = None


def lib() -> ctypes.CDLL:
    """Load libtac.so (built in-tree by paper_2603_13810_amd/build.py).  Raises if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libtac.so is not built: run `python paper_2603_13810_amd/build.py` "
                               "(there is no CPU fallback for the HIP path)")
        L = ctypes.CDLL(LIB_PATH)
        dp, vp, i32p = ctypes.POINTER(tac_layer_desc_t), ctypes.c_void_p, ctypes.POINTER(ctypes.c_int32)
        L.tac_out_shape.argtypes = [dp, i32p, i32p, i32p]
        L.tac_out_shape.restype = ctypes.c_int
        L.tac_packed_bytes.argtypes = [ctypes.c_int32] * 5
        L.tac_packed_bytes.restype = ctypes.c_size_t
        L.tac_select_kernel.argtypes = [dp]
        L.tac_select_kernel.restype = ctypes.c_int
        L.tac_prepared_weight_bytes.argtypes = [dp]
        L.tac_prepared_weight_bytes.restype = ctypes.c_size_t
        L.tac_prepare_weights.argtypes = [dp, vp, vp, vp]
        L.tac_prepare_weights.restype = ctypes.c_int
        L.tac_conv_lif.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp]
        L.tac_conv_lif.restype = ctypes.c_int
        L.tac_aggregate_tiles.argtypes = [dp]
        L.tac_aggregate_tiles.restype = ctypes.c_size_t
        L.tac_aggregate_sums.argtypes = [dp, vp, vp, vp]
        L.tac_aggregate_sums.restype = ctypes.c_int
        L.tac_mfma_probe_workgroups.argtypes = []
        L.tac_mfma_probe_workgroups.restype = ctypes.c_size_t
        L.tac_mfma_probe.argtypes = [ctypes.c_int32, vp, vp]
        L.tac_mfma_probe.restype = ctypes.c_int
        L.tac_pack_spikes.argtypes = [vp, vp, ctypes.c_int64, ctypes.c_int32, vp]
        L.tac_pack_spikes.restype = ctypes.c_int
        L.tac_unpack_spikes.argtypes = [vp, vp, ctypes.c_int64, ctypes.c_int32, vp]
        L.tac_unpack_spikes.restype = ctypes.c_int
        L.tac_fold_batchnorm.argtypes = [vp] * 6 + [ctypes.c_float, ctypes.c_int32, ctypes.c_int32, vp, vp, vp]
        L.tac_fold_batchnorm.restype = ctypes.c_int
        u64p = ctypes.POINTER(ctypes.c_uint64)
        L.tac_get_counters.argtypes = [u64p, u64p]
        L.tac_get_counters.restype = ctypes.c_int
        L.tac_stack_check.argtypes = [vp, ctypes.c_int32, i32p]
        L.tac_stack_check.restype = ctypes.c_int
        L.tac_stack_forward.argtypes = [vp, ctypes.c_int32, vp, vp]
        L.tac_stack_forward.restype = ctypes.c_int
        L.tac_conv_lif_backward.argtypes = [dp, ctypes.POINTER(tac_backward_desc_t)] + [vp] * 9
        L.tac_conv_lif_backward.restype = ctypes.c_int
        L.tac_conv_lif_backward_static.argtypes = [dp, ctypes.POINTER(tac_backward_desc_t)] + [vp] * 8
        L.tac_conv_lif_backward_static.restype = ctypes.c_int
        L.tac_stack_backward.argtypes = [vp, vp, ctypes.POINTER(tac_backward_desc_t), ctypes.c_int32, vp, vp, vp]
        L.tac_stack_backward.restype = ctypes.c_int
        L.tac_reset_counters.argtypes = []
        L.tac_reset_counters.restype = ctypes.c_int
        L.tac_status_string.argtypes = [ctypes.c_int]
        L.tac_status_string.restype = ctypes.c_char_p
        L.tac_last_error.argtypes = []
        L.tac_last_error.restype = ctypes.c_char_p
        _lib = L
    return _lib


def tac_status_string(status: int) -> str:
    return lib().tac_status_string(int(status)).decode()


def tac_last_error() -> str:
    return lib().tac_last_error().decode()


def _check(status: int) -> None:
    if status != TAC_OK:
        text = tac_status_string(status)
        if status == TAC_ERR_HIP:
            text += " [" + tac_last_error() + "]"
        raise TacError(status, text)


def make_desc(T, B, Cin, H, W, Cout, *, K=1, beta, theta, mode, stride=1, pad=1, kh=3, kw=3,
              precision=TAC_FP32, in_format=TAC_IN_BITS, kernel=TAC_KERNEL_AUTO, out_format=TAC_OUT_BITS) -> tac_layer_desc_t:
    return tac_layer_desc_t(T=T, B=B, Cin=Cin, H=H, W=W, Cout=Cout, kh=kh, kw=kw, stride=stride, pad=pad,
                            K=K, mode=mode, precision=precision, in_format=in_format, kernel=kernel,
                            out_format=out_format, beta=beta, theta=theta)


def stored_out_shape(desc: tac_layer_desc_t) -> Tuple[int, int, int]:
    """(T_out, rows, pixels per row) of the packed output tensor: tac_out_shape, halved by the pool in the writer."""
    T_out, Ho, Wo = tac_out_shape(desc)
    return (T_out, Ho // 2, Wo // 2) if desc.out_format == TAC_OUT_BITS_MAXPOOL2 else (T_out, Ho, Wo)


def tac_out_shape(desc: tac_layer_desc_t) -> Tuple[int, int, int]:
    t, h, w = ctypes.c_int32(), ctypes.c_int32(), ctypes.c_int32()
    _check(lib().tac_out_shape(ctypes.byref(desc), ctypes.byref(t), ctypes.byref(h), ctypes.byref(w)))
    return t.value, h.value, w.value


def tac_packed_bytes(T, B, C, H, W) -> int:
    return int(lib().tac_packed_bytes(T, B, C, H, W))


def tac_select_kernel(desc: tac_layer_desc_t) -> int:
    k = lib().tac_select_kernel(ctypes.byref(desc))
    if k < 0:
        _check(k)
    return k


def tac_prepared_weight_bytes(desc: tac_layer_desc_t) -> int:
    return int(lib().tac_prepared_weight_bytes(ctypes.byref(desc)))


def _stream(stream=None):
    if stream is not None:
        return ctypes.c_void_p(int(stream))
    import torch
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dev_ptr(t, dtype=None, name="tensor"):
    if t is None:
        return None
    import torch
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("%s must be a contiguous device tensor" % name)
    if dtype is not None and t.dtype != dtype:
        raise ValueError("%s must have dtype %s" % (name, dtype))
    return ctypes.c_void_p(t.data_ptr())


def tac_prepare_weights(desc, w_oihw, w_prepared=None, stream=None):
    """w_oihw: float32 device tensor [Cout,Cin,3,3].  Returns the prepared buffer (uint8 device tensor)."""
    import torch
    if tuple(w_oihw.shape) != (desc.Cout, desc.Cin, 3, 3):
        raise ValueError("weight shape does not match the layer description")
    tac_select_kernel(desc)            # raises on an invalid or unsupported description
    n = tac_prepared_weight_bytes(desc)
    if w_prepared is None:
        w_prepared = torch.empty(n, dtype=torch.uint8, device=w_oihw.device)
    elif w_prepared.numel() * w_prepared.element_size() < n:
        raise ValueError("prepared-weight buffer too small")
    _check(lib().tac_prepare_weights(ctypes.byref(desc), _dev_ptr(w_oihw, torch.float32, "w_oihw"),
                                     _dev_ptr(w_prepared, None, "w_prepared"), _stream(stream)))
    return w_prepared


def tac_conv_lif(desc, spikes_packed, w_prepared, bias=None, v_inout=None, out_spikes_packed=None,
                 v_trace=None, stream=None):
    """One layer call.  Tensors are device tensors; buffer sizes are checked against the
    description here because the C side only sees raw pointers.  Returns out_spikes_packed
    (int32 tensor [T_out,B,Cout,Ho,ceil(Wo/32)], allocated if not given)."""
    import torch
    T_out, Ho, Wo = tac_out_shape(desc)
    f = 2 if desc.in_format in (TAC_IN_BITS_POOL2, TAC_IN_BITS_MAXPOOL2) else 1
    if desc.in_format == TAC_IN_F32:
        need_in = desc.T * desc.B * desc.Cin * desc.H * desc.W * 4
        if spikes_packed.dtype != torch.float32:
            raise ValueError("TAC_IN_F32 needs a float32 input tensor")
    else:
        need_in = tac_packed_bytes(desc.T, desc.B, desc.Cin, desc.H * f, desc.W * f)
    if spikes_packed.numel() * spikes_packed.element_size() != need_in:
        raise ValueError("spikes_packed has %d bytes, the description needs %d" %
                         (spikes_packed.numel() * spikes_packed.element_size(), need_in))
    if w_prepared.numel() * w_prepared.element_size() < tac_prepared_weight_bytes(desc):
        raise ValueError("prepared-weight buffer too small for this description")
    _, Hs, Ws = stored_out_shape(desc)
    if out_spikes_packed is None:
        out_spikes_packed = torch.empty((T_out, desc.B, desc.Cout, Hs, (Ws + 31) // 32), dtype=torch.int32,
                                        device=spikes_packed.device)
    elif out_spikes_packed.numel() * out_spikes_packed.element_size() != tac_packed_bytes(T_out, desc.B, desc.Cout, Hs, Ws):
        raise ValueError("out_spikes_packed has the wrong size")
    if bias is not None and tuple(bias.shape) != (desc.Cout,):
        raise ValueError("bias must be [Cout]")
    if v_inout is not None and tuple(v_inout.shape) != (desc.B, desc.Cout, Ho, Wo):
        raise ValueError("v_inout must be [B,Cout,Ho,Wo]")
    if v_trace is not None and tuple(v_trace.shape) != (T_out, desc.B, desc.Cout, Ho, Wo):
        raise ValueError("v_trace must be [T_out,B,Cout,Ho,Wo]")
    _check(lib().tac_conv_lif(ctypes.byref(desc), _dev_ptr(spikes_packed, None, "spikes_packed"),
                              _dev_ptr(w_prepared, None, "w_prepared"), _dev_ptr(bias, torch.float32, "bias"),
                              _dev_ptr(v_inout, torch.float32, "v_inout"),
                              _dev_ptr(out_spikes_packed, None, "out_spikes_packed"),
                              _dev_ptr(v_trace, torch.float32, "v_trace"), _stream(stream)))
    return out_spikes_packed


def tac_aggregate_tiles(desc) -> int:
    return int(lib().tac_aggregate_tiles(ctypes.byref(desc)))


def tac_aggregate_sums(desc, spikes_packed, tile_sums=None, stream=None):
    """The aggregation stage alone (see include/tac.h).  Returns tile_sums (int64 device tensor, one per workgroup)."""
    import torch
    n = tac_aggregate_tiles(desc)
    if n == 0:
        _check(TAC_ERR_UNSUPPORTED)
    if spikes_packed.numel() * spikes_packed.element_size() != tac_packed_bytes(desc.T, desc.B, desc.Cin, desc.H, desc.W):
        raise ValueError("spikes_packed does not match the description")
    if tile_sums is None:
        tile_sums = torch.empty((n,), dtype=torch.int64, device=spikes_packed.device)
    elif tile_sums.numel() != n or tile_sums.element_size() != 8:
        raise ValueError("tile_sums must hold %d 64-bit words" % n)
    _check(lib().tac_aggregate_sums(ctypes.byref(desc), _dev_ptr(spikes_packed, None, "spikes_packed"),
                                    _dev_ptr(tile_sums, None, "tile_sums"), _stream(stream)))
    return tile_sums


TAC_SG_FAST_SIGMOID, TAC_SG_ARCTAN = 0, 1


class tac_backward_desc_t(ctypes.Structure):
    _fields_ = [("surrogate", ctypes.c_int32), ("detach_reset", ctypes.c_int32), ("alpha", ctypes.c_float),
                ("grad_in_per_group", ctypes.c_int32), ("grad_out_group_K", ctypes.c_int32), ("grad_out_group_beta", ctypes.c_float)]


def tac_conv_lif_backward(desc, spikes_packed, w_oihw, v_trace, grad_out, *, surrogate=TAC_SG_FAST_SIGMOID, alpha=25.0,
                          detach_reset=False, want_input_grad=True, grad_in_per_group=False, grad_out_group_K=0,
                          grad_out_group_beta=0.0, stream=None):
    """Backward pass of one layer.  Device tensors; returns dict(grad_y, grad_w, grad_bias, grad_in).
    grad_in_per_group: grad_in is dL/dA_k [G,B,Cin,H,W]; grad_out_group_K = Kc >= 2: grad_out is the next layer's
    dL/dA_k [ceil(T_out/Kc),B,Cout,Ho,Wo] and grad_out_group_beta that layer's beta."""
    import torch
    T_out, Ho, Wo = tac_out_shape(desc)
    K = 1 if desc.mode == TAC_PER_STEP else min(desc.K, desc.T)
    G = -(-desc.T // K)
    dev = spikes_packed.device
    f = 2 if desc.in_format in (TAC_IN_BITS_POOL2, TAC_IN_BITS_MAXPOOL2) else 1
    need = (desc.T * desc.B * desc.Cin * desc.H * desc.W * 4 if desc.in_format == TAC_IN_F32
            else tac_packed_bytes(desc.T, desc.B, desc.Cin, desc.H * f, desc.W * f))
    if spikes_packed.numel() * spikes_packed.element_size() != need:
        raise ValueError("the input tensor does not match the description")
    if tuple(w_oihw.shape) != (desc.Cout, desc.Cin, 3, 3):
        raise ValueError("w_oihw must be [Cout,Cin,3,3]")
    steps_go = -(-T_out // grad_out_group_K) if grad_out_group_K > 1 else T_out
    pf = 2 if desc.out_format == TAC_OUT_BITS_MAXPOOL2 else 1          # grad_out is that of the pooled spikes the layer stored
    for name, t, shape in (("v_trace", v_trace, (T_out, desc.B, desc.Cout, Ho, Wo)),
                           ("grad_out", grad_out, (steps_go, desc.B, desc.Cout, Ho // pf, Wo // pf))):
        if tuple(t.shape) != shape:
            raise ValueError("%s must be %s" % (name, list(shape)))
    grad_y = torch.empty((G, desc.B, desc.Cout, Ho, Wo), dtype=torch.float32, device=dev)
    grad_w = torch.empty((desc.Cout, desc.Cin, 3, 3), dtype=torch.float32, device=dev)
    grad_bias = torch.empty((desc.Cout,), dtype=torch.float32, device=dev)
    grad_in = (torch.empty((G if grad_in_per_group else desc.T, desc.B, desc.Cin, desc.H * f, desc.W * f), dtype=torch.float32, device=dev)
               if want_input_grad else None)
    bwd = tac_backward_desc_t(surrogate=surrogate, detach_reset=int(bool(detach_reset)), alpha=alpha,
                              grad_in_per_group=int(bool(grad_in_per_group)), grad_out_group_K=int(grad_out_group_K),
                              grad_out_group_beta=float(grad_out_group_beta))
    _check(lib().tac_conv_lif_backward(ctypes.byref(desc), ctypes.byref(bwd), _dev_ptr(spikes_packed, None, "spikes_packed"),
                                       _dev_ptr(w_oihw, torch.float32, "w_oihw"), _dev_ptr(v_trace, torch.float32, "v_trace"),
                                       _dev_ptr(grad_out, torch.float32, "grad_out"), _dev_ptr(grad_y), _dev_ptr(grad_w),
                                       _dev_ptr(grad_bias), _dev_ptr(grad_in), _stream(stream)))
    return dict(grad_y=grad_y, grad_w=grad_w, grad_bias=grad_bias, grad_in=grad_in)


TAC_STATIC_SCRATCH_BYTES = 64 << 20


def tac_conv_lif_backward_static(desc, spikes_packed, w_oihw, v_trace, grad_out, grad_w, grad_bias, grad_in, *,
                                 surrogate=TAC_SG_FAST_SIGMOID, alpha=25.0, detach_reset=False, stream=None):
    """tac_conv_lif_backward with dL/dY_k in the library's static scratch: the caller passes every output
    (grad_w, grad_bias or None, grad_in or None) and nothing is allocated here or in the library."""
    import torch
    bwd = tac_backward_desc_t(surrogate=surrogate, detach_reset=int(bool(detach_reset)), alpha=alpha)
    _check(lib().tac_conv_lif_backward_static(ctypes.byref(desc), ctypes.byref(bwd), _dev_ptr(spikes_packed, None, "spikes_packed"),
                                              _dev_ptr(w_oihw, torch.float32, "w_oihw"), _dev_ptr(v_trace, torch.float32, "v_trace"),
                                              _dev_ptr(grad_out, torch.float32, "grad_out"), _dev_ptr(grad_w, torch.float32, "grad_w"),
                                              _dev_ptr(grad_bias, torch.float32, "grad_bias"), _dev_ptr(grad_in, torch.float32, "grad_in"),
                                              _stream(stream)))


class tac_stack_layer_t(ctypes.Structure):
    _fields_ = [("desc", tac_layer_desc_t), ("w_prepared", ctypes.c_void_p), ("bias", ctypes.c_void_p),
                ("v_inout", ctypes.c_void_p), ("out_spikes_packed", ctypes.c_void_p), ("v_trace", ctypes.c_void_p)]


def make_stack(layers):
    """layers: list of dicts with desc, w_prepared and optionally bias, v_inout, out_spikes_packed, v_trace
    (device tensors; missing outputs are allocated).  Returns (ctypes array, list of output tensors); the
    list of dicts must stay alive as long as the array is used, it owns the tensors."""
    import torch
    arr = (tac_stack_layer_t * len(layers))()
    outs = []
    for i, L in enumerate(layers):
        desc = L["desc"]
        T_out, Ho, Wo = tac_out_shape(desc)
        _, Hs, Ws = stored_out_shape(desc)
        if L.get("out_spikes_packed") is None:
            L["out_spikes_packed"] = torch.empty((T_out, desc.B, desc.Cout, Hs, (Ws + 31) // 32), dtype=torch.int32,
                                                 device=L["w_prepared"].device)
        elif L["out_spikes_packed"].numel() * L["out_spikes_packed"].element_size() != tac_packed_bytes(T_out, desc.B, desc.Cout, Hs, Ws):
            raise ValueError("layer %d: out_spikes_packed has the wrong size" % i)
        if L["w_prepared"].numel() * L["w_prepared"].element_size() < tac_prepared_weight_bytes(desc):
            raise ValueError("layer %d: prepared-weight buffer too small for this description" % i)
        if L.get("bias") is not None and tuple(L["bias"].shape) != (desc.Cout,):
            raise ValueError("layer %d: bias must be [Cout]" % i)
        if L.get("v_inout") is not None and tuple(L["v_inout"].shape) != (desc.B, desc.Cout, Ho, Wo):
            raise ValueError("layer %d: v_inout must be [B,Cout,Ho,Wo]" % i)
        if L.get("v_trace") is not None and tuple(L["v_trace"].shape) != (T_out, desc.B, desc.Cout, Ho, Wo):
            raise ValueError("layer %d: v_trace must be [T_out,B,Cout,Ho,Wo]" % i)
        arr[i].desc = desc
        val = lambda p: None if p is None else p.value
        arr[i].w_prepared = val(_dev_ptr(L["w_prepared"], None, "w_prepared"))
        arr[i].bias = val(_dev_ptr(L.get("bias"), torch.float32, "bias"))
        arr[i].v_inout = val(_dev_ptr(L.get("v_inout"), torch.float32, "v_inout"))
        arr[i].out_spikes_packed = val(_dev_ptr(L["out_spikes_packed"], None, "out_spikes_packed"))
        arr[i].v_trace = val(_dev_ptr(L.get("v_trace"), torch.float32, "v_trace"))
        outs.append(L["out_spikes_packed"])
    return arr, outs


def tac_stack_check(stack) -> Tuple[int, int]:
    """(status, index of the layer that does not continue the one before, or -1)."""
    bad = ctypes.c_int32(-1)
    rc = lib().tac_stack_check(stack, len(stack), ctypes.byref(bad))
    return rc, bad.value


def tac_stack_forward(stack, input, stream=None) -> None:
    """Enqueues every layer of a stack built by make_stack; layer 0 reads `input` (device tensor)."""
    d0 = stack[0].desc
    f = 2 if d0.in_format in (TAC_IN_BITS_POOL2, TAC_IN_BITS_MAXPOOL2) else 1
    need = (d0.T * d0.B * d0.Cin * d0.H * d0.W * 4 if d0.in_format == TAC_IN_F32
            else tac_packed_bytes(d0.T, d0.B, d0.Cin, d0.H * f, d0.W * f))
    if input.numel() * input.element_size() != need:
        raise ValueError("input has %d bytes, layer 0 needs %d" % (input.numel() * input.element_size(), need))
    _check(lib().tac_stack_forward(stack, len(stack), _dev_ptr(input, None, "input"), _stream(stream)))


class tac_stack_grads_t(ctypes.Structure):
    _fields_ = [("w_oihw", ctypes.c_void_p), ("grad_y", ctypes.c_void_p), ("grad_w", ctypes.c_void_p),
                ("grad_bias", ctypes.c_void_p), ("grad_in", ctypes.c_void_p)]


def tac_stack_backward(stack, weights, input, grad_out_last, *, surrogate=TAC_SG_FAST_SIGMOID, alpha=25.0, detach_reset=False,
                       first_layer_input_grad=False, grad_in_per_group=False, stream=None):
    """Backward pass through a stack that tac_stack_forward has run with v_trace buffers.  weights: the layers'
    plain float32 weights (device tensors).  Returns a list of dicts (grad_y, grad_w, grad_bias, grad_in) per layer.
    grad_in_per_group: layers l >= 1 that group frames and have no pool on load hand dL/dA_k [G,..] to the layer before."""
    import torch
    pools = (TAC_IN_BITS_POOL2, TAC_IN_BITS_MAXPOOL2)
    n = len(stack)
    arr = (tac_stack_grads_t * n)()
    out = []
    for l in range(n):
        d = stack[l].desc
        T_out, Ho, Wo = tac_out_shape(d)
        K = 1 if d.mode == TAC_PER_STEP else min(d.K, d.T)
        dev = weights[l].device
        g = dict(grad_y=torch.empty((-(-d.T // K), d.B, d.Cout, Ho, Wo), dtype=torch.float32, device=dev),
                 grad_w=torch.empty((d.Cout, d.Cin, 3, 3), dtype=torch.float32, device=dev),
                 grad_bias=torch.empty((d.Cout,), dtype=torch.float32, device=dev),
                 grad_in=torch.empty((-(-d.T // K) if (grad_in_per_group and l > 0 and d.in_format not in pools) else d.T,
                                      d.B, d.Cin, d.H * (2 if d.in_format in pools else 1), d.W * (2 if d.in_format in pools else 1)),
                                     dtype=torch.float32, device=dev)
                 if (l > 0 or first_layer_input_grad) else None)
        if tuple(weights[l].shape) != (d.Cout, d.Cin, 3, 3):
            raise ValueError("layer %d: weights must be [Cout,Cin,3,3]" % l)
        val = lambda p: None if p is None else p.value
        arr[l].w_oihw = val(_dev_ptr(weights[l], torch.float32, "weights"))
        for k in ("grad_y", "grad_w", "grad_bias", "grad_in"):
            setattr(arr[l], k, val(_dev_ptr(g[k])))
        out.append(g)
    bwd = tac_backward_desc_t(surrogate=surrogate, detach_reset=int(bool(detach_reset)), alpha=alpha,
                              grad_in_per_group=int(bool(grad_in_per_group)))
    _check(lib().tac_stack_backward(stack, arr, ctypes.byref(bwd), n, _dev_ptr(input, None, "input"),
                                    _dev_ptr(grad_out_last, torch.float32, "grad_out_last"), _stream(stream)))
    return out


def tac_mfma_probe(iterations, sums=None, stream=None):
    """The matrix cores alone (measurement aid).  Returns (sums, FLOP executed by the launch)."""
    import torch
    wg = int(lib().tac_mfma_probe_workgroups())
    if sums is None:
        sums = torch.empty((wg, 256), dtype=torch.float32, device="cuda")
    elif sums.numel() != wg * 256:
        raise ValueError("sums must have %d elements" % (wg * 256))
    _check(lib().tac_mfma_probe(int(iterations), _dev_ptr(sums, torch.float32, "sums"), _stream(stream)))
    return sums, wg * 4 * int(iterations) * 8 * 32768


def tac_pack_spikes(dense01, packed=None, stream=None):
    """dense01: uint8 device tensor [..., W] -> int32 device tensor [..., ceil(W/32)]."""
    import torch
    W = dense01.shape[-1]
    rows = dense01.numel() // W
    if packed is None:
        packed = torch.empty(tuple(dense01.shape[:-1]) + ((W + 31) // 32,), dtype=torch.int32, device=dense01.device)
    elif packed.numel() != rows * ((W + 31) // 32) or packed.element_size() != 4:
        raise ValueError("packed buffer has the wrong size")
    _check(lib().tac_pack_spikes(_dev_ptr(dense01, torch.uint8, "dense01"), _dev_ptr(packed, None, "packed"),
                                 rows, W, _stream(stream)))
    return packed


def tac_unpack_spikes(packed, W, dense01=None, stream=None):
    """packed: int32 device tensor [..., ceil(W/32)] -> uint8 device tensor [..., W]."""
    import torch
    Ww = (W + 31) // 32
    if packed.shape[-1] != Ww:
        raise ValueError("last dimension of packed must be ceil(W/32)")
    rows = packed.numel() // Ww
    if dense01 is None:
        dense01 = torch.empty(tuple(packed.shape[:-1]) + (W,), dtype=torch.uint8, device=packed.device)
    elif dense01.numel() != rows * W:
        raise ValueError("dense buffer has the wrong size")
    _check(lib().tac_unpack_spikes(_dev_ptr(packed, None, "packed"), _dev_ptr(dense01, torch.uint8, "dense01"),
                                   rows, W, _stream(stream)))
    return dense01


def tac_fold_batchnorm(w_oihw, bias, gamma, beta_bn, mean, var, eps=1e-5, stream=None):
    """Folds an inference batch norm that follows the convolution into (weights, bias).
    Device fp32 tensors: w_oihw [Cout,Cin,kh,kw], bias [Cout] or None, gamma/beta_bn/mean/var [Cout].
    Returns new device tensors (w_folded, bias_folded)."""
    import torch
    Cout = w_oihw.shape[0]
    for t in (gamma, beta_bn, mean, var):
        if tuple(t.shape) != (Cout,):
            raise ValueError("batch-norm vectors must be [Cout]")
    if bias is not None and tuple(bias.shape) != (Cout,):
        raise ValueError("bias must be [Cout]")
    w_out = torch.empty_like(w_oihw)
    b_out = torch.empty((Cout,), dtype=torch.float32, device=w_oihw.device)
    f32 = torch.float32
    _check(lib().tac_fold_batchnorm(_dev_ptr(w_oihw, f32, "w_oihw"), _dev_ptr(bias, f32, "bias"),
                                    _dev_ptr(gamma, f32, "gamma"), _dev_ptr(beta_bn, f32, "beta_bn"),
                                    _dev_ptr(mean, f32, "mean"), _dev_ptr(var, f32, "var"), float(eps), Cout,
                                    w_oihw.numel() // Cout, _dev_ptr(w_out, f32, "w_out"), _dev_ptr(b_out, f32, "bias_out"),
                                    _stream(stream)))
    return w_out, b_out


def tac_get_counters() -> Tuple[int, int]:
    a, b = ctypes.c_uint64(), ctypes.c_uint64()
    _check(lib().tac_get_counters(ctypes.byref(a), ctypes.byref(b)))
    return a.value, b.value


def tac_reset_counters() -> None:
    _check(lib().tac_reset_counters())
