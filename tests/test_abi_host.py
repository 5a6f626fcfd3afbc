"""Host-side behaviour of the C-ABI library that needs no GPU: it loads, exports every
symbol the header declares, validates arguments before launching anything, and does the
shape / size / call-count accounting the paper's tables imply."""
import ctypes
import os
import re

import pytest

from paper_2603_13810_amd import api

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _desc(**kw):
    base = dict(T=8, B=2, Cin=3, H=16, W=20, Cout=8, K=2, beta=0.9, theta=1.0, mode=api.TAC_COLLAPSE)
    base.update(kw)
    return api.make_desc(**base)


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "tac.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(tac_[a-z_]+)\s*\(", header))
    assert declared == set(api.EXPORTS)
    L = api.lib()
    for name in declared:
        assert hasattr(L, name), name


def test_desc_struct_layout_matches_header():
    # sixteen int32 fields in the header's order, then beta and theta
    assert ctypes.sizeof(api.tac_layer_desc_t) == 16 * 4 + 2 * 4
    header = open(os.path.join(ROOT, "include", "tac.h")).read()
    body = header[header.index("typedef struct tac_layer_desc {"):header.index("} tac_layer_desc_t;")]
    names = [n.strip() for decl in re.findall(r"(?:int32_t|float)\s+([^;]+);", body) for n in decl.split(",")]
    assert names == [f[0] for f in api.tac_layer_desc_t._fields_]
    assert api.tac_layer_desc_t.out_format.offset == 15 * 4 and api.tac_layer_desc_t.beta.offset == 16 * 4


@pytest.mark.parametrize("mode,K,T_out", [(api.TAC_PER_STEP, 4, 8), (api.TAC_COLLAPSE, 4, 2),
                                          (api.TAC_PRESERVE, 4, 8), (api.TAC_COLLAPSE, 1, 8)])
def test_out_shape_collapse_vs_preserve(mode, K, T_out):
    # Alg. 1 returns T/K steps, Alg. 2 and the per-step layer T steps (App. B)
    assert api.tac_out_shape(_desc(mode=mode, K=K)) == (T_out, 16, 20)
    assert api.tac_out_shape(_desc(mode=mode, K=K, stride=2, H=128, W=128))[1:] == (64, 64)
    assert api.tac_out_shape(_desc(mode=mode, K=K, stride=2, H=5, W=7))[1:] == (3, 4)


def test_cascade_of_collapse_layers_divides_T():
    # App. B: TAC cascades to T / prod K_l, TAC-TP keeps T
    T = 16
    for K in (2, 2, 2, 2):
        T = api.tac_out_shape(_desc(T=T, K=K, mode=api.TAC_COLLAPSE))[0]
    assert T == 1
    T = 16
    for K in (2, 4, 8):
        T = api.tac_out_shape(_desc(T=T, K=K, mode=api.TAC_PRESERVE))[0]
    assert T == 16


def test_packed_bytes():
    assert api.tac_packed_bytes(32, 256, 128, 64, 64) == 512 * 1024 * 1024
    assert api.tac_packed_bytes(4, 4, 1, 28, 28) == 4 * 4 * 28 * 4
    assert api.tac_packed_bytes(1, 1, 1, 1, 33) == 8
    assert api.tac_packed_bytes(0, 1, 1, 1, 1) == 0


@pytest.mark.parametrize("kw,status", [
    (dict(T=0), api.TAC_ERR_BAD_SHAPE), (dict(Cout=-1), api.TAC_ERR_BAD_SHAPE),
    (dict(kh=5), api.TAC_ERR_BAD_SHAPE), (dict(stride=3), api.TAC_ERR_BAD_SHAPE), (dict(pad=0), api.TAC_ERR_BAD_SHAPE),
    (dict(K=33), api.TAC_ERR_BAD_K), (dict(K=0), api.TAC_ERR_BAD_K), (dict(T=64, K=64), api.TAC_ERR_BAD_K),
    (dict(beta=1.5), api.TAC_ERR_BAD_PARAM), (dict(beta=float("nan")), api.TAC_ERR_BAD_PARAM),
    (dict(theta=0.0), api.TAC_ERR_BAD_PARAM), (dict(theta=float("inf")), api.TAC_ERR_BAD_PARAM),
    (dict(mode=7), api.TAC_ERR_BAD_PARAM), (dict(precision=3), api.TAC_ERR_BAD_PARAM),
    (dict(in_format=4), api.TAC_ERR_BAD_PARAM), (dict(kernel=9), api.TAC_ERR_BAD_PARAM),
    (dict(B=70000), api.TAC_ERR_BAD_SHAPE),
    (dict(W=2049), api.TAC_ERR_UNSUPPORTED), (dict(W=1025, in_format=api.TAC_IN_BITS_POOL2), api.TAC_ERR_UNSUPPORTED),
])
def test_invalid_descriptions_are_rejected_before_any_launch(kw, status):
    L = api.lib()
    d = _desc(**kw)
    assert L.tac_out_shape(ctypes.byref(d), None, None, None) == status
    assert L.tac_select_kernel(ctypes.byref(d)) == status
    assert L.tac_prepared_weight_bytes(ctypes.byref(d)) == 0
    fake = ctypes.c_void_p(0x1000)
    assert L.tac_conv_lif(ctypes.byref(d), fake, fake, None, None, fake, None, None) == status
    assert L.tac_prepare_weights(ctypes.byref(d), fake, fake, None) == status
    assert api.tac_status_string(status) not in ("ok", "unknown status")


def test_sequence_length_need_not_be_a_multiple_of_K():
    # the frames left over form one more, shorter group: ceil(T/K) output steps for TAC, T for TAC-TP
    assert api.tac_out_shape(_desc(T=8, K=3, mode=api.TAC_COLLAPSE))[0] == 3
    assert api.tac_out_shape(_desc(T=8, K=3, mode=api.TAC_PRESERVE))[0] == 8
    assert api.tac_out_shape(_desc(T=25, K=16, mode=api.TAC_COLLAPSE))[0] == 2
    # a group longer than the sequence is one group of T frames
    assert api.tac_out_shape(_desc(T=3, K=8, mode=api.TAC_COLLAPSE))[0] == 1
    for f in (api.tac_select_kernel, api.tac_prepared_weight_bytes):
        assert f(_desc(T=3, K=8, mode=api.TAC_COLLAPSE)) == f(_desc(T=3, K=3, mode=api.TAC_COLLAPSE))
    # the short group is a second launch and takes the membrane from v_inout: refused without it,
    # before anything is launched
    L = api.lib()
    fake = ctypes.c_void_p(0x1000)
    d = _desc(T=8, K=3, mode=api.TAC_COLLAPSE)
    assert L.tac_conv_lif(ctypes.byref(d), fake, fake, None, None, fake, None, None) == api.TAC_ERR_NEED_STATE
    assert api.tac_status_string(api.TAC_ERR_NEED_STATE) not in ("ok", "unknown status")


def test_per_step_ignores_K():
    d = _desc(mode=api.TAC_PER_STEP, K=3)
    assert api.tac_out_shape(d)[0] == 8


def test_null_and_alignment_errors():
    L = api.lib()
    d = _desc()
    fake, odd = ctypes.c_void_p(0x1000), ctypes.c_void_p(0x1002)
    assert L.tac_out_shape(None, None, None, None) == api.TAC_ERR_NULL
    assert L.tac_conv_lif(ctypes.byref(d), None, fake, None, None, fake, None, None) == api.TAC_ERR_NULL
    assert L.tac_conv_lif(ctypes.byref(d), fake, None, None, None, fake, None, None) == api.TAC_ERR_NULL
    assert L.tac_conv_lif(ctypes.byref(d), fake, fake, None, None, None, None, None) == api.TAC_ERR_NULL
    assert L.tac_conv_lif(ctypes.byref(d), odd, fake, None, None, fake, None, None) == api.TAC_ERR_ALIGN
    assert L.tac_conv_lif(ctypes.byref(d), fake, fake, None, odd, fake, None, None) == api.TAC_ERR_ALIGN
    assert L.tac_prepare_weights(ctypes.byref(d), None, fake, None) == api.TAC_ERR_NULL
    assert L.tac_prepare_weights(ctypes.byref(d), fake, ctypes.c_void_p(0x1004), None) == api.TAC_ERR_ALIGN
    assert L.tac_pack_spikes(None, fake, 1, 1, None) == api.TAC_ERR_NULL
    assert L.tac_pack_spikes(fake, fake, 0, 1, None) == api.TAC_ERR_BAD_SHAPE
    assert L.tac_unpack_spikes(fake, fake, 1, 0, None) == api.TAC_ERR_BAD_SHAPE
    assert L.tac_get_counters(None, None) == api.TAC_ERR_NULL


def test_kernel_selection():
    # fp32 always runs on the vector-FMA kernel; forcing the matrix-core kernel on it is an error
    d = _desc(precision=api.TAC_FP32)
    assert api.tac_select_kernel(d) == api.TAC_KERNEL_DIRECT
    d.kernel = api.TAC_KERNEL_MFMA
    assert api.lib().tac_select_kernel(ctypes.byref(d)) == api.TAC_ERR_UNSUPPORTED
    d = _desc(precision=api.TAC_BF16, kernel=api.TAC_KERNEL_DIRECT)
    assert api.tac_select_kernel(d) == api.TAC_KERNEL_DIRECT
    assert api.tac_prepared_weight_bytes(d) == 3 * 9 * 32 * 4        # [Cin][tap][Cout padded to 32] fp32


def test_status_strings():
    assert api.tac_status_string(0) == "ok"
    assert api.tac_status_string(-99) == "unknown status"
    assert api.tac_last_error() == ""


def _stack(descs):
    arr = (api.tac_stack_layer_t * len(descs))()
    for i, d in enumerate(descs):
        arr[i].desc = d
        arr[i].w_prepared = 0x1000
        arr[i].out_spikes_packed = 0x2000
    return arr


def test_stack_check_follows_shapes_steps_and_pools_from_layer_to_layer():
    mk = lambda T, Cin, H, W, Cout, **kw: api.make_desc(T, 2, Cin, H, W, Cout, beta=0.9, theta=1.0, **kw)
    C, P, S = api.TAC_COLLAPSE, api.TAC_PRESERVE, api.TAC_PER_STEP
    good = [mk(25, 2, 64, 64, 16, K=4, mode=C, stride=2),                               # 25 -> 7 steps, 32 x 32
            mk(7, 16, 16, 16, 32, K=2, mode=P, in_format=api.TAC_IN_BITS_MAXPOOL2),     # pooled to 16 x 16, 7 steps
            mk(7, 32, 16, 16, 8, K=4, mode=C),                                          # 7 -> 2 steps
            mk(2, 8, 8, 8, 8, mode=S, in_format=api.TAC_IN_BITS_POOL2)]
    assert api.tac_stack_check(_stack(good)) == (api.TAC_OK, -1)
    assert api.tac_stack_check(_stack(good[:1])) == (api.TAC_OK, -1)
    for layer, change in [(1, dict(T=6)), (1, dict(Cin=8)), (1, dict(H=32)), (2, dict(T=4)), (3, dict(W=16)), (2, dict(B=3)),
                          (1, dict(in_format=api.TAC_IN_F32))]:
        bad = [api.tac_layer_desc_t.from_buffer_copy(d) for d in good]
        for k, v in change.items():
            setattr(bad[layer], k, v)
        assert api.tac_stack_check(_stack(bad)) == (api.TAC_ERR_BAD_SHAPE, layer), (layer, change)
    bad = [api.tac_layer_desc_t.from_buffer_copy(d) for d in good]
    bad[2].K = 0
    assert api.tac_stack_check(_stack(bad)) == (api.TAC_ERR_BAD_K, 2)
    # an odd size cannot be pooled
    odd = [mk(4, 2, 14, 14, 4, K=2, mode=P, stride=2), mk(4, 4, 3, 3, 4, mode=S, in_format=api.TAC_IN_BITS_POOL2)]
    assert api.tac_stack_check(_stack(odd)) == (api.TAC_ERR_BAD_SHAPE, 1)
    L = api.lib()
    assert L.tac_stack_check(None, 1, None) == api.TAC_ERR_NULL
    assert L.tac_stack_check(_stack(good), 0, None) == api.TAC_ERR_BAD_SHAPE
    assert L.tac_stack_forward(None, 1, None, None) == api.TAC_ERR_NULL


def test_backward_rejects_bad_requests_before_any_launch():
    L = api.lib()
    d = _desc()
    fake, odd = ctypes.c_void_p(0x1000), ctypes.c_void_p(0x1002)
    ok = api.tac_backward_desc_t(surrogate=api.TAC_SG_ARCTAN, detach_reset=1, alpha=2.0)
    call = lambda desc, bwd, *ptrs: L.tac_conv_lif_backward(ctypes.byref(desc), bwd if bwd is None else ctypes.byref(bwd), *ptrs, None)
    nine = [fake] * 9
    assert call(d, None, *nine) == api.TAC_ERR_NULL
    for i in range(6):                           # input, weights, membranes, grad_out, grad_y, grad_w are required
        ptrs = list(nine); ptrs[i] = None
        assert call(d, ok, *ptrs) == api.TAC_ERR_NULL, i
    ptrs = list(nine); ptrs[5] = odd
    assert call(d, ok, *ptrs) == api.TAC_ERR_ALIGN
    assert call(d, api.tac_backward_desc_t(surrogate=2, detach_reset=0, alpha=2.0), *nine) == api.TAC_ERR_BAD_PARAM
    assert call(d, api.tac_backward_desc_t(surrogate=0, detach_reset=0, alpha=0.0), *nine) == api.TAC_ERR_BAD_PARAM
    assert call(_desc(W=2048, in_format=api.TAC_IN_BITS), ok, *nine) == api.TAC_ERR_UNSUPPORTED
    assert call(_desc(K=0), ok, *nine) == api.TAC_ERR_BAD_K
    # gradients once per group of frames: the struct of include/tac.h, and what is refused
    assert ctypes.sizeof(api.tac_backward_desc_t) == 24
    mk = lambda **kw: api.tac_backward_desc_t(surrogate=api.TAC_SG_ARCTAN, detach_reset=1, alpha=2.0, **kw)
    for fmt in (api.TAC_IN_BITS_POOL2, api.TAC_IN_BITS_MAXPOOL2):
        assert call(_desc(in_format=fmt), mk(grad_in_per_group=1), *nine) == api.TAC_ERR_UNSUPPORTED
    assert call(d, mk(grad_out_group_K=api.TAC_MAX_K + 1, grad_out_group_beta=0.5), *nine) == api.TAC_ERR_BAD_K
    assert call(d, mk(grad_out_group_K=-1), *nine) == api.TAC_ERR_BAD_K
    assert call(d, mk(grad_out_group_K=4, grad_out_group_beta=1.5), *nine) == api.TAC_ERR_BAD_PARAM


def test_stack_backward_needs_membranes_and_input_gradients():
    L = api.lib()
    mk = lambda T, Cin, Cout, **kw: api.make_desc(T, 2, Cin, 8, 8, Cout, beta=0.9, theta=1.0, **kw)
    stack = _stack([mk(8, 2, 4, K=2, mode=api.TAC_COLLAPSE), mk(4, 4, 4, mode=api.TAC_PER_STEP)])
    grads = (api.tac_stack_grads_t * 2)()
    for g in grads:
        g.w_oihw = g.grad_y = g.grad_w = 0x3000
    bwd = api.tac_backward_desc_t(surrogate=api.TAC_SG_ARCTAN, detach_reset=1, alpha=2.0)
    fake = ctypes.c_void_p(0x1000)
    call = lambda: L.tac_stack_backward(stack, grads, ctypes.byref(bwd), 2, fake, fake, None)
    assert call() == api.TAC_ERR_NULL                      # no v_trace recorded
    for l in stack:
        l.v_trace = 0x4000
    assert call() == api.TAC_ERR_NULL                      # layer 1 has no grad_in to hand to layer 0
    assert L.tac_stack_backward(stack, None, ctypes.byref(bwd), 2, fake, fake, None) == api.TAC_ERR_NULL
    stack[1].desc.T = 5
    grads[1].grad_in = 0x5000
    assert call() == api.TAC_ERR_BAD_SHAPE                 # the stack itself does not chain


def test_pooled_output_validation_and_stack_chaining():
    # MaxPool(2) in the writer (Sec. 5.1 blocks): even output sizes, matrix-core kernels only
    ok = _desc(H=16, W=32, Cin=32, Cout=64, precision=api.TAC_BF16, out_format=api.TAC_OUT_BITS_MAXPOOL2)
    assert api.tac_select_kernel(ok) == api.TAC_KERNEL_MFMA
    assert api.tac_out_shape(ok)[1:] == (16, 32) and api.stored_out_shape(ok)[1:] == (8, 16)
    L = api.lib()
    odd = _desc(H=15, W=32, Cin=32, Cout=64, precision=api.TAC_BF16, out_format=api.TAC_OUT_BITS_MAXPOOL2)
    assert L.tac_select_kernel(ctypes.byref(odd)) == api.TAC_ERR_BAD_SHAPE
    fp32 = _desc(H=16, W=32, Cin=3, Cout=64, out_format=api.TAC_OUT_BITS_MAXPOOL2)      # vector kernel: no pooled output
    assert L.tac_select_kernel(ctypes.byref(fp32)) == api.TAC_ERR_UNSUPPORTED
    bad = _desc(H=16, W=32, out_format=7)
    assert L.tac_select_kernel(ctypes.byref(bad)) == api.TAC_ERR_BAD_PARAM
    # a stack: the layer behind a pooling writer sees half the size, as plain bits
    a = api.tac_stack_layer_t(desc=ok)
    nxt = _desc(T=api.tac_out_shape(ok)[0], H=8, W=16, Cin=64, Cout=32, precision=api.TAC_BF16)
    arr = (api.tac_stack_layer_t * 2)(a, api.tac_stack_layer_t(desc=nxt))
    assert api.tac_stack_check(arr) == (api.TAC_OK, -1)
    wrong = _desc(T=api.tac_out_shape(ok)[0], H=16, W=32, Cin=64, Cout=32, precision=api.TAC_BF16)
    arr = (api.tac_stack_layer_t * 2)(a, api.tac_stack_layer_t(desc=wrong))
    assert api.tac_stack_check(arr) == (api.TAC_ERR_BAD_SHAPE, 1)


def test_matrix_core_probe_rejects_bad_requests_before_any_launch():
    L = api.lib()
    fake = ctypes.c_void_p(0x1000)
    assert L.tac_mfma_probe(10, None, None) == api.TAC_ERR_NULL
    assert L.tac_mfma_probe(0, fake, None) == api.TAC_ERR_BAD_PARAM
    assert L.tac_mfma_probe(10, ctypes.c_void_p(0x1002), None) == api.TAC_ERR_ALIGN
    assert L.tac_mfma_probe_workgroups() % 4 == 0 and L.tac_mfma_probe_workgroups() > 0
