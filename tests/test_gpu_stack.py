"""Stacks of layers with per-layer mode and group size (App. B: TAC cascades T -> T/K_1 -> ..., TAC-TP keeps
T), packed spikes handed from layer to layer, run by one call through the C ABI; also recorded into a HIP graph."""
import numpy as np
import pytest
import torch

from paper_2603_13810_amd import api, synth
from gpu_util import run_oracle, ORACLE_MODE
from parity_util import np_pack, np_unpack, compare

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


def _build(spec, T, B, Cin, H, W, precision, seed, state=True, trace=True):
    """spec: list of (Cout, stride, pool before the layer, mode, K).  Returns (layer dicts, host weights/biases)."""
    layers, host = [], []
    r = _rng(seed)
    for i, (Cout, stride, pool, mode, K) in enumerate(spec):
        if pool:
            H, W = H // 2, W // 2
        fmt = {False: api.TAC_IN_BITS, True: api.TAC_IN_BITS_POOL2, "max": api.TAC_IN_BITS_MAXPOOL2}[pool]
        desc = api.make_desc(T, B, Cin, H, W, Cout, K=K, beta=0.9, theta=1.0, mode=mode, stride=stride, precision=precision,
                             in_format=fmt)
        w = synth.kaiming_normal(seed + i, Cout, Cin) * np.float32(2.0)
        bias = (r.standard_normal(Cout) * 0.1).astype(np.float32)
        T_out, Ho, Wo = api.tac_out_shape(desc)
        L = dict(desc=desc, w_prepared=api.tac_prepare_weights(desc, torch.from_numpy(w).to(DEV)),
                 bias=torch.from_numpy(bias).to(DEV))
        if state:
            L["v_inout"] = torch.zeros((B, Cout, Ho, Wo), dtype=torch.float32, device=DEV)
        if trace:
            L["v_trace"] = torch.full((T_out, B, Cout, Ho, Wo), float("nan"), dtype=torch.float32, device=DEV)
        layers.append(L)
        host.append((w, bias, stride, pool, mode, K))
        T, Cin, H, W = T_out, Cout, Ho, Wo
    return layers, host


STACKS = {
    # three TAC layers with K = 2 each: T = 16 -> 8 -> 4 -> 2 (App. B), vector kernel
    "cascade fp32": (16, 2, 16, 16, api.TAC_FP32,
                     [(8, 1, False, api.TAC_COLLAPSE, 2), (12, 2, False, api.TAC_COLLAPSE, 2), (16, 1, True, api.TAC_COLLAPSE, 2)]),
    # Conv-LIF-MaxPool blocks of the event-data network (Sec. 5.1) at reduced width, a group size per layer,
    # all three MFMA kernels (short contraction, long contraction twice, in between)
    "blocks bf16": (16, 2, 64, 64, api.TAC_BF16,
                    [(64, 1, False, api.TAC_PRESERVE, 4), (128, 1, "max", api.TAC_PRESERVE, 2),
                     (128, 1, False, api.TAC_COLLAPSE, 4), (128, 1, "max", api.TAC_PER_STEP, 1)]),
    # T = 25 as in the paper's runs: 25 -> 7 -> 7 -> 7 steps, shorter last groups in the first two layers
    "ragged bf16": (25, 2, 32, 32, api.TAC_BF16,
                    [(32, 1, False, api.TAC_COLLAPSE, 4), (64, 1, False, api.TAC_PRESERVE, 4), (128, 2, False, api.TAC_PER_STEP, 1)]),
}


@pytest.mark.parametrize("name", list(STACKS))
def test_stack_against_the_oracle_layer_after_layer(name):
    T, Cin, H, W, precision, spec = STACKS[name]
    B = 2
    r = _rng(700 + T + Cin + H)
    s = (r.random((T, B, Cin, H, W)) < 0.25).astype(np.uint8)
    layers, host = _build(spec, T, B, Cin, H, W, precision, seed=800 + T)
    stack, outs = api.make_stack(layers)
    assert api.tac_stack_check(stack) == (api.TAC_OK, -1)
    api.tac_reset_counters()
    api.tac_stack_forward(stack, torch.from_numpy(np_pack(s)).to(DEV))
    torch.cuda.synchronize()
    counters = api.tac_get_counters()
    # The oracle runs free, layer after layer on its own spikes.  The stack's output of a layer is compared with it
    # as long as every layer before came out identical; once a spike has flipped at the threshold the later layers
    # see other inputs on the two sides, and the comparison goes on with the layer called alone on the oracle's
    # spikes (that the stack's layers equal the layers called alone, bit for bit, is the next test).
    x, stages, steps, same = s, 0, 0, True
    for i, ((w, bias, stride, pool, mode, K), L) in enumerate(zip(host, layers)):
        ref = run_oracle(x, w, K=K, beta=0.9, theta=1.0, mode=mode, stride=stride, bias=bias, pool2=pool,
                         quantised=precision == api.TAC_BF16)
        Wo = ref[0].shape[-1]
        if not same:
            L["v_inout"].zero_()
            api.tac_conv_lif(L["desc"], torch.from_numpy(np_pack(x)).to(DEV), L["w_prepared"], L["bias"], L["v_inout"], outs[i],
                             L["v_trace"])
            torch.cuda.synchronize()
        got = np_unpack(outs[i].cpu().numpy(), Wo)
        par = compare(ref[0], ref[1], got, L["v_trace"].cpu().numpy(), 1.0, 1e-5 if precision == api.TAC_FP32 else 1e-3)
        assert par.ok, "layer %d: %s" % (i, par)
        assert ref[0].mean() > 0.002, "layer %d is silent" % i
        print("stack %s layer %d %s K=%d (%s): %s rate %.3f" % (name, i, api.MODE_NAMES[mode], K,
                                                              "from the stack" if same else "alone, on the oracle's spikes", par,
                                                              ref[0].mean()))
        Kg = 1 if mode == api.TAC_PER_STEP else min(K, x.shape[0])
        stages += -(-x.shape[0] // Kg)
        steps += ref[0].shape[0]
        same = same and par.flips == 0
        x = ref[0]
    assert counters == (stages, steps)


def test_stack_equals_the_layers_called_one_by_one():
    T, Cin, H, W, precision, spec = STACKS["ragged bf16"]
    r = _rng(901)
    s = torch.from_numpy(np_pack((r.random((T, 2, Cin, H, W)) < 0.25).astype(np.uint8))).to(DEV)
    layers, _ = _build(spec, T, 2, Cin, H, W, precision, seed=902)
    stack, outs = api.make_stack(layers)
    api.tac_stack_forward(stack, s)
    torch.cuda.synchronize()
    whole = [o.clone() for o in outs]
    finals = [L["v_inout"].clone() for L in layers]
    x = s
    for L in layers:
        L["v_inout"].zero_()
        x = api.tac_conv_lif(L["desc"], x, L["w_prepared"], L["bias"], L["v_inout"], None, None)
    torch.cuda.synchronize()
    assert torch.equal(x, whole[-1])
    assert all(torch.equal(L["v_inout"], f) for L, f in zip(layers, finals))


def test_stack_check_names_the_layer_that_does_not_fit():
    T, Cin, H, W, precision, spec = STACKS["cascade fp32"]
    layers, _ = _build(spec, T, 2, Cin, H, W, precision, seed=903, state=False, trace=False)
    stack, _ = api.make_stack(layers)
    stack[2].desc.T = 8                       # layer 1 hands over 4 steps
    assert api.tac_stack_check(stack) == (api.TAC_ERR_BAD_SHAPE, 2)
    stack[2].desc.T = 4
    stack[1].desc.Cin = 9
    assert api.tac_stack_check(stack) == (api.TAC_ERR_BAD_SHAPE, 1)
    with pytest.raises(api.TacError):
        api.tac_stack_forward(stack, torch.zeros(16 * 2 * 2 * 16, dtype=torch.int32, device=DEV))


def test_stack_recorded_into_a_graph_replays_like_the_eager_call():
    # no allocation, memset or synchronisation inside the call: capture the stream, replay several times with the
    # program's own eager work and synchronisations in between, every replay against the eager result
    T, Cin, H, W, precision, spec = STACKS["blocks bf16"]
    r = _rng(904)
    layers, _ = _build(spec, T, 2, Cin, H, W, precision, seed=905, state=False, trace=False)
    stack, outs = api.make_stack(layers)
    s = torch.from_numpy(np_pack((r.random((T, 2, Cin, H, W)) < 0.25).astype(np.uint8))).to(DEV)
    api.tac_stack_forward(stack, s)
    torch.cuda.synchronize()
    eager = [o.clone() for o in outs]
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.graph(graph, stream=side):
        api.tac_stack_forward(stack, s)
    for rep in range(3):
        for o in outs:
            o.fill_(-1)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert all(torch.equal(o, e) for o, e in zip(outs, eager)), "replay %d" % rep
        # new input in the same buffer: the graph reads it on the next replay
        s2 = torch.from_numpy(np_pack((r.random((T, 2, Cin, H, W)) < 0.25).astype(np.uint8))).to(DEV)
        keep = s.clone()
        s.copy_(s2)
        graph.replay()
        torch.cuda.synchronize()
        replayed = [o.clone() for o in outs]
        api.tac_stack_forward(stack, s)
        torch.cuda.synchronize()
        assert all(torch.equal(o, e) for o, e in zip(outs, replayed)), "replay %d on new input" % rep
        assert not torch.equal(outs[-1], eager[-1])
        s.copy_(keep)
