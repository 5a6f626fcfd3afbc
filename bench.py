#!/usr/bin/env python3
"""Benchmark of the conv-LIF layer (per-step / TAC / TAC-TP) on one MI355X.

A "step" is one call of tac_conv_lif over the whole synthetic input of the workload
(all T frames of all B samples, inputs already resident in HBM): spike loading, aggregation,
convolution, LIF and packed output.  Prints ONE JSON line:

  metric   spike-frames/s of the layer = B * T / latency (T is always the input T)
  value    for the headline mode (default TAC, K = 4) on the roofline workload (cfg5)
  roofline executed convolution FLOPs (2 B Ho Wo Cout Cin 9 T/K, the T/K stages the method
           needs) / average kernel duration (HIP events on the launch stream) against the
           dense bf16 MFMA peak
           traffic = HBM bytes of one launch from rocprofv3 counters (null when the kernel
           source has changed since they were taken)
  cpu_baseline  the CPU oracle timed on a bounded sample of the same workload
  config.aggregation_stage_GBps  packed input bytes / kernel duration: the rate at which the
           fused loader consumes spikes from HBM (it is not a separate pass)
  config.launch_per_group_ms  the headline mode as T/K launches of one group each, the membrane
           carried through v_inout, against ms_per_step for the single fused launch
  config.table  latency and speed-up over the per-step mode of the same kernel for every
           mode and K of the workload
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA
PEAK_FP32_TFLOPS = 157.3       # MI355X fp32 vector
CPU_SAMPLES = 40               # samples of the batch the CPU oracle is timed on (10-30 s of CPU work on cfg5)

# HBM traffic of one launch of the headline kernel (cfg5, TAC, K = 4), from two rocprofv3 --pmc
# runs (FETCH_SIZE, then WRITE_SIZE; summary and scale factors under profiles/).  The figures
# belong to one version of the kernel source: they are reported only while its hash matches.
TRAFFIC = {
    "kernel_source_sha256": "4ff995988f0643b646a289510e301c7cdc99ecab7b4fe2e2db74d97e70fddbc5",
    "workload": ("cfg5", "TAC", 4),
    "fetch_bytes": 538544600,
    "write_bytes": 134217728,
}


def measured_traffic(workload, mode, K):
    import hashlib
    src = os.path.join(ROOT, "paper_2603_13810_amd", "csrc", "tac_mfma.hip")
    try:
        sha = hashlib.sha256(open(src, "rb").read()).hexdigest()
    except OSError:
        return None
    if sha != TRAFFIC["kernel_source_sha256"] or TRAFFIC["workload"] != (workload, mode, K):
        return None
    return TRAFFIC["fetch_bytes"] + TRAFFIC["write_bytes"]


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=15)
    ap.add_argument("--workload", default="cfg5", choices=["cfg2", "cfg3", "cfg4", "cfg5"])
    ap.add_argument("--mode", default="TAC", choices=["per_step", "TAC", "TAC_TP"])
    ap.add_argument("--K", type=int, default=4)
    ap.add_argument("--rate", type=float, default=None, help="firing rate of the Bernoulli input (cfg5)")
    ap.add_argument("--no-table", action="store_true", help="time only the headline mode")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline")
    ap.add_argument("--batch", type=int, default=None, help="override the batch size (debugging only)")
    ap.add_argument("--backward", action="store_true",
                    help="also time the backward pass (surrogate-gradient BPTT) of the per-step layer and of the headline mode")
    return ap.parse_args()


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2603_13810_amd import api, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    dev = torch.device("cuda:0")
    wl = synth.WORKLOADS[args.workload]
    if len(wl.layers) > 1:
        return bench_stack(args, wl, dev)
    L = wl.layers[0]
    B = args.batch or wl.B
    T = wl.T
    rate = args.rate if args.rate is not None else wl.rate
    MODE = {"per_step": api.TAC_PER_STEP, "TAC": api.TAC_COLLAPSE, "TAC_TP": api.TAC_PRESERVE}

    # ---- synthetic input, resident in HBM, packed by the library's own packer
    Ww = (wl.W + 31) // 32
    spikes = torch.empty((T, B, wl.C, wl.H, Ww), dtype=torch.int32, device=dev)
    keep = {}                                    # dense frames of sample 0 for the CPU baseline
    if wl.spikes == "bernoulli":
        dense0 = np.empty((T, min(B, CPU_SAMPLES), wl.C, wl.H, wl.W), dtype=np.uint8)
        for t in range(T):
            fr = synth.bernoulli_device(wl.seed + t, B, wl.C, wl.H, wl.W, rate, dev)
            api.tac_pack_spikes(fr, spikes[t])
            dense0[t] = fr[:dense0.shape[1]].cpu().numpy()
            del fr
        keep["dense"] = dense0
    else:
        dense = wl.make_spikes(B=B)
        for t in range(T):
            api.tac_pack_spikes(torch.from_numpy(dense[t]).to(dev), spikes[t])
        keep["dense"] = dense[:, :CPU_SAMPLES]
    w32 = wl.make_weights(0)
    w_dev = torch.from_numpy(w32).to(dev)
    torch.cuda.synchronize()

    def make(mode, K):
        d = api.make_desc(T, B, L.Cin, wl.H, wl.W, L.Cout, K=K, beta=wl.beta, theta=wl.theta, mode=mode,
                          stride=L.stride, precision=api.TAC_BF16)
        wp = api.tac_prepare_weights(d, w_dev)
        T_out, Ho, Wo = api.tac_out_shape(d)
        out = torch.empty((T_out, B, L.Cout, Ho, (Wo + 31) // 32), dtype=torch.int32, device=dev)
        return d, wp, out, (T_out, Ho, Wo)

    def time_mode(mode, K, steps, warmup):
        d, wp, out, (T_out, Ho, Wo) = make(mode, K)
        for _ in range(warmup):
            api.tac_conv_lif(d, spikes, wp, None, None, out)
        torch.cuda.synchronize()
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
        t0 = time.perf_counter()
        for a, b in evs:
            a.record()
            api.tac_conv_lif(d, spikes, wp, None, None, out)
            b.record()
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t0) * 1e3 / steps
        kern_ms = float(np.mean([a.elapsed_time(b) for a, b in evs]))
        Kg = 1 if mode == api.TAC_PER_STEP else K
        flops = 2.0 * B * Ho * Wo * L.Cout * L.Cin * 9 * (T // Kg)
        fired = None
        return dict(mode=api.MODE_NAMES[mode], K=Kg, ms=wall_ms, kernel_ms=kern_ms, flops=flops,
                    kernel=("mfma" if api.tac_select_kernel(d) == api.TAC_KERNEL_MFMA else "direct"),
                    frames_per_s=B * T / (wall_ms * 1e-3), tflops=flops / (kern_ms * 1e-3) / 1e12,
                    out_bytes=out.numel() * 4)

    def time_per_group(mode, K, steps, warmup):
        """The same layer as one launch per group of K frames, the membrane carried through v_inout."""
        G = T // K
        d = api.make_desc(K, B, L.Cin, wl.H, wl.W, L.Cout, K=K, beta=wl.beta, theta=wl.theta, mode=mode,
                          stride=L.stride, precision=api.TAC_BF16)
        wp = api.tac_prepare_weights(d, w_dev)
        T_out, Ho, Wo = api.tac_out_shape(d)
        out = torch.empty((G * T_out, B, L.Cout, Ho, (Wo + 31) // 32), dtype=torch.int32, device=dev)
        v = torch.zeros((B, L.Cout, Ho, Wo), dtype=torch.float32, device=dev)

        def once():
            v.zero_()
            for g in range(G):
                api.tac_conv_lif(d, spikes[g * K:(g + 1) * K], wp, None, v, out[g * T_out:(g + 1) * T_out])
        for _ in range(warmup):
            once()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(steps):
            once()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / steps

    head = time_mode(MODE[args.mode], args.K, args.steps, args.warmup)
    per_group_ms = None
    if not args.no_table and args.mode != "per_step":
        per_group_ms = time_per_group(MODE[args.mode], args.K, max(3, args.steps // 4), 2)
    table = []
    if not args.no_table:
        base = time_mode(api.TAC_PER_STEP, 1, max(3, args.steps // 4), 2)
        table.append(dict(mode="per_step", K=1, ms=round(base["kernel_ms"], 4), speedup=1.0,
                          tflops=round(base["tflops"], 1)))
        for K in wl.Ks:
            if K == 1:
                continue
            for mode in (api.TAC_COLLAPSE, api.TAC_PRESERVE):
                r = time_mode(mode, K, max(3, args.steps // 4), 2)
                table.append(dict(mode=r["mode"], K=K, ms=round(r["kernel_ms"], 4),
                                  speedup=round(base["kernel_ms"] / r["kernel_ms"], 3), tflops=round(r["tflops"], 1)))

    backward = None
    if args.backward:
        def time_backward(mode, K):
            d, wp, out, (T_out, Ho, Wo) = make(mode, K)
            v = torch.zeros((B, L.Cout, Ho, Wo), dtype=torch.float32, device=dev)
            vt = torch.empty((T_out, B, L.Cout, Ho, Wo), dtype=torch.float32, device=dev)
            api.tac_conv_lif(d, spikes, wp, None, v, out, vt)          # the forward pass records the membranes
            gen = torch.Generator(device=dev)
            gen.manual_seed(wl.seed)
            g_out = torch.randn(vt.shape, device=dev, generator=gen)
            res = api.tac_conv_lif_backward(d, spikes, w_dev, vt, g_out, surrogate=api.TAC_SG_FAST_SIGMOID, alpha=25.0)
            torch.cuda.synchronize()
            del res
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            res = api.tac_conv_lif_backward(d, spikes, w_dev, vt, g_out, surrogate=api.TAC_SG_FAST_SIGMOID, alpha=25.0)
            b.record()
            torch.cuda.synchronize()
            Kg = 1 if mode == api.TAC_PER_STEP else K
            fl = 2 * 2.0 * B * Ho * Wo * L.Cout * L.Cin * 9 * (T // Kg)      # weight and input gradients
            return dict(mode=api.MODE_NAMES[mode], K=Kg, ms=round(a.elapsed_time(b), 3), conv_gradient_stages=T // Kg,
                        tflops=round(fl / (a.elapsed_time(b) * 1e-3) / 1e12, 2))
        backward = [time_backward(api.TAC_PER_STEP, 1)]
        for K in wl.Ks:
            if K > 1:
                backward.append(time_backward(api.TAC_COLLAPSE, K))
        fwd = {(r["mode"], r["K"]): r["ms"] for r in table}
        fwd[("per_step", 1)] = fwd.get(("per_step", 1), head["kernel_ms"] if args.mode == "per_step" else None)
        for r in backward:
            r["speedup"] = round(backward[0]["ms"] / r["ms"], 3)
            f, f0 = fwd.get((r["mode"], r["K"])), fwd.get(("per_step", 1))
            if f is not None and f0 is not None:      # forward + backward of the layer: one training step without the optimiser
                r["forward_plus_backward_ms"] = round(f + r["ms"], 3)
                r["training_step_speedup"] = round((f0 + backward[0]["ms"]) / (f + r["ms"]), 3)

    is_mfma = head["kernel"] == "mfma"
    peak = PEAK_BF16_TFLOPS if is_mfma else PEAK_FP32_TFLOPS
    roofline = dict(bound="mfma" if is_mfma else "alu", achieved=round(head["tflops"], 2), peak=peak,
                    unit="TFLOP/s", frac=round(head["tflops"] / peak, 4),
                    traffic=measured_traffic(wl.name, args.mode, head["K"]) if B == wl.B else None,
                    kernel_ms=round(head["kernel_ms"], 4),
                    algorithmic_bytes=int(spikes.numel() * 4 + head["out_bytes"]))

    cpu = None
    if not args.no_cpu:
        import oracle
        from oracle import PER_STEP, TAC, TAC_TP
        omode = {"per_step": PER_STEP, "TAC": TAC, "TAC_TP": TAC_TP}[args.mode]
        Kc = 1 if args.mode == "per_step" else args.K
        Tc = T
        sl = keep["dense"][:Tc]
        nth = oracle.max_threads()
        t0 = time.perf_counter()
        oracle.conv_lif(sl, w32.astype(np.float64), K=Kc, beta=wl.beta, theta=wl.theta, mode=omode,
                        stride=L.stride, nthreads=nth)
        dt = time.perf_counter() - t0
        cpu = dict(value=round(sl.shape[0] * sl.shape[1] / dt, 3), unit="spike-frames/s", cores=nth, kind="oracle",
                   sample="%d samples x %d frames of %s, mode %s K=%d, %.1f s wall" % (sl.shape[1], Tc, wl.name, args.mode, Kc, dt))

    line = {
        "metric": "spike-frames/s per conv-LIF layer",
        "value": round(head["frames_per_s"], 1),
        "unit": "spike-frames/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(head["ms"], 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "%s: conv-LIF 3x3 %d->%d, %dx%d, stride %d, B=%d, T=%d, Bernoulli rate %s, beta=%.2f"
                               % (wl.name, L.Cin, L.Cout, wl.H, wl.W, L.stride, B, T, rate, wl.beta),
                   "mode": args.mode, "K": head["K"], "kernel": head["kernel"],
                   "aggregation_stage_GBps": round(spikes.numel() * 4 / (head["kernel_ms"] * 1e-3) / 1e9, 1),
                   "launch_per_group_ms": None if per_group_ms is None else round(per_group_ms, 4),
                   "paper_context": "TAC training speed-ups 13.8x (Apple M3 Max) and 11.0x (NVIDIA V100), other hardware",
                   "table": table, "backward": backward},
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    print(json.dumps(line))


def bench_stack(args, wl, dev):
    """Multi-layer workloads (cfg2, cfg4): one step = all layers of the stack over the whole input,
    every inter-layer tensor packed bits in HBM, each layer fed the spikes the layer before wrote."""
    import torch
    from paper_2603_13810_amd import api
    MODE = {"per_step": api.TAC_PER_STEP, "TAC": api.TAC_COLLAPSE, "TAC_TP": api.TAC_PRESERVE}
    mode = MODE[args.mode]
    B, T0 = args.batch or wl.B, wl.T
    dense = wl.make_spikes(B=B)
    x0 = torch.empty((T0, B, wl.C, wl.H, (wl.W + 31) // 32), dtype=torch.int32, device=dev)
    for t in range(T0):
        api.tac_pack_spikes(torch.from_numpy(dense[t]).to(dev), x0[t])
    layers, T, H, W, flops = [], T0, wl.H, wl.W, 0.0
    for li, L in enumerate(wl.layers):
        if L.pool2_in:
            H, W = H // 2, W // 2
        K = args.K if (mode != api.TAC_PER_STEP and T % args.K == 0) else 1
        d = api.make_desc(T, B, L.Cin, H, W, L.Cout, K=K, beta=wl.beta, theta=wl.theta, mode=mode, stride=L.stride,
                          precision=api.TAC_BF16,
                          in_format=api.TAC_IN_BITS_POOL2 if L.pool2_in else api.TAC_IN_BITS)
        w32 = wl.make_weights(li)
        wp = api.tac_prepare_weights(d, torch.from_numpy(w32).to(dev))
        T_out, Ho, Wo = api.tac_out_shape(d)
        out = torch.empty((T_out, B, L.Cout, Ho, (Wo + 31) // 32), dtype=torch.int32, device=dev)
        Kg = 1 if mode == api.TAC_PER_STEP else K
        fl = 2.0 * B * Ho * Wo * L.Cout * L.Cin * 9 * (T // Kg)
        layers.append(dict(desc=d, wp=wp, out=out, w32=w32, K=K, flops=fl, stride=L.stride, pool2=L.pool2_in,
                           kernel="mfma" if api.tac_select_kernel(d) == api.TAC_KERNEL_MFMA else "direct",
                           shape="%d->%d %dx%d s%d T%d" % (L.Cin, L.Cout, H, W, L.stride, T)))
        flops += fl
        T, H, W = T_out, Ho, Wo

    stack, _ = api.make_stack([dict(desc=l["desc"], w_prepared=l["wp"], out_spikes_packed=l["out"]) for l in layers])

    def step():                                     # one call: every layer enqueued in order
        api.tac_stack_forward(stack, x0)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    t0 = time.perf_counter()
    for a, b in evs:
        a.record()
        step()
        b.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / args.steps
    kern_ms = float(np.mean([a.elapsed_time(b) for a, b in evs]))
    per_layer = []
    x = x0
    for l in layers:                                # each layer alone, same inputs
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(5):
            api.tac_conv_lif(l["desc"], x, l["wp"], None, None, l["out"])
        b.record()
        torch.cuda.synchronize()
        ms = a.elapsed_time(b) / 5
        per_layer.append(dict(layer=l["shape"], kernel=l["kernel"], K=l["K"], ms=round(ms, 4),
                              tflops=round(l["flops"] / (ms * 1e-3) / 1e12, 1),
                              out_rate=round(float(_bit_rate(l["out"])), 4)))
        x = l["out"]
    dom = max(per_layer, key=lambda r: r["ms"])
    dom_peak = PEAK_BF16_TFLOPS if dom["kernel"] == "mfma" else PEAK_FP32_TFLOPS
    cpu = None
    if not args.no_cpu:
        import oracle
        omode = {"per_step": oracle.PER_STEP, "TAC": oracle.TAC, "TAC_TP": oracle.TAC_TP}[args.mode]
        n_s = min(B, 16) if wl.name == "cfg4" else B
        xs = dense[:, :n_s]
        nth = oracle.max_threads()
        t0 = time.perf_counter()
        for l in layers:
            o = oracle.conv_lif(xs, l["w32"].astype(np.float64), K=l["K"], beta=wl.beta, theta=wl.theta, mode=omode,
                                stride=l["stride"], pool2=l["pool2"], nthreads=nth)
            xs = o[0]
        dt = time.perf_counter() - t0
        cpu = dict(value=round(n_s * T0 / dt, 3), unit="spike-frames/s", cores=nth, kind="oracle",
                   sample="%d sample(s) x %d frames through all %d layers of %s, mode %s K=%d, %.1f s wall" %
                          (n_s, T0, len(layers), wl.name, args.mode, args.K, dt))
    line = {
        "metric": "spike-frames/s through the layer stack", "value": round(B * T0 / (wall_ms * 1e-3), 1),
        "unit": "spike-frames/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(wall_ms, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "%s: %d conv-LIF layers, B=%d, T=%d, beta=%.2f" % (wl.name, len(layers), B, T0, wl.beta),
                   "mode": args.mode, "K": args.K, "layers": per_layer},
        # the layer that takes longest decides which roof the stack is held against
        "roofline": dict(bound="mfma" if dom["kernel"] == "mfma" else "alu",
                         achieved=round(flops / (kern_ms * 1e-3) / 1e12, 2), peak=dom_peak, unit="TFLOP/s",
                         frac=round(flops / (kern_ms * 1e-3) / 1e12 / dom_peak, 4), traffic=None,
                         kernel_ms=round(kern_ms, 4), dominant_layer=dom["layer"]),
        "cpu_baseline": cpu,
    }
    print(json.dumps(line))


def _bit_rate(packed):
    """Fraction of set bits in a packed tensor (pad bits are zero, so slightly below the firing rate)."""
    import torch
    x = packed.view(torch.uint8).to(torch.int16)
    cnt = torch.zeros((), dtype=torch.int64, device=packed.device)
    for sft in range(8):
        cnt += ((x >> sft) & 1).sum()
    return cnt.item() / (packed.numel() * 32)


if __name__ == "__main__":
    main()
