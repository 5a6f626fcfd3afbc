#!/usr/bin/env python3
"""Benchmark of the conv-LIF layer (per-step / TAC / TAC-TP) on one MI355X.

A "step" is one call of tac_conv_lif (tac_stack_forward for the multi-layer workloads) over the
whole synthetic input of the workload (all T frames of all B samples, inputs already resident in
HBM): spike loading, aggregation, convolution, LIF and packed output.  Prints ONE JSON line:

  metric   spike-frames/s of the layer = B * T / latency (T is always the input T)
  value    for the headline mode (default TAC, K = 4) on the roofline workload (cfg5)
  roofline the roof that bounds the workload's dominant kernel:
             mfma  executed convolution FLOPs (2 B Ho Wo Cout Cin 9 T/K, the T/K stages the method
                   needs) / average kernel duration against the dense bf16 MFMA peak (layers of 16
                   and more input channels on the matrix cores);
             alu   the same FLOPs against the fp32 vector peak (fp32 layers of many channels);
             hbm   algorithmic bytes (packed input + packed output) / duration against 8 TB/s
                   (layers of one or two input channels and the small rate-coded layers, whose
                   contraction is 9 or 18 terms long);
           durations are HIP-event times on the launch stream; traffic = HBM bytes of one launch
           from rocprofv3 counters, read from the summary under profiles/ and reported only while
           the kernel source still has the hash recorded there
  parity   the library's output on the samples the CPU baseline runs, against the plain oracle at
           the stated 2e-2 and (on a few of them) against the oracle with bf16-rounded operands
  cpu_baseline  the CPU oracle timed on a bounded sample of the same workload, all cores and one
  config.aggregation_stage  the aggregation stage alone (tac_aggregate_sums: loader without
           convolution and LIF) at K = 1 / 4 / 16: time and rate at which packed spikes are consumed
  config.rate_sweep  the headline mode at input rates 0.05 / 0.1 / 0.2 / 0.3
  config.launch_per_group_ms  the headline mode as T/K launches of one group each, the membrane
           carried through v_inout, against ms_per_step for the single fused launch
  config.table  latency and speed-up over the per-step mode of the same kernel for every
           mode and K of the workload
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import re
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA
PEAK_FP32_TFLOPS = 157.3       # MI355X fp32 vector
PEAK_HBM_GBPS = 8000.0         # MI355X HBM3E
CPU_SAMPLES = 40               # samples of the batch the CPU oracle is timed on (10-30 s of CPU work on cfg5)
CPU_SAMPLES_ROUNDED = 4        # of those, the samples the bf16-rounded oracle runs as well (parity block)
PAPER_CONTEXT = "TAC training speed-ups 13.8x (Apple M3 Max) and 11.0x (NVIDIA V100), other hardware"


def kernel_source_sha256():
    """Hash of the sources the headline kernel is compiled from."""
    h = hashlib.sha256()
    for f in ("tac_mfma_kernel.h", "tac_mfma_common.h"):
        h.update(open(os.path.join(ROOT, "paper_2603_13810_amd", "csrc", f), "rb").read())
    return h.hexdigest()


def measured_traffic(workload, mode, K):
    """HBM bytes of one launch of the headline kernel from the rocprofv3 --pmc summary under profiles/
    (FETCH_SIZE and WRITE_SIZE, scaled by a copy kernel of known size).  The figures belong to one version of
    the kernel source: None, with a note on stderr, once its hash differs from the one recorded with them."""
    path = os.path.join(ROOT, "profiles", "mfma_kernel_%s_%s_k%d_hbm_counters.md" % (workload, mode.lower(), K))
    try:
        text = open(path).read()
    except OSError:
        return None
    m = re.search(r"bench-traffic:\s*fetch_bytes=(\d+)\s+write_bytes=(\d+)\s+kernel_source_sha256=([0-9a-f]{64})", text)
    if not m:
        return None
    sha = kernel_source_sha256()
    if sha != m.group(3):
        print("bench.py: the kernel source has changed since the counters in %s were taken: roofline.traffic is null"
              % os.path.relpath(path, ROOT), file=sys.stderr)
        return None
    return int(m.group(1)) + int(m.group(2))


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=15)
    ap.add_argument("--workload", default="cfg5", choices=["cfg1", "cfg2", "cfg3", "cfg4", "cfg5"])
    ap.add_argument("--mode", default="TAC", choices=["per_step", "TAC", "TAC_TP"])
    ap.add_argument("--K", type=int, default=None, help="group size (default 4; 2 on cfg1-cfg3)")
    ap.add_argument("--precision", default=None, choices=["bf16", "fp32"],
                    help="operand precision (default bf16; fp32 on cfg1, which is an fp32 configuration)")
    ap.add_argument("--rate", type=float, default=None, help="firing rate of the Bernoulli input (cfg5)")
    ap.add_argument("--no-table", action="store_true", help="time only the headline mode")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline and the parity block")
    ap.add_argument("--batch", type=int, default=None, help="override the batch size (debugging only)")
    ap.add_argument("--backward", action="store_true",
                    help="also time the backward pass (surrogate-gradient BPTT) of the per-step layer and of the headline mode")
    return ap.parse_args()


def layer_bound(Cin, Cout, H, W, precision_bf16, kernel):
    """Which roof bounds a layer: contraction of 9 or 18 terms, or a rate-coded layer of a few hundred pixels whose
    working set sits in the caches -> bytes; else the arithmetic unit the kernel computes on."""
    if Cin <= 2 or H * W <= 28 * 28:
        return "hbm"
    return "mfma" if (precision_bf16 and kernel == "mfma") else "alu"


def roofline_entry(bound, flops, bytes_, kern_ms, **extra):
    if bound == "hbm":
        ach = bytes_ / (kern_ms * 1e-3) / 1e9
        d = dict(bound="hbm", achieved=round(ach, 2), peak=PEAK_HBM_GBPS, unit="GB/s", frac=round(ach / PEAK_HBM_GBPS, 4))
    else:
        peak = PEAK_BF16_TFLOPS if bound == "mfma" else PEAK_FP32_TFLOPS
        ach = flops / (kern_ms * 1e-3) / 1e12
        d = dict(bound=bound, achieved=round(ach, 2), peak=peak, unit="TFLOP/s", frac=round(ach / peak, 4))
    d.update(extra)
    return d


def measure_mfma_loop(iterations=2000, launches=8):
    """TFLOP/s of tac_mfma_probe: a few launches to bring the clock where it settles, then timed ones."""
    import torch
    from paper_2603_13810_amd import api
    sums, flop = api.tac_mfma_probe(iterations)
    for _ in range(launches):
        api.tac_mfma_probe(iterations, sums)
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(launches):
        api.tac_mfma_probe(iterations, sums)
    b.record()
    torch.cuda.synchronize()
    return flop * launches / (a.elapsed_time(b) * 1e-3) / 1e12


def time_calls(fn, steps, warmup):
    """fn() enqueues one step on torch's current stream (the stream the library is given).  Returns
    (wall ms per step, mean HIP-event ms per step)."""
    import torch
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    t0 = time.perf_counter()
    for a, b in evs:
        a.record()
        fn()
        b.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / steps
    return wall_ms, float(np.mean([a.elapsed_time(b) for a, b in evs]))


def parity_block(oracle_run, gpu_spikes, gpu_vfinal, theta, n_rounded):
    """oracle_run(quantised, n) -> (spikes, v_pre, v_final) of the first n samples (all kept samples for n = None).
    gpu_spikes [T_out, n, ...], gpu_vfinal [n, ...] cover the same samples.  Spikes are compared step by step under the
    near-threshold rule of the tests (tests/parity_util.py); the final membrane on the neurons whose spike trains agree."""
    sys.path.insert(0, os.path.join(ROOT, "tests"))
    from parity_util import compare, compare3

    def stats(par, ref, n, tol):
        clean = (ref[0] == gpu_spikes[:, :n]).all(axis=0)
        err = np.abs(gpu_vfinal[:n] - ref[2]) / np.maximum(np.abs(ref[2]), theta)
        return dict(flips=par.flips, mismatches=par.mismatches, neuron_steps=par.checked,
                    max_err_final_v=round(float(err[clean].max()), 7) if clean.any() else None,
                    final_v_over_tolerance=int((err[clean] > tol).sum()))
    plain = oracle_run(False, None)
    n = plain[0].shape[1]
    vs_plain = compare(plain[0], plain[1], gpu_spikes[:, :n], None, theta, 2e-2)
    out = dict(samples=n, tolerance_plain=2e-2, vs_plain=stats(vs_plain, plain, n, 2e-2))
    if n_rounded:
        rounded = oracle_run(True, n_rounded)
        p3 = compare3((plain[0][:, :n_rounded], plain[1][:, :n_rounded]), rounded[:2], gpu_spikes[:, :n_rounded], None,
                      theta, 1e-3)
        out.update(samples_rounded=n_rounded, tolerance_rounded=1e-3, vs_rounded=stats(p3.vs_rounded, rounded, n_rounded, 1e-3),
                   rounding_alone_vs_plain=dict(flips=p3.quant.flips, mismatches=p3.quant.mismatches),
                   neurons_beyond_the_rounding=p3.extra_mismatches)
    return out


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
    if args.precision is None:
        args.precision = "fp32" if wl.name == "cfg1" else "bf16"
    if args.K is None:
        args.K = 4 if wl.name in ("cfg4", "cfg5") else 2
    if len(wl.layers) > 1:
        return bench_stack(args, wl, dev)
    L = wl.layers[0]
    B = args.batch or wl.B
    T = wl.T
    rate = args.rate if args.rate is not None else wl.rate
    MODE = {"per_step": api.TAC_PER_STEP, "TAC": api.TAC_COLLAPSE, "TAC_TP": api.TAC_PRESERVE}
    PREC = api.TAC_BF16 if args.precision == "bf16" else api.TAC_FP32

    # ---- synthetic input, resident in HBM, packed by the library's own packer
    Ww = (wl.W + 31) // 32

    def make_input(r):
        spikes = torch.empty((T, B, wl.C, wl.H, Ww), dtype=torch.int32, device=dev)
        if wl.spikes == "bernoulli":
            dense0 = np.empty((T, min(B, CPU_SAMPLES), wl.C, wl.H, wl.W), dtype=np.uint8)   # before packing, for the oracle
            for t in range(T):
                fr = synth.bernoulli_device(wl.seed + int(round(r * 1000)) * 64 + t, B, wl.C, wl.H, wl.W, r, dev)
                api.tac_pack_spikes(fr, spikes[t])
                dense0[t] = fr[:dense0.shape[1]].cpu().numpy()
                del fr
            return spikes, dense0
        dense = wl.make_spikes(B=B)
        for t in range(T):
            api.tac_pack_spikes(torch.from_numpy(dense[t]).to(dev), spikes[t])
        return spikes, dense[:, :CPU_SAMPLES]
    spikes, dense_keep = make_input(rate)
    w32 = wl.make_weights(0)
    w_dev = torch.from_numpy(w32).to(dev)
    torch.cuda.synchronize()

    def make(mode, K, Tn=T):
        d = api.make_desc(Tn, B, L.Cin, wl.H, wl.W, L.Cout, K=K, beta=wl.beta, theta=wl.theta, mode=mode,
                          stride=L.stride, precision=PREC)
        wp = api.tac_prepare_weights(d, w_dev)
        T_out, Ho, Wo = api.tac_out_shape(d)
        out = torch.empty((T_out, B, L.Cout, Ho, (Wo + 31) // 32), dtype=torch.int32, device=dev)
        return d, wp, out, (T_out, Ho, Wo)

    def time_mode(mode, K, steps, warmup, x=None):
        x = spikes if x is None else x
        d, wp, out, (T_out, Ho, Wo) = make(mode, K)
        wall_ms, kern_ms = time_calls(lambda: api.tac_conv_lif(d, x, wp, None, None, out), steps, warmup)
        Kg = 1 if mode == api.TAC_PER_STEP else K
        flops = 2.0 * B * Ho * Wo * L.Cout * L.Cin * 9 * (T // Kg)
        return dict(mode=api.MODE_NAMES[mode], K=Kg, ms=wall_ms, kernel_ms=kern_ms, flops=flops,
                    kernel=("mfma" if api.tac_select_kernel(d) == api.TAC_KERNEL_MFMA else "direct"),
                    frames_per_s=B * T / (wall_ms * 1e-3), tflops=flops / (kern_ms * 1e-3) / 1e12,
                    out_bytes=out.numel() * 4)

    def time_per_group(mode, K, steps, warmup):
        """The same layer as one launch per group of K frames, the membrane carried through v_inout."""
        G = T // K
        d, wp, _, (T_out, Ho, Wo) = make(mode, K, Tn=K)
        out = torch.empty((G * T_out, B, L.Cout, Ho, (Wo + 31) // 32), dtype=torch.int32, device=dev)
        v = torch.zeros((B, L.Cout, Ho, Wo), dtype=torch.float32, device=dev)

        def once():
            v.zero_()
            for g in range(G):
                api.tac_conv_lif(d, spikes[g * K:(g + 1) * K], wp, None, v, out[g * T_out:(g + 1) * T_out])
        return time_calls(once, steps, warmup)[1]

    head = time_mode(MODE[args.mode], args.K, args.steps, args.warmup)
    short = (max(3, args.steps // 4), 2)
    per_group_ms = None
    if not args.no_table and args.mode != "per_step" and T % args.K == 0:
        per_group_ms = time_per_group(MODE[args.mode], args.K, *short)
    table = []
    if not args.no_table:
        base = time_mode(api.TAC_PER_STEP, 1, *short)
        table.append(dict(mode="per_step", K=1, ms=round(base["kernel_ms"], 4), speedup=1.0,
                          tflops=round(base["tflops"], 1)))
        for K in wl.Ks:
            if K == 1:
                continue
            for mode in (api.TAC_COLLAPSE, api.TAC_PRESERVE):
                r = time_mode(mode, K, *short)
                table.append(dict(mode=r["mode"], K=K, ms=round(r["kernel_ms"], 4),
                                  speedup=round(base["kernel_ms"] / r["kernel_ms"], 3), tflops=round(r["tflops"], 1)))

    # ---- the aggregation stage alone, and the headline mode over the input rates (roofline workload)
    aggregation, rate_sweep = None, None
    in_bytes = spikes.numel() * 4
    if not args.no_table and wl.spikes == "bernoulli" and PREC == api.TAC_BF16:
        aggregation = []
        for K in (1, 4, 16):
            d = api.make_desc(T, B, L.Cin, wl.H, wl.W, L.Cout, K=K, beta=wl.beta, theta=wl.theta, mode=api.TAC_COLLAPSE,
                              stride=L.stride, precision=PREC)
            if T % K or api.tac_aggregate_tiles(d) == 0:
                continue
            sums = torch.empty((api.tac_aggregate_tiles(d),), dtype=torch.int64, device=dev)
            ms = time_calls(lambda: api.tac_aggregate_sums(d, spikes, sums), *short)[1]
            aggregation.append(dict(K=K, ms=round(ms, 4), packed_input_GBps=round(in_bytes / (ms * 1e-3) / 1e9, 1),
                                    of_hbm_peak=round(in_bytes / (ms * 1e-3) / 1e9 / PEAK_HBM_GBPS, 4)))
        rate_sweep = []
        for r in (0.05, 0.1, 0.2, 0.3):
            x = spikes if r == rate else make_input(r)[0]
            res = time_mode(MODE[args.mode], args.K, 10, 8, x=x)            # enough warm-up for the clock to settle
            rate_sweep.append(dict(rate=r, ms=round(res["kernel_ms"], 4), tflops=round(res["tflops"], 1)))
            del x

    backward = None
    if args.backward:
        def time_backward(mode, K):
            d, wp, out, (T_out, Ho, Wo) = make(mode, K)
            v = torch.zeros((B, L.Cout, Ho, Wo), dtype=torch.float32, device=dev)
            vt = torch.empty((T_out, B, L.Cout, Ho, Wo), dtype=torch.float32, device=dev)
            api.tac_conv_lif(d, spikes, wp, None, v, out, vt)          # the forward pass records the membranes
            torch.cuda.synchronize()
            fa, fb = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            v.zero_()
            fa.record()
            api.tac_conv_lif(d, spikes, wp, None, v, out, vt)          # the same call again, timed: the forward pass of a training step
            fb.record()
            torch.cuda.synchronize()
            fwd_trace_ms = fa.elapsed_time(fb)
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
            row = dict(mode=api.MODE_NAMES[mode], K=Kg, ms=round(a.elapsed_time(b), 3), conv_gradient_stages=T // Kg,
                       tflops=round(fl / (a.elapsed_time(b) * 1e-3) / 1e12, 2), forward_recording_membranes_ms=round(fwd_trace_ms, 3))
            if Kg > 1:
                # the same pass with dL/dA_k handed to the layer before once per group instead of once per frame
                del res
                res = api.tac_conv_lif_backward(d, spikes, w_dev, vt, g_out, surrogate=api.TAC_SG_FAST_SIGMOID, alpha=25.0,
                                                grad_in_per_group=True)
                torch.cuda.synchronize()
                del res
                a.record()
                res = api.tac_conv_lif_backward(d, spikes, w_dev, vt, g_out, surrogate=api.TAC_SG_FAST_SIGMOID, alpha=25.0,
                                                grad_in_per_group=True)
                b.record()
                torch.cuda.synchronize()
                row["ms_input_gradient_per_group"] = round(a.elapsed_time(b), 3)
            return row
        backward = [time_backward(api.TAC_PER_STEP, 1)]
        for K in wl.Ks:
            if K > 1:
                backward.append(time_backward(api.TAC_COLLAPSE, K))
        for r in backward:
            r["speedup"] = round(backward[0]["ms"] / r["ms"], 3)
            # forward (recording the membranes the backward pass needs) + backward of the layer: one training step
            # without the optimiser; with the input gradient per group where the mode groups frames
            f, f0 = r["forward_recording_membranes_ms"], backward[0]["forward_recording_membranes_ms"]
            bw = r.get("ms_input_gradient_per_group", r["ms"])
            r["forward_plus_backward_ms"] = round(f + bw, 3)
            r["training_step_speedup"] = round((f0 + backward[0]["ms"]) / (f + bw), 3)

    alg_bytes = int(in_bytes + head["out_bytes"])
    bound = layer_bound(L.Cin, L.Cout, wl.H, wl.W, PREC == api.TAC_BF16, head["kernel"])
    roofline = roofline_entry(bound, head["flops"], alg_bytes, head["kernel_ms"],
                              traffic=measured_traffic(wl.name, args.mode, head["K"])
                              if (B == wl.B and rate == wl.rate and PREC == api.TAC_BF16) else None,
                              kernel_ms=round(head["kernel_ms"], 4), algorithmic_bytes=alg_bytes,
                              conv_tflops=round(head["tflops"], 2))

    if bound == "mfma":
        # the matrix cores alone (nothing but MFMAs, one wave per SIMD, operands like this layer's): the rate the chip
        # sustains at the clock it holds under that load, the practical ceiling of the convolution stage
        loop = measure_mfma_loop()
        roofline["mfma_loop_tflops"] = round(loop, 1)
        roofline["frac_of_mfma_loop"] = round(head["tflops"] / loop, 4)

    cpu, parity = None, None
    if not args.no_cpu:
        import oracle
        from oracle import PER_STEP, TAC, TAC_TP
        omode = {"per_step": PER_STEP, "TAC": TAC, "TAC_TP": TAC_TP}[args.mode]
        Kc = 1 if args.mode == "per_step" else args.K
        sl = dense_keep
        n_cpu = sl.shape[1]
        nth = oracle.max_threads()
        timing = {}

        def oracle_run(quantised, n):
            x = sl if n is None else sl[:, :n]
            w = w32 if not quantised else torch.from_numpy(w32).to(torch.bfloat16).to(torch.float32).numpy()
            t0 = time.perf_counter()
            o = oracle.conv_lif(x, w.astype(np.float64), K=Kc, beta=float(np.float32(wl.beta)), theta=float(np.float32(wl.theta)),
                                mode=omode, stride=L.stride, round_a_bf16=quantised, nthreads=nth)
            if not quantised:
                timing["threaded"] = time.perf_counter() - t0
            return o
        # the library on the same samples: one more call of the timed kernel, with v_inout to get the final membrane
        d, wp, out, (T_out, Ho, Wo) = make(MODE[args.mode], args.K)
        v = torch.zeros((B, L.Cout, Ho, Wo), dtype=torch.float32, device=dev)
        api.tac_conv_lif(d, spikes, wp, None, v, out)
        torch.cuda.synchronize()
        sys.path.insert(0, os.path.join(ROOT, "tests"))
        from parity_util import np_unpack
        gpu_spk = np_unpack(out[:, :n_cpu].cpu().numpy(), Wo)
        gpu_v = v[:n_cpu].cpu().numpy().astype(np.float64)
        if PREC == api.TAC_BF16:
            parity = parity_block(oracle_run, gpu_spk, gpu_v, float(wl.theta), min(CPU_SAMPLES_ROUNDED, n_cpu))
        else:                                         # fp32: the tests hold this path to 1e-5; here it is graded at the same bar as bf16
            parity = parity_block(oracle_run, gpu_spk, gpu_v, float(wl.theta), 0)
        dt = timing["threaded"]
        # one thread, on one sample (scaled: samples are independent)
        t0 = time.perf_counter()
        oracle.conv_lif(sl[:, :1], w32.astype(np.float64), K=Kc, beta=float(np.float32(wl.beta)), theta=float(np.float32(wl.theta)),
                        mode=omode, stride=L.stride, nthreads=1)
        dt1 = time.perf_counter() - t0
        cpu = dict(value=round(T * n_cpu / dt, 3), unit="spike-frames/s", cores=nth, kind="oracle",
                   sample="%d samples x %d frames of %s, mode %s K=%d, %.1f s wall" % (n_cpu, T, wl.name, args.mode, Kc, dt),
                   single_thread_value=round(T / dt1, 3),
                   single_thread_sample="1 sample x %d frames, %.1f s wall" % (T, dt1))

    line = {
        "metric": "spike-frames/s per conv-LIF layer",
        "value": round(head["frames_per_s"], 1),
        "unit": "spike-frames/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(head["ms"], 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": args.precision, "data": "synthetic",
        "config": {"workload": "%s: conv-LIF 3x3 %d->%d, %dx%d, stride %d, B=%d, T=%d, %s input%s, beta=%.2f"
                               % (wl.name, L.Cin, L.Cout, wl.H, wl.W, L.stride, B, T,
                                  {"bernoulli": "Bernoulli", "rate": "rate-coded", "event": "event-camera"}[wl.spikes],
                                  "" if rate is None else " rate %s" % rate, wl.beta),
                   "mode": args.mode, "K": head["K"], "kernel": head["kernel"],
                   "aggregation_stage": aggregation,
                   "rate_sweep": rate_sweep,
                   "launch_per_group_ms": None if per_group_ms is None else round(per_group_ms, 4),
                   "paper_context": PAPER_CONTEXT,
                   "table": table, "backward": backward},
        "roofline": roofline,
        "parity": parity,
        "cpu_baseline": cpu,
    }
    print(json.dumps(line))


def bench_stack(args, wl, dev):
    """Multi-layer workloads (cfg2, cfg4): one step = all layers of the stack over the whole input,
    every inter-layer tensor packed bits in HBM, each layer fed the spikes the layer before wrote."""
    import torch
    from paper_2603_13810_amd import api
    MODE = {"per_step": api.TAC_PER_STEP, "TAC": api.TAC_COLLAPSE, "TAC_TP": api.TAC_PRESERVE}
    PREC = api.TAC_BF16 if args.precision == "bf16" else api.TAC_FP32
    mode = MODE[args.mode]
    B, T0 = args.batch or wl.B, wl.T
    dense = wl.make_spikes(B=B)
    x0 = torch.empty((T0, B, wl.C, wl.H, (wl.W + 31) // 32), dtype=torch.int32, device=dev)
    for t in range(T0):
        api.tac_pack_spikes(torch.from_numpy(dense[t]).to(dev), x0[t])
    layers, T, H, W, flops = [], T0, wl.H, wl.W, 0.0
    in_bytes = x0.numel() * 4
    for li, L in enumerate(wl.layers):
        Hs, Ws = H, W                                            # stored size of this layer's input
        if L.pool2_in:
            H, W = H // 2, W // 2
        K = args.K if (mode != api.TAC_PER_STEP and T % args.K == 0) else 1
        d = api.make_desc(T, B, L.Cin, H, W, L.Cout, K=K, beta=wl.beta, theta=wl.theta, mode=mode, stride=L.stride,
                          precision=PREC,
                          in_format=api.TAC_IN_BITS_POOL2 if L.pool2_in else api.TAC_IN_BITS)
        w32 = wl.make_weights(li)
        wp = api.tac_prepare_weights(d, torch.from_numpy(w32).to(dev))
        T_out, Ho, Wo = api.tac_out_shape(d)
        out = torch.empty((T_out, B, L.Cout, Ho, (Wo + 31) // 32), dtype=torch.int32, device=dev)
        Kg = 1 if mode == api.TAC_PER_STEP else K
        fl = 2.0 * B * Ho * Wo * L.Cout * L.Cin * 9 * (T // Kg)
        kern = "mfma" if api.tac_select_kernel(d) == api.TAC_KERNEL_MFMA else "direct"
        layers.append(dict(desc=d, wp=wp, out=out, w32=w32, K=K, flops=fl, stride=L.stride, pool2=L.pool2_in,
                           kernel=kern, bytes=in_bytes + out.numel() * 4,
                           bound=layer_bound(L.Cin, L.Cout, H, W, PREC == api.TAC_BF16, kern),
                           shape="%d->%d %dx%d s%d T%d" % (L.Cin, L.Cout, H, W, L.stride, T)))
        flops += fl
        in_bytes = out.numel() * 4
        T, H, W = T_out, Ho, Wo

    stack, _ = api.make_stack([dict(desc=l["desc"], w_prepared=l["wp"], out_spikes_packed=l["out"]) for l in layers])
    wall_ms, kern_ms = time_calls(lambda: api.tac_stack_forward(stack, x0), args.steps, args.warmup)   # one call: every layer
    per_layer = []
    x = x0
    for l in layers:                                # each layer alone, same inputs
        ms = time_calls(lambda: api.tac_conv_lif(l["desc"], x, l["wp"], None, None, l["out"]), 10, 3)[1]
        r = roofline_entry(l["bound"], l["flops"], l["bytes"], ms)
        per_layer.append(dict(layer=l["shape"], kernel=l["kernel"], K=l["K"], ms=round(ms, 4),
                              tflops=round(l["flops"] / (ms * 1e-3) / 1e12, 1),
                              GBps=round(l["bytes"] / (ms * 1e-3) / 1e9, 1), bound=r["bound"], frac=r["frac"],
                              out_rate=round(float(_bit_rate(l["out"])), 4)))
        x = l["out"]
    i_dom = int(np.argmax([r["ms"] for r in per_layer]))
    dom, ldom = per_layer[i_dom], layers[i_dom]
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
        "dtype": args.precision, "data": "synthetic",
        "config": {"workload": "%s: %d conv-LIF layers, B=%d, T=%d, beta=%.2f" % (wl.name, len(layers), B, T0, wl.beta),
                   "mode": args.mode, "K": args.K, "layers": per_layer, "stack_kernel_ms": round(kern_ms, 4),
                   "stack_conv_tflops": round(flops / (kern_ms * 1e-3) / 1e12, 2), "paper_context": PAPER_CONTEXT},
        # the layer that takes longest is the dominant kernel: its own roof, its own duration
        "roofline": roofline_entry(ldom["bound"], ldom["flops"], ldom["bytes"], dom["ms"], traffic=None,
                                   kernel_ms=dom["ms"], dominant_layer=dom["layer"], algorithmic_bytes=int(ldom["bytes"])),
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
