"""Seeded synthetic inputs shaped like the paper's workloads.

This module draws random numbers and nothing else: it contains none of the
method's arithmetic (no aggregation, convolution or LIF), so both the GPU
library's tests and the CPU oracle may be fed from it.

The paper trains on rate-coded MNIST / Fashion-MNIST (28x28, Poisson rate
coding, Sec. 5.1) and on DVS128-Gesture event frames (two polarity channels,
Sec. 5.1 and App. F).  Neither dataset is available, so the generators below
stand in for them with the same shapes and comparable firing statistics:

* ``rate_coded``    one rate map per sample, p ~ U[0,1] per pixel, then
                    independent Bernoulli(p) draws per timestep;
* ``event_camera``  sparse background (rate 0.02) with a 24x24 patch of rate
                    0.3 whose centre moves 4 px per timestep along a direction
                    drawn per sample;
* ``bernoulli``     i.i.d. Bernoulli(rate) frames for the roofline sweep.

All spike tensors are uint8 0/1 in the paper's layout S[T, B, C, H, W].
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Optional, Tuple

import numpy as np


def _rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(int(seed)))


def rate_coded(seed: int, T: int, B: int, C: int, H: int, W: int) -> np.ndarray:
    rng = _rng(seed)
    p = rng.random((B, C, H, W))
    u = rng.random((T, B, C, H, W))
    return (u < p[None]).astype(np.uint8)


def bernoulli(seed: int, T: int, B: int, C: int, H: int, W: int, rate: float) -> np.ndarray:
    rng = _rng(seed)
    out = np.empty((T, B, C, H, W), dtype=np.uint8)
    for t in range(T):
        out[t] = rng.random((B, C, H, W), dtype=np.float32) < np.float32(rate)
    return out


def event_camera(seed: int, T: int, B: int, H: int = 128, W: int = 128, C: int = 2,
                 base_rate: float = 0.02, patch_rate: float = 0.3, patch: int = 24,
                 speed: float = 4.0) -> np.ndarray:
    """Moving-patch event frames.  Sample b gets a direction phi_b ~ U[0, 2pi); the patch
    centre at step t is (H/2, W/2) + (t - (T-1)/2) * speed * (sin phi, cos phi), rounded to
    whole pixels, and the patch is clipped at the frame border.  All C channels share the
    rate map and are drawn independently."""
    rng = _rng(seed)
    phi = rng.random(B) * 2.0 * math.pi
    out = np.empty((T, B, C, H, W), dtype=np.uint8)
    half = patch // 2
    for t in range(T):
        rate = np.full((B, 1, H, W), base_rate, dtype=np.float32)
        for b in range(B):
            cy = int(round(H / 2 + (t - (T - 1) / 2) * speed * math.sin(phi[b])))
            cx = int(round(W / 2 + (t - (T - 1) / 2) * speed * math.cos(phi[b])))
            y0, y1 = max(cy - half, 0), min(cy - half + patch, H)
            x0, x1 = max(cx - half, 0), min(cx - half + patch, W)
            if y1 > y0 and x1 > x0:
                rate[b, 0, y0:y1, x0:x1] = patch_rate
        out[t] = rng.random((B, C, H, W), dtype=np.float32) < rate
    return out


def kaiming_normal(seed: int, Cout: int, Cin: int, kh: int = 3, kw: int = 3) -> np.ndarray:
    """float32 weights [Cout, Cin, kh, kw] ~ N(0, 2 / (Cin kh kw))."""
    rng = _rng(seed)
    std = math.sqrt(2.0 / (Cin * kh * kw))
    return (rng.standard_normal((Cout, Cin, kh, kw)) * std).astype(np.float32)


def bernoulli_device(seed: int, B: int, C: int, H: int, W: int, rate: float, device):
    """One i.i.d. Bernoulli(rate) frame [B, C, H, W] as a uint8 torch tensor, drawn on
    `device` (the full-size roofline inputs are too large to draw on the host)."""
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return (torch.rand((B, C, H, W), generator=g, device=device) < rate).to(torch.uint8)


# --------------------------------------------------------------------------------------
# The five benchmark configurations.
# --------------------------------------------------------------------------------------

@dataclass(frozen=True)
class LayerSpec:
    Cin: int
    Cout: int
    stride: int = 1
    pad: int = 1
    pool2_in: bool = False     # a 2x2 mean pool sits between the previous layer and this one


@dataclass(frozen=True)
class Workload:
    name: str
    T: int
    B: int
    C: int
    H: int
    W: int
    beta: float
    theta: float
    layers: Tuple[LayerSpec, ...]
    spikes: str                 # "rate" | "event" | "bernoulli"
    rate: Optional[float] = None
    seed: int = 0
    Ks: Tuple[int, ...] = (1,)
    note: str = ""

    def make_spikes(self, B: Optional[int] = None, T: Optional[int] = None,
                    rate: Optional[float] = None) -> np.ndarray:
        B = self.B if B is None else B
        T = self.T if T is None else T
        if self.spikes == "rate":
            return rate_coded(self.seed, T, B, self.C, self.H, self.W)
        if self.spikes == "event":
            return event_camera(self.seed, T, B, self.H, self.W, self.C)
        return bernoulli(self.seed, T, B, self.C, self.H, self.W,
                         self.rate if rate is None else rate)

    def make_weights(self, layer: int = 0) -> np.ndarray:
        L = self.layers[layer]
        return kaiming_normal(self.seed * 100 + 17 + layer, L.Cout, L.Cin)


WORKLOADS = {
    # single small layer, fp32, TAC K=2
    "cfg1": Workload("cfg1", T=4, B=4, C=1, H=28, W=28, beta=0.9, theta=1.0,
                     layers=(LayerSpec(1, 8),), spikes="rate", seed=1000, Ks=(2,)),
    # two-layer rate-coded net: conv 1->32, LIF, 2x2 mean pool, conv 32->64, LIF
    "cfg2": Workload("cfg2", T=8, B=128, C=1, H=28, W=28, beta=0.9, theta=1.0,
                     layers=(LayerSpec(1, 32), LayerSpec(32, 64, pool2_in=True)),
                     spikes="rate", seed=2000, Ks=(2, 4, 8)),
    # event-camera-shaped single layer, stride 2
    "cfg3": Workload("cfg3", T=16, B=32, C=2, H=128, W=128, beta=0.5, theta=1.0,
                     layers=(LayerSpec(2, 64, stride=2),), spikes="event", seed=3000, Ks=(2,)),
    # five-layer VGG-style event stack
    "cfg4": Workload("cfg4", T=16, B=16, C=2, H=128, W=128, beta=0.5, theta=1.0,
                     layers=(LayerSpec(2, 64, stride=2), LayerSpec(64, 128), LayerSpec(128, 128, stride=2),
                             LayerSpec(128, 256), LayerSpec(256, 256, stride=2)),
                     spikes="event", seed=4000, Ks=(2, 4)),
    # large roofline sweep
    "cfg5": Workload("cfg5", T=32, B=256, C=128, H=64, W=64, beta=0.9, theta=1.0,
                     layers=(LayerSpec(128, 128),), spikes="bernoulli", rate=0.1, seed=5000,
                     Ks=(1, 2, 4, 8, 16)),
}
