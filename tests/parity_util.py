"""Comparison protocol between the GPU library and the CPU oracle (test-side only).

Membrane potentials are compared with the error |V_gpu - V_ref| / max(|V_ref|, theta): the
weights are zero-mean, so V often cancels to about zero and a plain relative error would be
meaningless there.  Spikes must be bit-exact, except where the oracle's own membrane is
within the tolerance of the threshold: there both outcomes are correct.  Such a tolerated
flip changes that neuron's membrane by theta from then on, so the neuron is marked tainted
for the rest of the call and left out of later checks.  The counts are reported.
"""
from dataclasses import dataclass

import numpy as np

TOL_FP32 = 1e-5
TOL_BF16 = 2e-2


def np_pack(dense: np.ndarray) -> np.ndarray:
    """uint8 0/1 [..., W] -> int32 [..., ceil(W/32)], pixel x = bit x%32 of word x//32."""
    W = dense.shape[-1]
    Ww = (W + 31) // 32
    padded = np.zeros(dense.shape[:-1] + (Ww * 32,), dtype=np.uint8)
    padded[..., :W] = dense != 0
    by = np.packbits(padded, axis=-1, bitorder="little")
    return np.ascontiguousarray(by).view("<u4").astype(np.uint32).view(np.int32).reshape(dense.shape[:-1] + (Ww,))


def np_unpack(packed: np.ndarray, W: int) -> np.ndarray:
    """int32 [..., ceil(W/32)] -> uint8 [..., W]; also returns nothing about pad bits (see pad_bits_zero)."""
    by = np.ascontiguousarray(packed).view(np.uint8)
    bits = np.unpackbits(by, axis=-1, bitorder="little")
    return np.ascontiguousarray(bits[..., :W])


def pad_bits_zero(packed: np.ndarray, W: int) -> bool:
    by = np.ascontiguousarray(packed).view(np.uint8)
    bits = np.unpackbits(by, axis=-1, bitorder="little")
    return not bits[..., W:].any()


@dataclass
class Parity:
    max_err: float          # over untainted neurons
    flips: int              # tolerated spike differences (oracle V within tol of theta)
    mismatches: int         # untolerated spike differences
    v_violations: int       # untainted membrane values outside the tolerance
    checked: int
    tainted: int

    @property
    def ok(self) -> bool:
        return self.mismatches == 0 and self.v_violations == 0

    def short(self):
        return ("max_err=%.3g flips=%d mismatches=%d v_violations=%d tainted=%d/%d" %
                (self.max_err, self.flips, self.mismatches, self.v_violations, self.tainted, self.checked))

    def __str__(self):
        p3 = getattr(self, "p3", None)       # set by check_layer on the bf16 path
        if p3 is None:
            return self.short()
        return ("%s | vs plain oracle at 2e-2: %s | operand rounding alone (CPU): %s | beyond it: %.2g of scale, %d neurons" %
                (self.short(), p3.vs_plain.short(), p3.quant.short(), p3.excess, p3.extra_mismatches))


def compare(ref_spikes, ref_vpre, gpu_spikes, gpu_vpre, theta: float, tol: float,
            decay: float = None, v0=None, detail: bool = False):
    """All arrays are [steps, ...neurons...]; gpu_vpre may be None (spikes only).

    Error scale.  decay=None: max(|V_ref|, theta).  With `decay` (the membrane decay per LIF
    step) the scale is max(|V_ref|, theta, M) where M is the running sum of magnitudes the
    membrane was built from, M_t = decay M_{t-1} + |Y_t| (Y_t recovered from the oracle's own
    trace).  V is a decayed running sum of the Y's that the resets keep near theta, so an
    error that is relative in every Y (operand rounding) is relative to M, not to |V|.
    """
    steps = ref_spikes.shape[0]
    rs = ref_spikes.reshape(steps, -1)
    gs = gpu_spikes.reshape(steps, -1)
    rv = ref_vpre.reshape(steps, -1)
    gv = None if gpu_vpre is None else gpu_vpre.reshape(steps, -1).astype(np.float64)
    n = rs.shape[1]
    tainted = np.zeros(n, dtype=bool)
    max_err, flips, mism, vviol = 0.0, 0, 0, 0
    first = np.full(n, -1, dtype=np.int64)      # step of a neuron's first spike difference
    near_first = np.zeros(n, dtype=bool)        # ... and whether it was within the tolerance of the threshold
    post = np.zeros(n) if v0 is None else np.asarray(v0, dtype=np.float64).reshape(-1)
    M = np.abs(post)
    for s in range(steps):
        scale = np.maximum(np.abs(rv[s]), theta)
        if decay is not None:
            M = decay * M + np.abs(rv[s] - decay * post)
            post = rv[s] - theta * rs[s]
            scale = np.maximum(scale, M)
        live = ~tainted
        if gv is not None:
            err = np.abs(gv[s] - rv[s]) / scale
            if live.any():
                max_err = max(max_err, float(err[live].max()))
            vviol += int((err[live] > tol).sum())
        diff = (rs[s] != gs[s]) & live
        if diff.any():
            near = np.abs(rv[s] - theta) <= tol * scale
            flips += int((diff & near).sum())
            mism += int((diff & ~near).sum())
            tainted |= diff
            first[diff] = s
            near_first[diff] = near[diff]
    par = Parity(max_err, flips, mism, vviol, n * steps, int(tainted.sum()))
    return (par, first, near_first) if detail else par


@dataclass
class Parity3:
    """The bf16 path against both readings of the oracle.

    vs_rounded  library against the oracle run on bf16-rounded W and A_k, at `tol_same`: what is left is
                the order of the fp32 sums;
    vs_plain    library against the plain double-precision oracle at the stated 2e-2;
    quant       the rounded oracle against the plain one at 2e-2: what rounding the operands does by
                itself, on the CPU alone;
    bounded     the library adds nothing to the quantisation: every neuron whose spikes leave the plain
                oracle's does so at the step where the rounded oracle's do (or at a tolerated flip
                against the rounded oracle), and until then |V_gpu - V_plain| <= |V_rounded - V_plain|
                + tol_same * max(|V_plain|, |V_rounded|, theta).
    """
    vs_rounded: Parity
    vs_plain: Parity
    quant: Parity
    bounded: bool
    excess: float            # largest |V_gpu - V_plain| - |V_rounded - V_plain| over the scale, while comparable
    extra_mismatches: int    # neurons that leave the plain oracle although the rounded oracle does not

    def __str__(self):
        return ("vs rounded oracle [%s] | vs plain oracle at 2e-2 [%s] | rounding alone, on the CPU [%s] | "
                "beyond the rounding: %.2g of scale, %d neurons" %
                (self.vs_rounded.short(), self.vs_plain.short(), self.quant.short(), self.excess, self.extra_mismatches))


def compare3(plain, rounded, gpu_spikes, gpu_vpre, theta: float, tol_same: float, tol_plain: float = TOL_BF16) -> Parity3:
    """plain, rounded: (spikes, v_pre) of the two oracle runs; gpu_vpre may be None (spikes only)."""
    steps = plain[0].shape[0]
    vs_r, first_r, _ = compare(rounded[0], rounded[1], gpu_spikes, gpu_vpre, theta, tol_same, detail=True)
    vs_p, first_p, _ = compare(plain[0], plain[1], gpu_spikes, gpu_vpre, theta, tol_plain, detail=True)
    quant, first_q, _ = compare(plain[0], plain[1], rounded[0], rounded[1], theta, tol_plain, detail=True)
    # a neuron may leave the plain oracle's spike train only where the rounded oracle leaves it, or where
    # the library differs from the rounded oracle (a flip tolerated above, or an error counted above)
    left = first_p >= 0
    explained = (first_q == first_p) | ((first_r >= 0) & (first_r <= np.where(left, first_p, steps)))
    extra = int((left & ~explained).sum())
    excess = 0.0
    if gpu_vpre is not None:
        pv = plain[1].reshape(steps, -1)
        qv = rounded[1].reshape(steps, -1)
        gv = gpu_vpre.reshape(steps, -1).astype(np.float64)
        sidx = np.arange(steps)[:, None]
        # comparable: before the neuron's first difference in any of the three comparisons
        lim = np.minimum.reduce([np.where(f >= 0, f, steps) for f in (first_r, first_p, first_q)])
        live = sidx <= lim[None, :]
        scale = np.maximum(np.maximum(np.abs(pv), np.abs(qv)), theta)
        over = (np.abs(gv - pv) - np.abs(qv - pv)) / scale
        excess = float(over[live].max()) if live.any() else 0.0
    return Parity3(vs_r, vs_p, quant, extra == 0 and excess <= tol_same, excess, extra)
