"""Seeded synthetic inputs shaped like the hidden states ToMA runs on.

This module holds no arithmetic of the method: it only draws tensors.  Both the HIP path and the
CPU oracle are fed from it, so that they see the same values.  The workloads stand in for SDXL-base
and Flux.1-dev layers (paper Sec. 5.1 and the layer sizes of its FLOP table, App. G): a spatially
smooth random field per channel (neighbouring tokens resemble each other, the locality Sec. 4.3.1
relies on) plus white noise.
"""
from dataclasses import dataclass, replace

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    index: int          # seeds are index*1000 + tensor id (the tiny workload uses seed 0)
    dtype: str          # "f32" or "bf16"
    B: int
    H: int
    W: int
    C: int
    tile_h: int
    tile_w: int
    keep: float         # fraction of tokens kept as destinations
    heads: int
    T_extra: int        # unmerged extra (text) tokens that join the attention
    sigma: float        # blur width in tokens
    noise: float        # std of the added white noise
    tau: float = 0.1
    steps: int = 1      # > 1: a denoising-like sequence X_t = X_{t-1} + drift * N(0,1)
    drift: float = 0.0
    reselect_every: int = 1
    reweight_every: int = 1

    @property
    def N(self):
        return self.H * self.W

    @property
    def P(self):
        return (self.H // self.tile_h) * (self.W // self.tile_w)

    @property
    def n_loc(self):
        return self.tile_h * self.tile_w

    @property
    def d_loc(self):
        return int(round(self.keep * self.n_loc))

    @property
    def D(self):
        return self.P * self.d_loc

    @property
    def head_dim(self):
        return self.C // self.heads


WORKLOADS = {
    "tiny": Workload("tiny", 0, "f32", 1, 16, 16, 64, 8, 8, 0.5, 1, 0, 1.5, 0.1),
    "sdxl1": Workload("sdxl1", 1, "bf16", 2, 64, 64, 640, 16, 16, 0.5, 10, 0, 2.0, 0.2),
    "sdxl2": Workload("sdxl2", 2, "bf16", 2, 32, 32, 1280, 8, 8, 0.5, 20, 0, 1.5, 0.2),
    "flux": Workload("flux", 3, "bf16", 1, 64, 64, 3072, 16, 16, 0.25, 24, 512, 2.0, 0.0),
    "hires": Workload("hires", 4, "bf16", 2, 128, 128, 640, 16, 16, 0.5, 10, 0, 3.0, 0.0,
                      steps=10, drift=0.02, reselect_every=5, reweight_every=2),
    # the SDXL stage-1 shape with stripe-shaped regions (Sec. 4.3.1: contiguous rows, four grid rows
    # = 256 tokens per region): same inputs as "sdxl1", only the region map differs
    "sdxl1_stripe": Workload("sdxl1_stripe", 1, "bf16", 2, 64, 64, 640, 4, 64, 0.5, 10, 0, 2.0, 0.2),
    # the SDXL stage-1 shape with four regions of 1024 tokens per sample: the few-regions end of the
    # region-count ablation (Sec. 4.3.1; more regions are cheaper, fewer select more globally)
    "sdxl1_4regions": Workload("sdxl1_4regions", 1, "bf16", 2, 64, 64, 640, 32, 32, 0.5, 10, 0, 2.0, 0.2),
}


def scaled(w, **kw):
    """A smaller or altered copy of a workload (used by tests)."""
    return replace(w, **kw)


def _seed(w, tensor_id):
    return 0 + tensor_id if w.index == 0 else w.index * 1000 + tensor_id


def _rng(w, tensor_id):
    return np.random.Generator(np.random.PCG64(_seed(w, tensor_id)))


def gaussian_kernel(sigma):
    r = int(np.ceil(4.0 * sigma))
    x = np.arange(-r, r + 1, dtype=np.float64)
    k = np.exp(-0.5 * (x / sigma) ** 2)
    return k / k.sum()


def _blur_axis(a, k, axis):
    r = (len(k) - 1) // 2
    pad = [(0, 0)] * a.ndim
    pad[axis] = (r, r)
    n = a.shape[axis]
    if r >= n:  # reflect padding needs r < n; fall back to repeated reflection
        ap = np.pad(a, pad, mode="symmetric")
    else:
        ap = np.pad(a, pad, mode="reflect")
    out = np.zeros_like(a)
    for t in range(len(k)):
        sl = [slice(None)] * a.ndim
        sl[axis] = slice(t, t + n)
        out += k[t] * ap[tuple(sl)]
    return out


def smooth_field(rng, B, H, W, C, sigma, noise):
    """[B, H*W, C] float32: blurred N(0,1) field rescaled to unit marginal variance, plus noise."""
    z = rng.standard_normal((B, H, W, C), dtype=np.float32)
    if sigma > 0:
        k = gaussian_kernel(sigma).astype(np.float32)
        z = _blur_axis(_blur_axis(z, k, 1), k, 2)
        z /= np.float32(np.sum(gaussian_kernel(sigma) ** 2))
    if noise > 0:
        z = z + np.float32(noise) * rng.standard_normal((B, H, W, C), dtype=np.float32)
    return np.ascontiguousarray(z.reshape(B, H * W, C), dtype=np.float32)


def round_to_bf16(x):
    """float32 -> nearest-even bf16, returned as float32 values."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) & np.uint32(0xFFFF0000)).view(np.float32)


def bf16_bits(x):
    """float32 values that are exactly representable in bf16 -> their uint16 bit patterns."""
    return (np.ascontiguousarray(x, dtype=np.float32).view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def bits_to_f32(u16):
    return (np.ascontiguousarray(u16, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def quantize(w, x):
    """Round to the workload's element type; the result (float32 array) is what BOTH sides read."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    return round_to_bf16(x) if w.dtype == "bf16" else x


def make_inputs(w):
    """Dict of float32 arrays already rounded to the workload's dtype:
    X [B,N,C] (or a list X_steps for sequences), X_extra [B,T,C] or None, Wq/Wk/Wv [C,C]."""
    out = {}
    X0 = smooth_field(_rng(w, 1), w.B, w.H, w.W, w.C, w.sigma, w.noise)
    if w.steps > 1:
        rng = _rng(w, 6)
        seq = [X0]
        for _ in range(1, w.steps):
            seq.append(seq[-1] + np.float32(w.drift) * rng.standard_normal(X0.shape, dtype=np.float32))
        out["X_steps"] = [quantize(w, x) for x in seq]
        out["X"] = out["X_steps"][0]
    else:
        out["X"] = quantize(w, X0)
    if w.T_extra > 0:
        out["X_extra"] = quantize(w, _rng(w, 2).standard_normal((w.B, w.T_extra, w.C), dtype=np.float32))
    else:
        out["X_extra"] = None
    std = np.float32(1.0 / np.sqrt(w.C))
    for i, name in enumerate(("Wq", "Wk", "Wv")):
        out[name] = quantize(w, std * _rng(w, 3 + i).standard_normal((w.C, w.C), dtype=np.float32))
    return out


def reuse_schedule(w):
    """Per step: (reselect, reweight).  Destinations are re-selected every reselect_every steps;
    the merge weights are recomputed when (t - t_last_select) % reweight_every == 0."""
    plan = []
    last = 0
    for t in range(w.steps):
        sel = (t % w.reselect_every == 0)
        if sel:
            last = t
        plan.append((sel, sel or ((t - last) % w.reweight_every == 0)))
    return plan
