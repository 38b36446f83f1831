"""Seeded synthetic workloads shaped like the paper's Wan2.1-1.3B attention layers.

This module only draws random inputs and names shapes.  It contains none of the method's
arithmetic and is the one module that both the CPU oracle's tests and the GPU path's callers
use, so that both sides see bit-identical inputs.

The paper evaluates on Wan2.1 1.3B at 81 x 480 x 832 (Sec. 4, "Evaluation"): 12 heads of width
128 and 21 x 30 x 52 = 32760 latent tokens per clip.  Real activations and trained feature maps
are not available, so q, k, v are iid normal scaled by d^-1/2 and the feature-map weights are
N(0, 1/fan_in) with N(0, 0.1^2) biases; only the shapes follow the paper.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    H: int
    N: int
    d: int
    dtype: str            # "bf16" or "f32": io dtype of q, k, v, out and the MLP weights
    block_size: int
    R: int                # integer hybrid rate; r = 1/R, R = 0 means r = 0 (pure linear)
    d_hidden: int
    d_feat: int
    poly_degree: int = 2
    seed: int = 0
    grid: tuple = ()      # (frames, rows, cols) of the latent grid, metadata only
    qk_gain: float = 1.0  # stress sets multiply q and k by this
    w_gain: float = 1.0   # stress sets multiply the MLP weights by this
    d_mid: int = 0        # width of the second hidden layer of a three-layer feature map (0: two layers)
    split_granularity: int = 0   # > 1: the block-granular variant of the split (groups of this many tokens)
    causal_chunk: int = 0        # > 0: the chunk-causal variant (chunks of this many tokens)
    local_window: int = 0        # > 0: the local-window variant (tokens on either side of the query's tile; R = 0)

    @property
    def rate(self):
        """What the binding takes as hybrid_rate: R, or (R, group size[, causal chunk]) for the variants."""
        if self.local_window > 0:
            return (0, 0, 0, self.local_window)
        if self.causal_chunk > 0:
            return (self.R, self.split_granularity, self.causal_chunk)
        return (self.R, self.split_granularity) if self.split_granularity > 1 else self.R

    def softmax_before(self, t):
        """Number of softmax tokens among the first t tokens."""
        if self.R == 0:
            return 0
        g = max(self.split_granularity, 1)
        return (t // (self.R * g)) * g + min(t % (self.R * g), g)

    @property
    def n_softmax(self):
        if self.R == 0:
            return 0
        g = max(self.split_granularity, 1)
        return (self.N // (self.R * g)) * g + min(self.N % (self.R * g), g)

    @property
    def n_linear(self):
        return self.N - self.n_softmax

    @property
    def scale(self):
        return 1.0 / float(np.sqrt(self.d))


# The five benchmark configurations (tokens laid out frame-major over frames x rows x cols).
TINY = Workload("tiny", 1, 2, 1024, 64, "f32", 64, 4, 64, 64, grid=(4, 16, 16))
WAN_480P_81F = Workload("wan1.3b_480p_81f", 1, 12, 32760, 128, "bf16", 128, 4, 128, 128, grid=(21, 30, 52))
WAN_480P_161F = Workload("wan1.3b_480p_161f", 1, 12, 63960, 128, "bf16", 128, 8, 128, 128, grid=(41, 30, 52))
WAN_720P_81F_CFG = Workload("wan1.3b_720p_81f_cfg2", 2, 12, 75600, 128, "bf16", 128, 4, 128, 128, grid=(21, 45, 80))
RATE_SWEEP = (0, 8, 4, 2, 1)
STACK_RATES = (16, 8, 4)          # per-layer rates of the 30-layer stack cycle through these
STACK_LAYERS = 30


def with_rate(w: Workload, R: int) -> Workload:
    return Workload(**{**w.__dict__, "R": R})


def replace(w: Workload, **kw) -> Workload:
    return Workload(**{**w.__dict__, **kw})


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16 (ties to even); result stays float32."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = ((u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)) << np.uint32(16)
    return r.view(np.float32)


@dataclass
class FeatureMapParams:
    w1: np.ndarray   # [H, Hd, d]  float32 (bf16-exact when the io dtype is bf16)
    b1: np.ndarray   # [H, Hd]     float32
    w2: np.ndarray   # [H, F, Hd]
    b2: np.ndarray   # [H, F]
    poly_degree: int
    w_mid: Optional[np.ndarray] = None   # [H, Dm, Hd]: three-layer map (then w2 is [H, F, Dm])
    b_mid: Optional[np.ndarray] = None   # [H, Dm]


@dataclass
class Inputs:
    q: np.ndarray    # [B, H, N, d] float32
    k: np.ndarray
    v: np.ndarray
    phi_q: FeatureMapParams
    phi_k: FeatureMapParams
    workload: Workload = field(repr=False, default=None)


def _draw_map(rng, H, d, Hd, F, P, io_round, w_gain, Dm=0):
    w1 = rng.standard_normal((H, Hd, d), dtype=np.float32) * np.float32(w_gain / np.sqrt(d))
    b1 = rng.standard_normal((H, Hd), dtype=np.float32) * np.float32(0.1)
    kl = Dm if Dm > 0 else Hd
    w2 = rng.standard_normal((H, F, kl), dtype=np.float32) * np.float32(w_gain / np.sqrt(kl))
    b2 = rng.standard_normal((H, F), dtype=np.float32) * np.float32(0.1)
    if Dm > 0:
        w_mid = rng.standard_normal((H, Dm, Hd), dtype=np.float32) * np.float32(w_gain / np.sqrt(Hd))
        b_mid = rng.standard_normal((H, Dm), dtype=np.float32) * np.float32(0.1)
        return FeatureMapParams(io_round(w1), b1, io_round(w2), b2, P, io_round(w_mid), b_mid)
    return FeatureMapParams(io_round(w1), b1, io_round(w2), b2, P)


def make_inputs(w: Workload, heads: Optional[int] = None) -> Inputs:
    """Draw q, k, v, phi_q, phi_k for a workload from one numpy Generator stream (seed = w.seed),
    in that order.  `heads` optionally truncates H (for bounded CPU samples)."""
    H = w.H if heads is None else heads
    rng = np.random.default_rng(w.seed)
    io_round = round_to_bf16 if w.dtype == "bf16" else (lambda a: np.ascontiguousarray(a, dtype=np.float32))
    s = np.float32(w.qk_gain / np.sqrt(w.d))
    shape = (w.B, H, w.N, w.d)
    q = io_round(rng.standard_normal(shape, dtype=np.float32) * s)
    k = io_round(rng.standard_normal(shape, dtype=np.float32) * s)
    v = io_round(rng.standard_normal(shape, dtype=np.float32) * np.float32(1.0 / np.sqrt(w.d)))
    phi_q = _draw_map(rng, H, w.d, w.d_hidden, w.d_feat, w.poly_degree, io_round, w.w_gain, w.d_mid)
    phi_k = _draw_map(rng, H, w.d, w.d_hidden, w.d_feat, w.poly_degree, io_round, w.w_gain, w.d_mid)
    return Inputs(q, k, v, phi_q, phi_k, replace(w, H=H))


def make_inputs_on_device(w: Workload, device="cuda"):
    """The same distributions drawn on the device with a seeded torch.Generator (seed = w.seed), for workloads too
    large to draw on the host (the 720p stack: 1.9 GB per layer): q, k, v in the io dtype, then the tensors of phi_q
    and of phi_k as dicts (w1, b1, w2, b2[, w_mid, b_mid]), in that order from one generator.  Benchmarks and parity
    tests both call this, so both see the same tensors."""
    import torch
    dt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    gen = torch.Generator(device=device).manual_seed(w.seed)
    s = w.qk_gain * w.d ** -0.5
    q, k = ((torch.randn(w.B, w.H, w.N, w.d, generator=gen, device=device, dtype=torch.float32) * s).to(dt) for _ in range(2))
    v = (torch.randn(w.B, w.H, w.N, w.d, generator=gen, device=device, dtype=torch.float32) * w.d ** -0.5).to(dt)

    def draw_map():
        kl = w.d_mid if w.d_mid else w.d_hidden
        m = dict(w1=(torch.randn(w.H, w.d_hidden, w.d, generator=gen, device=device) * (w.w_gain * w.d ** -0.5)).to(dt),
                 b1=torch.randn(w.H, w.d_hidden, generator=gen, device=device) * 0.1,
                 w2=(torch.randn(w.H, w.d_feat, kl, generator=gen, device=device) * (w.w_gain * kl ** -0.5)).to(dt),
                 b2=torch.randn(w.H, w.d_feat, generator=gen, device=device) * 0.1)
        if w.d_mid:
            m["w_mid"] = (torch.randn(w.H, w.d_mid, w.d_hidden, generator=gen, device=device) * (w.w_gain * w.d_hidden ** -0.5)).to(dt)
            m["b_mid"] = torch.randn(w.H, w.d_mid, generator=gen, device=device) * 0.1
        return m
    return q, k, v, draw_map(), draw_map()


def sample_rows(w: Workload, n_random: int = 256, seed: int = 12345) -> np.ndarray:
    """Query rows for sampled parity at sizes the oracle cannot cover in full: the first tile,
    the ragged tail tile, both sides of every 16th tile boundary, and n_random random rows."""
    bs = max(w.block_size, 1)
    rows = set(range(min(bs, w.N)))
    rows.update(range(max(0, w.N - bs), w.N))
    for t in range(16 * bs, w.N, 16 * bs):
        rows.update((t - 1, t))
    rng = np.random.default_rng(seed)
    rows.update(int(i) for i in rng.integers(0, w.N, size=n_random))
    return np.array(sorted(rows), dtype=np.int64)


def softmax_pairs(w: Workload) -> float:
    """Number of (query, softmax key) pairs per (batch, head): N N_S for the paper's operator, fewer for the variants."""
    N = w.N
    if w.local_window > 0:
        T = 2 * w.block_size
        wt = w.local_window // T
        return float(sum((min(lo + T, N) - lo) * (min((lo // T + wt + 1) * T, N) - max(lo // T - wt, 0) * T) for lo in range(0, N, T)))
    if 0 < w.causal_chunk < N:
        C = w.causal_chunk
        return float(sum((min(lo + C, N) - lo) * w.softmax_before(min(lo + C, N)) for lo in range(0, N, C)))
    return float(N) * w.n_softmax


def algorithmic_flops(w: Workload) -> float:
    """FLOPs the method itself needs for one forward: the two GEMMs of the softmax part, both
    feature-map MLPs (phi_k on linear keys only), the state, and its contraction with phi_q(q).
    exp, max, powers and the division are not counted; with no linear keys phi is skipped."""
    n_s, n_l, N, d, Hd, F = w.n_softmax, w.n_linear, w.N, w.d, w.d_hidden, w.d_feat
    per_head = 4.0 * N * n_s * d
    per_head = 4.0 * d * softmax_pairs(w)
    if w.local_window > 0:           # local-window variant: every token is a linear key of the tiles that do not see it
        n_l = N
    if n_l > 0:
        mlp = d * Hd + (Hd * w.d_mid + w.d_mid * F if w.d_mid else Hd * F)       # multiply-adds per token
        per_head += 2.0 * (N + n_l) * mlp
        per_head += 2.0 * n_l * F * d + n_l * F
        per_head += 2.0 * N * F * d + 2.0 * N * F
    return w.B * w.H * per_head


def algorithmic_bytes(w: Workload) -> float:
    """Compulsory HBM bytes of one forward: q, k, v read once and out written once in the io
    dtype, the MLP weights, and the state S, z written and read once."""
    io = 2 if w.dtype == "bf16" else 4
    qkvo = 4.0 * w.B * w.H * w.N * w.d * io
    weights = 2.0 * w.H * (w.d * w.d_hidden + w.d_hidden * w.d_feat) * io
    state = w.B * w.H * (w.d_feat * w.d + w.d_feat) * 4.0
    return qkvo + weights + state
