"""Seeded synthetic workloads shaped like the paper's serving scenarios.

This module only draws inputs (sequence lengths, hidden states, LM-head and prediction-head
weights) and rounds them to their storage type.  It contains none of the method's
arithmetic -- no entropy, no pooling, no prefix sums -- and imports neither the GPU binding
nor the CPU oracle, so that both can consume exactly the same bits.

Real activations, tokenisers and datasets are not available here; ragged long-tailed
length draws and Gaussian activations with the hidden / vocabulary sizes of the model
families the paper evaluates stand in for them.

All draws use ``numpy.random.default_rng`` (PCG64) in a fixed order:
lengths -> hidden Gaussian -> per-token scale -> W_lm -> W1 -> w2.
Values are generated in fp32 and, for bf16 workloads, rounded once (round-to-nearest-even)
to bf16 bit patterns stored as ``uint16``.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Dict, Optional

import numpy as np


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (nearest even); returns the 16-bit patterns as uint16."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + r) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns to fp32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


@dataclass(frozen=True)
class Spec:
    """Shape of one workload. ``lengths`` fixes the lengths; otherwise they are drawn."""
    name: str
    seed: int
    B: int
    d: int
    V: int
    d_h: int
    dtype: str                      # "f32" or "bf16"
    lengths: Optional[tuple] = None
    len_dist: str = "lognormal"     # "lognormal" | "uniform"
    len_mu: float = 0.0
    len_sigma: float = 0.0
    len_lo: int = 1
    len_hi: int = 1
    token_scale: Optional[tuple] = None   # per-token scale ~ U(lo, hi); None = 1


# The five workloads.  C3 is the one throughput is quoted on.
SPECS: Dict[str, Spec] = {
    "tiny": Spec("tiny", seed=0, B=4, d=256, V=4096, d_h=128, dtype="f32",
                 lengths=(17, 64, 100, 128)),
    "mid": Spec("mid", seed=1, B=32, d=2048, V=32000, d_h=512, dtype="bf16",
                len_mu=5.5, len_sigma=0.8, len_lo=16, len_hi=2048, token_scale=(0.5, 2.0)),
    "serving": Spec("serving", seed=2, B=128, d=4096, V=151936, d_h=1024, dtype="bf16",
                    len_mu=6.5, len_sigma=1.0, len_lo=32, len_hi=8192, token_scale=(0.5, 2.0)),
    # one new token per sequence per step; lengths are all 1
    "plp_decode": Spec("plp_decode", seed=3, B=512, d=4096, V=151936, d_h=1024, dtype="bf16",
                       lengths=tuple([1] * 512), token_scale=(0.5, 2.0)),
    # prompts of the one-to-many sampling scenario; continuations come from rl_continuations()
    "rl_prompts": Spec("rl_prompts", seed=4, B=64, d=5120, V=151936, d_h=1280, dtype="bf16",
                       len_dist="uniform", len_lo=128, len_hi=1024, token_scale=(0.5, 2.0)),
}


@dataclass
class Workload:
    spec: Spec
    lengths: np.ndarray            # [B] int32
    hidden: np.ndarray             # [T x d] fp32, or uint16 bf16 bits
    w_lm: np.ndarray               # [V x d] same storage type
    w1: np.ndarray                 # [d_h x d]
    w2: np.ndarray                 # [1 x d_h]
    extras: dict = field(default_factory=dict)

    @property
    def T(self) -> int:
        return int(self.hidden.shape[0])


def scaled(spec: Spec, **kw) -> Spec:
    """A copy of ``spec`` with some sizes replaced (parity tests use reduced sizes)."""
    return replace(spec, **kw)


def draw_lengths(spec: Spec, rng: np.random.Generator) -> np.ndarray:
    if spec.lengths is not None:
        assert len(spec.lengths) == spec.B
        return np.asarray(spec.lengths, dtype=np.int32)
    if spec.len_dist == "uniform":
        return rng.integers(spec.len_lo, spec.len_hi + 1, size=spec.B).astype(np.int32)
    raw = np.exp(rng.normal(spec.len_mu, spec.len_sigma, size=spec.B))
    return np.clip(np.rint(raw), spec.len_lo, spec.len_hi).astype(np.int32)


def _store(x: np.ndarray, dtype: str) -> np.ndarray:
    return to_bf16_bits(x) if dtype == "bf16" else np.ascontiguousarray(x, dtype=np.float32)


def _gauss_rows(rng, rows: int, cols: int, std: float, dtype: str, row_scale=None,
                chunk_rows: int = 8192) -> np.ndarray:
    """rows x cols of N(0, std^2), optionally scaled per row, stored as ``dtype``.
    Drawn in row chunks to bound peak memory; the stream is the same as one big draw."""
    out = np.empty((rows, cols), dtype=np.uint16 if dtype == "bf16" else np.float32)
    for r0 in range(0, rows, chunk_rows):
        r1 = min(rows, r0 + chunk_rows)
        g = rng.standard_normal((r1 - r0, cols), dtype=np.float32)
        if std != 1.0:
            g *= np.float32(std)
        if row_scale is not None:
            g *= row_scale[r0:r1, None]
        out[r0:r1] = _store(g, dtype)
    return out


def draw_hidden(spec: Spec, rng: np.random.Generator, T: int) -> np.ndarray:
    """T hidden states: unit Gaussians, times a per-token scale when the spec has one.
    The Gaussians are drawn first, then the scales (fixed order of draws)."""
    g = rng.standard_normal((T, spec.d), dtype=np.float32)
    if spec.token_scale is not None:
        lo, hi = spec.token_scale
        s = rng.uniform(lo, hi, size=T).astype(np.float32)
        g *= s[:, None]
    return _store(g, spec.dtype)


def make(spec: Spec) -> Workload:
    rng = np.random.default_rng(spec.seed)
    lengths = draw_lengths(spec, rng)
    T = int(lengths.sum())
    hidden = draw_hidden(spec, rng, T)
    w_lm = _gauss_rows(rng, spec.V, spec.d, 1.0 / np.sqrt(spec.d), spec.dtype)
    w1 = _gauss_rows(rng, spec.d_h, spec.d, 1.0 / np.sqrt(spec.d), spec.dtype)
    w2 = _gauss_rows(rng, 1, spec.d_h, 1.0 / np.sqrt(spec.d_h), spec.dtype)
    return Workload(spec, lengths, hidden, w_lm, w1, w2)


def decode_hidden(spec: Spec, step: int, rows: Optional[int] = None) -> np.ndarray:
    """Fresh hidden states for decode step ``step`` (1-based): [rows x d], seeded by
    (spec.seed, step) so that any step can be regenerated on its own."""
    rng = np.random.default_rng([spec.seed, step])
    return draw_hidden(spec, rng, spec.B if rows is None else rows)


def rl_continuations(spec: Spec, samples_per_prompt: int = 16, mu: float = 7.0,
                     sigma: float = 1.2, lo: int = 1, hi: int = 16384) -> np.ndarray:
    """Continuation lengths of the one-to-many sampling scenario:
    [B * samples_per_prompt] int32, log-normal, clipped."""
    rng = np.random.default_rng([spec.seed, 1 << 20])
    raw = np.exp(rng.normal(mu, sigma, size=spec.B * samples_per_prompt))
    return np.clip(np.rint(raw), lo, hi).astype(np.int32)


# --------------------------------------------------------------------------- head training data
@dataclass
class TrainSet:
    """Synthetic (feature, length) pairs and an initial K-bin head, all fp32.

    Stands in for pooled vectors of a frozen model paired with observed generation lengths:
    features are Gaussian, the length is log-normal around a fixed random direction of the
    feature plus noise (long-tailed, clipped to [1, max_len]).  Bins are ``K`` equal-width
    intervals of [0, max_len] with their midpoints as centres -- the paper leaves the bin edges
    open, so the binning is part of the input recipe, not of the method.
    """
    x: np.ndarray          # [B x d] fp32
    y: np.ndarray          # [B] fp32 target length (remaining length for PLP samples)
    bins: np.ndarray       # [B] int32
    centers: np.ndarray    # [K] fp32
    w1: np.ndarray         # [d_h x d]
    b1: np.ndarray         # [d_h]
    w2: np.ndarray         # [K x d_h]
    b2: np.ndarray         # [K]
    steps: Optional[np.ndarray] = None   # [B] int32: decode steps of the sample's sequence (PLP)
    n_seqs: int = 0


def make_train(seed: int, B: int, d: int, d_h: int, K: int, max_len: float = 2048.0,
               plp_seqs: int = 0) -> TrainSet:
    """Draw order: direction -> features -> noise -> W1 -> b1 -> W2 -> b2 [-> steps per sequence].

    plp_seqs > 0: the B samples are decode steps of ``plp_seqs`` sequences (every sequence gets
    at least one, the rest are dealt at random); ``steps[b]`` is how many its sequence holds."""
    rng = np.random.default_rng([seed, 1 << 21])
    u = rng.standard_normal(d).astype(np.float32) / np.float32(np.sqrt(d))
    x = rng.standard_normal((B, d)).astype(np.float32)
    noise = rng.standard_normal(B).astype(np.float32)
    y = np.exp(np.float32(5.5) + np.float32(0.8) * (x @ u) + np.float32(0.3) * noise)
    y = np.clip(y, 1.0, max_len - 1.0).astype(np.float32)
    width = np.float32(max_len / K)
    bins = np.minimum((y / width).astype(np.int32), K - 1).astype(np.int32)
    centers = ((np.arange(K, dtype=np.float32) + np.float32(0.5)) * width).astype(np.float32)
    w1 = (rng.standard_normal((d_h, d)) / np.sqrt(d)).astype(np.float32)
    b1 = (0.1 * rng.standard_normal(d_h)).astype(np.float32)
    w2 = (rng.standard_normal((K, d_h)) / np.sqrt(d_h)).astype(np.float32)
    b2 = (0.1 * rng.standard_normal(K)).astype(np.float32)
    ts = TrainSet(x, y, bins, centers, w1, b1, w2, b2)
    if plp_seqs > 0:
        assert plp_seqs <= B
        owner = np.concatenate([np.arange(plp_seqs), rng.integers(0, plp_seqs, size=B - plp_seqs)])
        owner = rng.permutation(owner)
        counts = np.bincount(owner, minlength=plp_seqs)
        ts.steps = counts[owner].astype(np.int32)
        ts.n_seqs = plp_seqs
    return ts
