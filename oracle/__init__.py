"""fp64 CPU oracle for EGTP / PLP -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.

Thin ctypes access to ``egtp_oracle.c`` (plain C, fp64, the paper's equations written
out) plus the two compositions that the paper defines on top of them:

* ``egtp``  -- Eq. 2 (token entropy) -> Eq. 3 (entropy softmax weights) -> Eq. 4 (weighted
  pooling) -> Section 3.2 prediction head.
* ``plp``   -- Eq. 8: at decode step t the same pipeline applied to the prompt tokens
  followed by generated tokens 1..t of each sequence.  No running state is kept: every step
  recomputes from the stored history, so a streaming implementation is checked against the
  non-streaming definition.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this module.
It imports nothing from the GPU package.

Array conventions: ``float32`` arrays are fp32 data, ``uint16`` arrays are bf16 bit
patterns, ``float64`` arrays are fp64 data.  Everything returned is fp64 (or int32).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "egtp_oracle.c")
_LIB = os.path.join(_HERE, "libegtp_oracle.so")

F32, BF16, F64 = 0, 1, 2


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (OpenMP over tokens only). Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        # -ffp-contract=off: no fused multiply-adds, every product and sum is rounded as written
        cmd = ["gcc", "-O2", "-std=c99", "-fopenmp", "-ffp-contract=off", "-fPIC", "-shared",
               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        i32, i64, dbl, vp = ctypes.c_int32, ctypes.c_int64, ctypes.c_double, ctypes.c_void_p
        ci = ctypes.c_int
        _lib.oracle_offsets.argtypes = [vp, i32, vp]
        _lib.oracle_seg_ids.argtypes = [vp, i32, i64, vp]
        _lib.oracle_entropy_from_logits.argtypes = [vp, i64, i32, vp]
        _lib.oracle_logits.argtypes = [vp, vp, ci, i32, i32, vp]
        _lib.oracle_entropy.argtypes = [vp, vp, ci, i64, i32, i32, vp]
        _lib.oracle_pool.argtypes = [vp, ci, i32, vp, vp, i32, dbl, vp, vp, vp]
        _lib.oracle_pool_ablation.argtypes = [vp, ci, i32, vp, i32, ci, vp]
        _lib.oracle_head.argtypes = [vp, i32, i32, i32, i32, vp, vp, vp, vp, ci, vp]
        _lib.oracle_bin_decode.argtypes = [vp, i32, i32, vp, vp, vp]
        _lib.oracle_soft_label.argtypes = [i32, i32, vp]
        _lib.oracle_head_loss_grad.argtypes = [vp, vp, vp, vp, i32, i32, i32, i32, vp, vp, vp, vp, vp, dbl,
                                               vp, vp, vp, vp, vp]
        _lib.oracle_adamw.argtypes = [vp, vp, vp, vp, i64, dbl, dbl, dbl, dbl, dbl, i64]
        for name in ("oracle_offsets", "oracle_seg_ids", "oracle_entropy_from_logits",
                     "oracle_logits", "oracle_entropy", "oracle_pool", "oracle_pool_ablation",
                     "oracle_head", "oracle_bin_decode", "oracle_soft_label", "oracle_head_loss_grad",
                     "oracle_adamw"):
            getattr(_lib, name).restype = ci
    return _lib


def _dtype_code(a: np.ndarray) -> int:
    if a.dtype == np.float32:
        return F32
    if a.dtype == np.uint16:
        return BF16
    if a.dtype == np.float64:
        return F64
    raise TypeError(f"unsupported storage dtype {a.dtype}")


def _c(a: np.ndarray) -> np.ndarray:
    return np.ascontiguousarray(a)


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _check(rc: int, what: str):
    if rc != 0:
        raise ValueError(f"oracle {what}: error {rc}")


def num_threads() -> int:
    """Threads the OpenMP loops will use (OMP_NUM_THREADS, else the visible cores)."""
    env = os.environ.get("OMP_NUM_THREADS", "")
    if env.isdigit() and int(env) > 0:
        return int(env)
    try:
        return len(os.sched_getaffinity(0))
    except AttributeError:
        return os.cpu_count() or 1


# --------------------------------------------------------------------------- plumbing
def offsets_from_lengths(lengths) -> np.ndarray:
    lengths = _c(np.asarray(lengths, dtype=np.int32))
    out = np.zeros(lengths.size + 1, dtype=np.int32)
    _check(_load().oracle_offsets(_p(lengths), lengths.size, _p(out)), "offsets")
    return out


def seg_ids(offsets, T: int) -> np.ndarray:
    offsets = _c(np.asarray(offsets, dtype=np.int32))
    out = np.zeros(T, dtype=np.int32)
    _check(_load().oracle_seg_ids(_p(offsets), offsets.size - 1, T, _p(out)), "seg_ids")
    return out


# --------------------------------------------------------------------------- Eq. 2
def entropy_from_logits(z) -> np.ndarray:
    z = _c(np.asarray(z, dtype=np.float64))
    if z.ndim == 1:
        z = z[None, :]
    H = np.zeros(z.shape[0], dtype=np.float64)
    _check(_load().oracle_entropy_from_logits(_p(z), z.shape[0], z.shape[1], _p(H)), "entropy")
    return H


def logits(hidden_row: np.ndarray, w_lm: np.ndarray) -> np.ndarray:
    hidden_row, w_lm = _c(hidden_row), _c(w_lm)
    V, d = w_lm.shape
    assert hidden_row.shape == (d,) and hidden_row.dtype == w_lm.dtype
    z = np.zeros(V, dtype=np.float64)
    _check(_load().oracle_logits(_p(hidden_row), _p(w_lm), _dtype_code(w_lm), d, V, _p(z)),
           "logits")
    return z


def entropy(hidden: np.ndarray, w_lm: np.ndarray) -> np.ndarray:
    """H[t] of Eq. 2 for every row of hidden[T x d] under the LM head w_lm[V x d]."""
    hidden, w_lm = _c(hidden), _c(w_lm)
    V, d = w_lm.shape
    assert hidden.ndim == 2 and hidden.shape[1] == d and hidden.dtype == w_lm.dtype
    T = hidden.shape[0]
    H = np.zeros(T, dtype=np.float64)
    _check(_load().oracle_entropy(_p(hidden), _p(w_lm), _dtype_code(w_lm), T, d, V, _p(H)),
           "entropy")
    return H


# --------------------------------------------------------------------------- Eq. 3, 4
def pool(hidden: np.ndarray, H, offsets, alpha: float = 1.0):
    """Returns (weights[T], pooled[B x d], lse[B]) of Eq. 3-4 over ragged offsets."""
    hidden = _c(hidden)
    H = _c(np.asarray(H, dtype=np.float64))
    offsets = _c(np.asarray(offsets, dtype=np.int32))
    T, d = hidden.shape
    B = offsets.size - 1
    assert H.shape == (T,) and offsets[-1] == T
    w = np.zeros(T, dtype=np.float64)
    pooled = np.zeros((B, d), dtype=np.float64)
    lse = np.zeros(B, dtype=np.float64)
    _check(_load().oracle_pool(_p(hidden), _dtype_code(hidden), d, _p(H), _p(offsets), B,
                               float(alpha), _p(w), _p(pooled), _p(lse)), "pool")
    return w, pooled, lse


POOL_AVERAGE, POOL_MAX, POOL_LAST = 0, 1, 2


def pool_ablation(hidden: np.ndarray, offsets, kind: int) -> np.ndarray:
    """Average / max / last-token pooling (the ablation's alternatives) over ragged offsets."""
    hidden = _c(hidden)
    offsets = _c(np.asarray(offsets, dtype=np.int32))
    T, d = hidden.shape
    B = offsets.size - 1
    assert offsets[-1] == T
    pooled = np.zeros((B, d), dtype=np.float64)
    _check(_load().oracle_pool_ablation(_p(hidden), _dtype_code(hidden), d, _p(offsets), B,
                                        int(kind), _p(pooled)), "pool_ablation")
    return pooled


# --------------------------------------------------------------------------- head
@dataclass
class Head:
    """Two-layer perceptron d -> d_h (ReLU) -> n_out. Weights fp32 or bf16 bits (uint16)."""
    w1: np.ndarray                        # [d_h x d]
    w2: np.ndarray                        # [n_out x d_h]
    b1: Optional[np.ndarray] = None       # [d_h] fp32
    b2: Optional[np.ndarray] = None       # [n_out] fp32
    bin_centers: Optional[np.ndarray] = None  # [n_out]; only for the K-bin decode of Eq. 6


def head_raw(x, head: Head) -> np.ndarray:
    """[B x n_out] outputs of the perceptron, before any softmax."""
    x = _c(np.asarray(x, dtype=np.float64))
    w1, w2 = _c(head.w1), _c(head.w2)
    B, d = x.shape
    d_h, n_out = w1.shape[0], w2.shape[0]
    assert w1.shape == (d_h, d) and w2.shape == (n_out, d_h) and w1.dtype == w2.dtype
    b1 = None if head.b1 is None else _c(np.asarray(head.b1, dtype=np.float32))
    b2 = None if head.b2 is None else _c(np.asarray(head.b2, dtype=np.float32))
    out = np.zeros((B, n_out), dtype=np.float64)
    _check(_load().oracle_head(_p(x), B, d, d_h, n_out, _p(w1), _p(b1), _p(w2), _p(b2),
                               _dtype_code(w1), _p(out)), "head")
    return out


def bin_decode(logits_bk, centers):
    """Eq. 6: (p_hat[B x K], y_hat[B])."""
    z = _c(np.asarray(logits_bk, dtype=np.float64))
    c = _c(np.asarray(centers, dtype=np.float64))
    B, K = z.shape
    assert c.shape == (K,)
    p = np.zeros((B, K), dtype=np.float64)
    y = np.zeros(B, dtype=np.float64)
    _check(_load().oracle_bin_decode(_p(z), B, K, _p(c), _p(p), _p(y)), "bin_decode")
    return p, y


def predict(x, head: Head) -> np.ndarray:
    """Predicted length per row of x: the scalar output, or Eq. 6 when the head has K bins."""
    raw = head_raw(x, head)
    if head.bin_centers is None:
        assert raw.shape[1] == 1
        return raw[:, 0].copy()
    return bin_decode(raw, head.bin_centers)[1]


# --------------------------------------------------------------------------- compositions
@dataclass
class EgtpResult:
    entropy: np.ndarray   # [T]
    weights: np.ndarray   # [T]
    pooled: np.ndarray    # [B x d]
    lse: np.ndarray       # [B]
    pred: np.ndarray      # [B]


def egtp(hidden: np.ndarray, offsets, w_lm: np.ndarray, head: Head, alpha: float = 1.0,
         entropy_in=None) -> EgtpResult:
    """Eq. 2 -> Eq. 3 -> Eq. 4 -> head.  ``entropy_in`` replaces step 1 (used to check the
    pooling and the head on their own against another source of entropies)."""
    H = entropy(hidden, w_lm) if entropy_in is None else np.asarray(entropy_in, dtype=np.float64)
    w, pooled, lse = pool(hidden, H, offsets, alpha)
    return EgtpResult(H, w, pooled, lse, predict(pooled, head))


def plp(prompt_hidden: np.ndarray, prompt_offsets, generated: Sequence[np.ndarray],
        w_lm: np.ndarray, head_rem: Head, alpha: float = 1.0):
    """Eq. 8 with the running-pool reading of Aggregate: for t = 1..len(generated), the
    remaining-length prediction from the prompt tokens followed by generated tokens 1..t.

    ``generated[t-1]`` is [B x d]: one new hidden state per sequence at step t.
    Returns a list of EgtpResult, one per step (entropy/weights over the concatenation)."""
    prompt_offsets = np.asarray(prompt_offsets, dtype=np.int32)
    B = prompt_offsets.size - 1
    out = []
    for t in range(1, len(generated) + 1):
        rows, lens = [], []
        for b in range(B):
            rows.append(prompt_hidden[prompt_offsets[b]:prompt_offsets[b + 1]])
            for s in range(t):
                rows.append(generated[s][b:b + 1])
            lens.append(int(prompt_offsets[b + 1] - prompt_offsets[b]) + t)
        cat = np.concatenate(rows, axis=0)
        out.append(egtp(cat, offsets_from_lengths(lens), w_lm, head_rem, alpha))
    return out


# --------------------------------------------------------------------------- training objective
def soft_label(i: int, K: int) -> np.ndarray:
    """Eq. 5: soft label distribution over K bins for a target in bin i (0-based)."""
    p = np.zeros(K, dtype=np.float64)
    _check(_load().oracle_soft_label(int(i), int(K), _p(p)), "soft_label")
    return p


@dataclass
class TrainHead:
    """fp64 parameters of a K-bin head d -> d_h (ReLU) -> K and its AdamW moments."""
    w1: np.ndarray
    b1: np.ndarray
    w2: np.ndarray
    b2: np.ndarray
    centers: np.ndarray
    m: Optional[list] = None
    v: Optional[list] = None
    t: int = 0

    def params(self):
        return [self.w1, self.b1, self.w2, self.b2]


def head_loss_grad(x, bins, y, head: TrainHead, lam: float, weight=None):
    """Eq. 7 (Eq. 9 via weights): returns (loss3 = [total, CE, MSE], [g_w1, g_b1, g_w2, g_b2])."""
    x = _c(np.asarray(x, dtype=np.float64))
    bins = _c(np.asarray(bins, dtype=np.int32))
    y = _c(np.asarray(y, dtype=np.float64))
    wgt = None if weight is None else _c(np.asarray(weight, dtype=np.float64))
    B, d = x.shape
    d_h, K = head.w1.shape[0], head.w2.shape[0]
    ps = [_c(np.asarray(a, dtype=np.float64)) for a in (head.w1, head.b1, head.w2, head.b2, head.centers)]
    loss = np.zeros(3, dtype=np.float64)
    gs = [np.zeros_like(ps[i]) for i in range(4)]
    _check(_load().oracle_head_loss_grad(_p(x), _p(bins), _p(y), _p(wgt), B, d, d_h, K, _p(ps[0]), _p(ps[1]),
                                         _p(ps[2]), _p(ps[3]), _p(ps[4]), float(lam), _p(loss), _p(gs[0]),
                                         _p(gs[1]), _p(gs[2]), _p(gs[3])), "head_loss_grad")
    return loss, gs


def adamw_step(w, m, v, g, lr, beta1, beta2, eps, weight_decay, t) -> None:
    """One AdamW step in place on fp64 arrays (contiguous)."""
    for a in (w, m, v, g):
        assert a.dtype == np.float64 and a.flags["C_CONTIGUOUS"]
    _check(_load().oracle_adamw(_p(w), _p(m), _p(v), _p(g), w.size, float(lr), float(beta1), float(beta2),
                                float(eps), float(weight_decay), int(t)), "adamw")


def train_step(x, bins, y, head: TrainHead, lam=0.95, lr=2e-5, beta1=0.9, beta2=0.999, eps=1e-8,
               weight_decay=0.01, weight=None):
    """Loss, gradient and one AdamW update of every head parameter (in place). Returns loss3."""
    loss, gs = head_loss_grad(x, bins, y, head, lam, weight)
    if head.m is None:
        head.m = [np.zeros_like(p) for p in head.params()]
        head.v = [np.zeros_like(p) for p in head.params()]
    head.t += 1
    for p, m, v, g in zip(head.params(), head.m, head.v, gs):
        adamw_step(p, m, v, g, lr, beta1, beta2, eps, weight_decay, head.t)
    return loss
