"""ctypes binding of the C-ABI library (``include/egtp.h``): same names, argument marshalling only.

Every step of EGTP / PLP runs in the HIP kernels behind these calls.  PyTorch is used for
device memory and streams and for nothing else; there is no CPU or eager fallback -- if the
built library is missing this module raises.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import (POINTER, Structure, byref, c_char_p, c_double, c_float, c_int, c_int32, c_int64, c_size_t,
                    c_void_p)
from typing import Optional

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libegtp.so")

EGTP_OK = 0
EGTP_F32, EGTP_BF16 = 0, 1
EGTP_POOL_AVERAGE, EGTP_POOL_MAX, EGTP_POOL_LAST = 0, 1, 2

EXPORTS = ("egtp_create", "egtp_destroy", "egtp_workspace_bytes", "egtp_status_string",
           "egtp_last_hip_error", "egtp_build_offsets", "egtp_score", "plp_step", "egtp_pool_ablation",
           "egtp_profile_enable", "egtp_profile_read", "egtp_mfma_probe_sink_floats", "egtp_mfma_probe",
           "egtp_packed_w_lm_bytes", "egtp_pack_w_lm", "egtp_adopt_packed_w_lm", "egtp_score_dist", "plp_step_dist", "egtp_launch_plan_query", "egtp_hbm_read_probe", "egtp_hbm_read_probe_sink_bytes", "plp_step_static", "egtp_static_scratch_bytes",
           "egtp_head_train_workspace_bytes", "egtp_head_train_step", "egtp_sjf_order", "egtp_simulate_batches")


class egtp_head(Structure):
    _fields_ = [("d_h", c_int32), ("n_out", c_int32), ("wdtype", c_int),
                ("w1", c_void_p), ("b1", c_void_p), ("w2", c_void_p), ("b2", c_void_p),
                ("bin_centers", c_void_p)]


class egtp_config(Structure):
    _fields_ = [("d", c_int32), ("vocab", c_int32), ("dtype", c_int), ("w_lm", c_void_p),
                ("alpha", c_float), ("head_len", egtp_head), ("head_rem", egtp_head)]


class egtp_head_train(Structure):
    _fields_ = [("d", c_int32), ("d_h", c_int32), ("K", c_int32),
                ("w1", c_void_p), ("b1", c_void_p), ("w2", c_void_p), ("b2", c_void_p),
                ("m_w1", c_void_p), ("v_w1", c_void_p), ("m_b1", c_void_p), ("v_b1", c_void_p),
                ("m_w2", c_void_p), ("v_w2", c_void_p), ("m_b2", c_void_p), ("v_b2", c_void_p),
                ("bin_centers", c_void_p),
                ("lambda_", c_float), ("lr", c_float), ("beta1", c_float), ("beta2", c_float),
                ("eps", c_float), ("weight_decay", c_float), ("t", c_int64),
                ("g_w1", c_void_p), ("g_b1", c_void_p), ("g_w2", c_void_p), ("g_b2", c_void_p)]


class egtp_sched_report(Structure):
    _fields_ = [("n_batches", c_int32), ("actual_tokens", c_int64), ("allocated_tokens", c_int64),
                ("makespan_steps", c_int64), ("sum_jct_steps", c_int64), ("padding_ratio", c_double),
                ("avg_jct_steps", c_double), ("throughput", c_double)]


class egtp_launch_plan(Structure):
    _fields_ = [("tokens_per_block", c_int32), ("rows_per_tile", c_int32), ("token_blocks", c_int32),
                ("vocab_tiles", c_int32), ("vocab_ranges", c_int32), ("tiles_per_range", c_int32),
                ("paced", c_int32)]


class EgtpError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__(f"{what}: status {status} ({egtp_status_string(status)})")


_lib = None


def load_library() -> ctypes.CDLL:
    """Load the in-tree HIP library; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it first (python -m paper_2602_11812_amd.build); "
                           "there is no fallback path")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, i64 = c_void_p, c_int32, c_int64
    lib.egtp_create.argtypes = [POINTER(egtp_config), POINTER(vp)]
    lib.egtp_create.restype = c_int
    lib.egtp_destroy.argtypes = [vp]
    lib.egtp_destroy.restype = c_int
    lib.egtp_workspace_bytes.argtypes = [vp, i64, i32]
    lib.egtp_workspace_bytes.restype = c_size_t
    lib.egtp_status_string.argtypes = [c_int]
    lib.egtp_status_string.restype = c_char_p
    lib.egtp_last_hip_error.argtypes = [vp]
    lib.egtp_last_hip_error.restype = c_int
    lib.egtp_build_offsets.argtypes = [vp, vp, i32, vp, vp, i64, vp]
    lib.egtp_build_offsets.restype = c_int
    lib.egtp_score.argtypes = [vp, vp, vp, vp, i32, i64, vp, c_size_t, vp, vp, vp, vp, vp]
    lib.egtp_score.restype = c_int
    lib.plp_step.argtypes = [vp, vp, vp, vp, vp, i32, i64, vp, vp, vp, c_size_t, vp, vp, vp]
    lib.plp_step.restype = c_int
    lib.egtp_score_dist.argtypes = [vp, vp, vp, vp, i32, i64, vp, c_size_t, vp, vp, vp, vp, vp, vp]
    lib.egtp_score_dist.restype = c_int
    lib.plp_step_dist.argtypes = [vp, vp, vp, vp, vp, i32, i64, vp, vp, vp, c_size_t, vp, vp, vp, vp]
    lib.plp_step_dist.restype = c_int
    lib.egtp_adopt_packed_w_lm.argtypes = [vp, vp, c_size_t]
    lib.egtp_adopt_packed_w_lm.restype = c_int
    lib.plp_step_static.argtypes = [vp, vp, vp, vp, vp, i32, i64, vp, vp, vp, vp, vp]
    lib.plp_step_static.restype = c_int
    lib.egtp_static_scratch_bytes.argtypes = []
    lib.egtp_static_scratch_bytes.restype = c_size_t
    lib.egtp_hbm_read_probe_sink_bytes.argtypes = []
    lib.egtp_hbm_read_probe_sink_bytes.restype = c_size_t
    lib.egtp_hbm_read_probe.argtypes = [vp, vp, c_size_t, vp, c_size_t, i32, vp, vp]
    lib.egtp_hbm_read_probe.restype = c_int
    lib.egtp_launch_plan_query.argtypes = [c_int, i32, i32, i64, POINTER(egtp_launch_plan)]
    lib.egtp_launch_plan_query.restype = c_int
    lib.egtp_pool_ablation.argtypes = [vp, vp, vp, vp, i32, i64, c_int, vp, c_size_t, vp, vp, vp]
    lib.egtp_pool_ablation.restype = c_int
    lib.egtp_packed_w_lm_bytes.argtypes = [vp]
    lib.egtp_packed_w_lm_bytes.restype = c_size_t
    lib.egtp_pack_w_lm.argtypes = [vp, vp, c_size_t, vp]
    lib.egtp_pack_w_lm.restype = c_int
    lib.egtp_profile_enable.argtypes = [vp, c_int, c_int]
    lib.egtp_profile_enable.restype = c_int
    lib.egtp_profile_read.argtypes = [vp, vp, c_int]
    lib.egtp_profile_read.restype = c_int
    lib.egtp_mfma_probe_sink_floats.argtypes = []
    lib.egtp_mfma_probe_sink_floats.restype = c_size_t
    lib.egtp_mfma_probe.argtypes = [vp, vp, c_size_t, i32, i32, i32, vp, vp]
    lib.egtp_mfma_probe.restype = c_int
    lib.egtp_head_train_workspace_bytes.argtypes = [i32, i32, i32, i32]
    lib.egtp_head_train_workspace_bytes.restype = c_size_t
    lib.egtp_head_train_step.argtypes = [POINTER(egtp_head_train), vp, vp, vp, vp, i32, i32, vp, c_size_t, vp, vp]
    lib.egtp_head_train_step.restype = c_int
    lib.egtp_sjf_order.argtypes = [vp, i32, vp]
    lib.egtp_sjf_order.restype = c_int
    lib.egtp_simulate_batches.argtypes = [vp, vp, i32, i32, POINTER(egtp_sched_report), vp, vp]
    lib.egtp_simulate_batches.restype = c_int
    _lib = lib
    return lib


# --------------------------------------------------------------------------- marshalling helpers
def _dev(t: Optional[torch.Tensor]) -> Optional[int]:
    """Device pointer of a contiguous CUDA tensor (None stays NULL)."""
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("expected a contiguous device tensor")
    return t.data_ptr()


def _host_i32(a) -> Optional[np.ndarray]:
    if a is None:
        return None
    return np.ascontiguousarray(np.asarray(a, dtype=np.int32))


def _host_ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(c_void_p)


def _stream(stream) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream or None


def to_device(a: np.ndarray) -> torch.Tensor:
    """numpy -> device tensor; uint16 arrays are bf16 bit patterns."""
    if a.dtype == np.uint16:
        return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.bfloat16:
        return EGTP_BF16
    if t.dtype == torch.float32:
        return EGTP_F32
    raise TypeError(f"unsupported storage type {t.dtype}")


def make_head(w1: torch.Tensor, w2: torch.Tensor, b1: Optional[torch.Tensor] = None,
              b2: Optional[torch.Tensor] = None, bin_centers: Optional[torch.Tensor] = None) -> egtp_head:
    h = egtp_head()
    h.d_h, h.n_out, h.wdtype = w1.shape[0], w2.shape[0], dtype_code(w1)
    h.w1, h.b1, h.w2, h.b2, h.bin_centers = _dev(w1), _dev(b1), _dev(w2), _dev(b2), _dev(bin_centers)
    h._keep = (w1, w2, b1, b2, bin_centers)  # the struct only borrows the device memory
    return h


# --------------------------------------------------------------------------- the C calls
def egtp_status_string(status: int) -> str:
    return load_library().egtp_status_string(int(status)).decode()


def egtp_create(cfg: egtp_config) -> c_void_p:
    ctx = c_void_p()
    st = load_library().egtp_create(byref(cfg), byref(ctx))
    if st != EGTP_OK:
        raise EgtpError(st, "egtp_create")
    return ctx


def egtp_destroy(ctx) -> None:
    load_library().egtp_destroy(ctx)


def egtp_workspace_bytes(ctx, max_tokens: int, max_seqs: int) -> int:
    return int(load_library().egtp_workspace_bytes(ctx, int(max_tokens), int(max_seqs)))


def egtp_packed_w_lm_bytes(ctx) -> int:
    return int(load_library().egtp_packed_w_lm_bytes(ctx))


def egtp_pack_w_lm(ctx, packed_dev, stream=None) -> None:
    nbytes = packed_dev.numel() * packed_dev.element_size() if packed_dev is not None else 0
    st = load_library().egtp_pack_w_lm(ctx, _dev(packed_dev), nbytes, _stream(stream))
    if st != EGTP_OK:
        raise EgtpError(st, "egtp_pack_w_lm")


def egtp_adopt_packed_w_lm(ctx, packed_dev) -> None:
    st = load_library().egtp_adopt_packed_w_lm(ctx, _dev(packed_dev), packed_dev.numel() * packed_dev.element_size())
    if st != EGTP_OK:
        raise EgtpError(st, "egtp_adopt_packed_w_lm")


def egtp_launch_plan_query(dtype: int, d: int, vocab: int, T: int) -> egtp_launch_plan:
    plan = egtp_launch_plan()
    st = load_library().egtp_launch_plan_query(int(dtype), int(d), int(vocab), int(T), byref(plan))
    if st != EGTP_OK:
        raise EgtpError(st, "egtp_launch_plan_query")
    return plan


def egtp_last_hip_error(ctx) -> int:
    return int(load_library().egtp_last_hip_error(ctx))


def egtp_build_offsets(ctx, lengths_dev, B, offsets_dev, seg_ids_dev, T, stream=None) -> None:
    st = load_library().egtp_build_offsets(ctx, _dev(lengths_dev), int(B), _dev(offsets_dev), _dev(seg_ids_dev),
                                           int(T), _stream(stream))
    if st != EGTP_OK:
        raise EgtpError(st, "egtp_build_offsets")


def egtp_score(ctx, hidden, offsets_dev, offsets_host, B, T, workspace, entropy_out, pooled_out, lse_out,
               pred_out, stream=None) -> None:
    oh = _host_i32(offsets_host)
    st = load_library().egtp_score(ctx, _dev(hidden), _dev(offsets_dev), _host_ptr(oh), int(B), int(T),
                                   _dev(workspace), workspace.numel() * workspace.element_size() if workspace is not None else 0,
                                   _dev(entropy_out), _dev(pooled_out), _dev(lse_out), _dev(pred_out),
                                   _stream(stream))
    if st != EGTP_OK:
        raise EgtpError(st, "egtp_score")


def _nbytes(t) -> int:
    return t.numel() * t.element_size() if t is not None else 0


def egtp_score_dist(ctx, hidden, offsets_dev, offsets_host, B, T, workspace, entropy_out, pooled_out, lse_out,
                    pred_out, p_hat_out, stream=None) -> None:
    oh = _host_i32(offsets_host)
    st = load_library().egtp_score_dist(ctx, _dev(hidden), _dev(offsets_dev), _host_ptr(oh), int(B), int(T),
                                        _dev(workspace), _nbytes(workspace), _dev(entropy_out), _dev(pooled_out),
                                        _dev(lse_out), _dev(pred_out), _dev(p_hat_out), _stream(stream))
    if st != EGTP_OK:
        raise EgtpError(st, "egtp_score_dist")


def plp_step_dist(ctx, hidden_new, offsets_new_dev, offsets_new_host, slot_dev, B, T_new, pooled_state, lse_state,
                  workspace, entropy_out, rem_pred_out, p_hat_out, stream=None) -> None:
    oh = _host_i32(offsets_new_host)
    st = load_library().plp_step_dist(ctx, _dev(hidden_new), _dev(offsets_new_dev), _host_ptr(oh), _dev(slot_dev),
                                      int(B), int(T_new), _dev(pooled_state), _dev(lse_state), _dev(workspace),
                                      _nbytes(workspace), _dev(entropy_out), _dev(rem_pred_out), _dev(p_hat_out),
                                      _stream(stream))
    if st != EGTP_OK:
        raise EgtpError(st, "plp_step_dist")


def egtp_static_scratch_bytes() -> int:
    return int(load_library().egtp_static_scratch_bytes())


def plp_step_static(ctx, hidden_new, offsets_new_dev, offsets_new_host, slot_dev, B, T_new, pooled_state, lse_state,
                    entropy_out, rem_pred_out, stream=None) -> None:
    oh = _host_i32(offsets_new_host)
    st = load_library().plp_step_static(ctx, _dev(hidden_new), _dev(offsets_new_dev), _host_ptr(oh), _dev(slot_dev),
                                        int(B), int(T_new), _dev(pooled_state), _dev(lse_state), _dev(entropy_out),
                                        _dev(rem_pred_out), _stream(stream))
    if st != EGTP_OK:
        raise EgtpError(st, "plp_step_static")


def plp_step(ctx, hidden_new, offsets_new_dev, offsets_new_host, slot_dev, B, T_new, pooled_state, lse_state,
             workspace, entropy_out, rem_pred_out, stream=None) -> None:
    oh = _host_i32(offsets_new_host)
    st = load_library().plp_step(ctx, _dev(hidden_new), _dev(offsets_new_dev), _host_ptr(oh), _dev(slot_dev),
                                 int(B), int(T_new), _dev(pooled_state), _dev(lse_state), _dev(workspace),
                                 workspace.numel() * workspace.element_size() if workspace is not None else 0,
                                 _dev(entropy_out), _dev(rem_pred_out), _stream(stream))
    if st != EGTP_OK:
        raise EgtpError(st, "plp_step")


def egtp_pool_ablation(ctx, hidden, offsets_dev, offsets_host, B, T, kind, workspace, pooled_out, pred_out,
                       stream=None) -> None:
    oh = _host_i32(offsets_host)
    st = load_library().egtp_pool_ablation(ctx, _dev(hidden), _dev(offsets_dev), _host_ptr(oh), int(B), int(T),
                                           int(kind), _dev(workspace),
                                           workspace.numel() * workspace.element_size() if workspace is not None else 0,
                                           _dev(pooled_out), _dev(pred_out), _stream(stream))
    if st != EGTP_OK:
        raise EgtpError(st, "egtp_pool_ablation")


def egtp_profile_enable(ctx, on: bool, capacity: int = 256) -> None:
    st = load_library().egtp_profile_enable(ctx, int(bool(on)), int(capacity))
    if st != EGTP_OK:
        raise EgtpError(st, "egtp_profile_enable")


def egtp_profile_read(ctx, cap: int = 1024) -> np.ndarray:
    """Elapsed ms of each recorded fused-entropy kernel since the last read (stream must be idle)."""
    buf = np.zeros(cap, dtype=np.float32)
    n = load_library().egtp_profile_read(ctx, buf.ctypes.data_as(c_void_p), cap)
    if n < 0:
        raise RuntimeError("egtp_profile_read failed")
    return buf[:n].copy()


def egtp_mfma_probe_sink_floats() -> int:
    return int(load_library().egtp_mfma_probe_sink_floats())


def egtp_mfma_probe(ctx, sink: torch.Tensor, iters: int, random_operands: bool, launches: int,
                    stream=None) -> np.ndarray:
    """TFLOP/s of each of `launches` register-only MFMA kernels run back to back (blocks until done)."""
    assert sink.is_cuda and sink.dtype == torch.float32 and sink.is_contiguous()
    out = np.zeros(int(launches), dtype=np.float64)
    st = load_library().egtp_mfma_probe(ctx, _dev(sink), sink.numel(), int(iters), int(bool(random_operands)),
                                        int(launches), out.ctypes.data_as(c_void_p), _stream(stream))
    if st != EGTP_OK:
        raise EgtpError(st, "egtp_mfma_probe")
    return out


def egtp_hbm_read_probe_sink_bytes() -> int:
    return int(load_library().egtp_hbm_read_probe_sink_bytes())


def egtp_hbm_read_probe(ctx, buf: torch.Tensor, sink: torch.Tensor, launches: int, stream=None) -> np.ndarray:
    """GB/s of each of `launches` plain streaming reads of `buf` run back to back (blocks until done)."""
    out = np.zeros(int(launches), dtype=np.float64)
    st = load_library().egtp_hbm_read_probe(ctx, _dev(buf), _nbytes(buf), _dev(sink), _nbytes(sink), int(launches),
                                            out.ctypes.data_as(c_void_p), _stream(stream))
    if st != EGTP_OK:
        raise EgtpError(st, "egtp_hbm_read_probe")
    return out


def egtp_head_train_workspace_bytes(B: int, d: int, d_h: int, K: int) -> int:
    return int(load_library().egtp_head_train_workspace_bytes(int(B), int(d), int(d_h), int(K)))


def egtp_head_train_step(head: egtp_head_train, x, bin, y, steps_per_seq, n_seqs, B, workspace, loss_out,
                         stream=None) -> None:
    st = load_library().egtp_head_train_step(byref(head), _dev(x), _dev(bin), _dev(y), _dev(steps_per_seq),
                                             int(n_seqs), int(B), _dev(workspace),
                                             workspace.numel() * workspace.element_size() if workspace is not None else 0,
                                             _dev(loss_out), _stream(stream))
    if st != EGTP_OK:
        raise EgtpError(st, "egtp_head_train_step")


# --------------------------------------------------------------------------- host-side scheduling model
def egtp_sjf_order(pred) -> np.ndarray:
    """Shortest-predicted-job-first permutation of host predictions (fp32)."""
    p = np.ascontiguousarray(np.asarray(pred, dtype=np.float32))
    order = np.empty(p.size, dtype=np.int32)
    st = load_library().egtp_sjf_order(_host_ptr(p), p.size, _host_ptr(order))
    if st != EGTP_OK:
        raise EgtpError(st, "egtp_sjf_order")
    return order


def egtp_simulate_batches(order, true_len, batch_size: int):
    """Returns (egtp_sched_report, completion_step[n] int64, batch_of[n] int32)."""
    o, t = _host_i32(order), _host_i32(true_len)
    n = t.size
    rep = egtp_sched_report()
    done = np.zeros(n, dtype=np.int64)
    batch_of = np.zeros(n, dtype=np.int32)
    st = load_library().egtp_simulate_batches(_host_ptr(o), _host_ptr(t), n, int(batch_size), byref(rep),
                                              _host_ptr(done), _host_ptr(batch_of))
    if st != EGTP_OK:
        raise EgtpError(st, "egtp_simulate_batches")
    return rep, done, batch_of


# --------------------------------------------------------------------------- convenience (memory only)
class HeadTrainer:
    """Owns the fp32 parameters, AdamW moments and workspace of one K-bin head.  No arithmetic here."""

    def __init__(self, w1, b1, w2, b2, bin_centers, lam=0.95, lr=2e-5, beta1=0.9, beta2=0.999, eps=1e-8,
                 weight_decay=0.01, keep_grads=False):
        self.params = dict(w1=w1, b1=b1, w2=w2, b2=b2)
        for p in self.params.values():
            if p.dtype != torch.float32:
                raise TypeError("training keeps fp32 parameters")
        self.centers = bin_centers
        self.m = {k: torch.zeros_like(p) for k, p in self.params.items()}
        self.v = {k: torch.zeros_like(p) for k, p in self.params.items()}
        self.grads = {k: torch.zeros_like(p) for k, p in self.params.items()} if keep_grads else None
        self.hyper = dict(lam=lam, lr=lr, beta1=beta1, beta2=beta2, eps=eps, weight_decay=weight_decay)
        self.t = 0
        self.d_h, self.d = w1.shape
        self.K = w2.shape[0]
        self.loss = torch.zeros(3, dtype=torch.float32, device="cuda")
        self._ws = None

    def _struct(self) -> egtp_head_train:
        h = egtp_head_train()
        h.d, h.d_h, h.K = self.d, self.d_h, self.K
        for k, p in self.params.items():
            setattr(h, k, _dev(p))
            setattr(h, "m_" + k, _dev(self.m[k]))
            setattr(h, "v_" + k, _dev(self.v[k]))
            setattr(h, "g_" + k, _dev(self.grads[k]) if self.grads else None)
        h.bin_centers = _dev(self.centers)
        hp = self.hyper
        h.lambda_, h.lr, h.beta1, h.beta2 = hp["lam"], hp["lr"], hp["beta1"], hp["beta2"]
        h.eps, h.weight_decay, h.t = hp["eps"], hp["weight_decay"], self.t
        return h

    def step(self, x, bins, y, steps_per_seq=None, n_seqs=0) -> torch.Tensor:
        """One optimisation step; returns the device tensor [loss, CE, MSE] (valid after a sync)."""
        B = x.shape[0]
        need = egtp_head_train_workspace_bytes(B, self.d, self.d_h, self.K)
        if self._ws is None or self._ws.numel() < need:
            self._ws = torch.empty(max(need, 256), dtype=torch.uint8, device="cuda")
        h = self._struct()
        h.t = self.t + 1
        egtp_head_train_step(h, x, bins, y, steps_per_seq, n_seqs, B, self._ws, self.loss)
        self.t += 1                      # only a step that was enqueued counts
        return self.loss

    def as_head(self) -> egtp_head:
        """The trained parameters as a scoring head (fp32 storage, n_out = K)."""
        p = self.params
        return make_head(p["w1"], p["w2"], p["b1"], p["b2"], self.centers)


class Scorer:
    """Owns a context plus torch-allocated outputs and workspace.  No arithmetic here."""

    def __init__(self, w_lm: torch.Tensor, head_len: egtp_head, head_rem: Optional[egtp_head] = None,
                 alpha: float = 1.0, pack_w_lm: bool = True):
        cfg = egtp_config()
        cfg.vocab, cfg.d = w_lm.shape
        cfg.dtype = dtype_code(w_lm)
        cfg.w_lm = _dev(w_lm)
        cfg.alpha = alpha
        cfg.head_len = head_len
        if head_rem is not None:
            cfg.head_rem = head_rem
        self._keep = (w_lm, head_len, head_rem)
        self.d, self.vocab, self.storage = int(cfg.d), int(cfg.vocab), w_lm.dtype
        self.ctx = egtp_create(cfg)
        self._ws = None
        self._w_packed = None
        if pack_w_lm:
            self._w_packed = torch.empty(egtp_packed_w_lm_bytes(self.ctx), dtype=torch.uint8, device="cuda")
            egtp_pack_w_lm(self.ctx, self._w_packed)

    def close(self):
        if self.ctx is not None:
            egtp_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def workspace(self, T: int, B: int) -> torch.Tensor:
        need = egtp_workspace_bytes(self.ctx, T, B)
        if self._ws is None or self._ws.numel() < need:
            self._ws = torch.empty(max(need, 256), dtype=torch.uint8, device="cuda")
        return self._ws

    def build_offsets(self, lengths_dev: torch.Tensor, T: int, want_seg_ids: bool = False):
        B = lengths_dev.numel()
        offsets = torch.empty(B + 1, dtype=torch.int32, device="cuda")
        seg = torch.empty(T, dtype=torch.int32, device="cuda") if want_seg_ids else None
        egtp_build_offsets(self.ctx, lengths_dev, B, offsets, seg, T)
        return (offsets, seg) if want_seg_ids else offsets

    def score(self, hidden: torch.Tensor, offsets_dev: torch.Tensor, offsets_host=None, out=None):
        """Returns dict(entropy[T], pooled[B x d], lse[B], pred[B]) of device tensors."""
        T, B = hidden.shape[0], offsets_dev.numel() - 1
        if out is None:
            out = dict(entropy=torch.empty(T, dtype=torch.float32, device="cuda"),
                       pooled=torch.empty(B, self.d, dtype=torch.float32, device="cuda"),
                       lse=torch.empty(B, dtype=torch.float32, device="cuda"),
                       pred=torch.empty(B, dtype=torch.float32, device="cuda"))
        egtp_score(self.ctx, hidden, offsets_dev, offsets_host, B, T, self.workspace(T, B), out["entropy"],
                   out["pooled"], out["lse"], out["pred"])
        return out

    def step(self, hidden_new: torch.Tensor, pooled_state: torch.Tensor, lse_state: torch.Tensor,
             offsets_new_dev=None, offsets_new_host=None, slot_dev=None, entropy_out=None, rem_pred_out=None):
        T_new = hidden_new.shape[0]
        B = T_new if offsets_new_dev is None else offsets_new_dev.numel() - 1
        if rem_pred_out is None:
            rem_pred_out = torch.empty(B, dtype=torch.float32, device="cuda")
        plp_step(self.ctx, hidden_new, offsets_new_dev, offsets_new_host, slot_dev, B, T_new, pooled_state,
                 lse_state, self.workspace(T_new, B), entropy_out, rem_pred_out)
        return rem_pred_out

    def pool_ablation(self, hidden, offsets_dev, kind: int, offsets_host=None, want_pred: bool = True):
        T, B = hidden.shape[0], offsets_dev.numel() - 1
        pooled = torch.empty(B, self.d, dtype=torch.float32, device="cuda")
        pred = torch.empty(B, dtype=torch.float32, device="cuda") if want_pred else None
        egtp_pool_ablation(self.ctx, hidden, offsets_dev, offsets_host, B, T, kind, self.workspace(T, B), pooled, pred)
        return pooled, pred
