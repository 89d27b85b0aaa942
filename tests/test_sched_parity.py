"""The library's host-side scheduling calls against the step-by-step reference: integer results
bit for bit, the three ratios as the same single double division.  Needs no GPU."""
import ctypes

import numpy as np
import pytest

from oracle import sched
from paper_2602_11812_amd import binding


def _same(rep, done, batch_of, want):
    assert rep.n_batches == want.n_batches
    assert rep.actual_tokens == want.actual_tokens and rep.allocated_tokens == want.allocated_tokens
    assert rep.makespan_steps == want.makespan_steps and rep.sum_jct_steps == want.sum_jct_steps
    assert rep.padding_ratio == want.padding_ratio
    assert rep.avg_jct_steps == want.avg_jct_steps and rep.throughput == want.throughput
    assert done.tolist() == want.completion and batch_of.tolist() == want.batch_of


@pytest.mark.parametrize("n,bs,seed", [(1, 1, 0), (7, 2, 1), (33, 8, 2), (64, 16, 3), (50, 64, 4), (40, 1, 5)])
def test_simulation_matches_reference(n, bs, seed):
    rng = np.random.default_rng(seed)
    t = np.clip(np.rint(np.exp(rng.normal(3.5, 1.0, size=n))), 0, 400).astype(np.int32)
    pred = (t * np.exp(rng.normal(0, 0.4, size=n))).astype(np.float32)       # noisy predictions
    pred[rng.random(n) < 0.2] = np.float32(17.0)                              # ties
    order = binding.egtp_sjf_order(pred)
    assert order.tolist() == sched.sjf_order(pred.tolist())
    rep, done, batch_of = binding.egtp_simulate_batches(order, t, bs)
    _same(rep, done, batch_of, sched.simulate(order.tolist(), t.tolist(), bs))
    fcfs = np.arange(n, dtype=np.int32)
    rep, done, batch_of = binding.egtp_simulate_batches(fcfs, t, bs)
    _same(rep, done, batch_of, sched.simulate(fcfs.tolist(), t.tolist(), bs))


def test_order_with_nan_inf_and_empty():
    pred = np.array([np.nan, 3.0, -np.inf, np.nan, np.inf, 3.0, -0.0, 0.0], dtype=np.float32)
    assert binding.egtp_sjf_order(pred).tolist() == sched.sjf_order(pred.tolist()) == [2, 6, 7, 1, 5, 4, 0, 3]
    assert binding.egtp_sjf_order(np.zeros(0, np.float32)).size == 0
    rep, done, _ = binding.egtp_simulate_batches(np.zeros(0, np.int32), np.zeros(0, np.int32), 4)
    assert rep.n_batches == 0 and rep.padding_ratio == 0.0 and done.size == 0


def test_better_predictions_pad_less_on_a_long_tailed_draw():
    # what the predictions are for: on a long-tailed draw, padding falls from submission order
    # to noisy shortest-first to exact shortest-first (and exact order is optimal)
    rng = np.random.default_rng(9)
    t = np.clip(np.rint(np.exp(rng.normal(6.0, 1.0, size=512))), 1, 8192).astype(np.int32)
    ratios = []
    for sigma in (None, 0.6, 0.2, 0.0):
        if sigma is None:
            order = np.arange(t.size, dtype=np.int32)
        else:
            order = binding.egtp_sjf_order((t * np.exp(rng.normal(0, sigma, size=t.size))).astype(np.float32))
        ratios.append(binding.egtp_simulate_batches(order, t, 16)[0].padding_ratio)
    assert ratios[0] > ratios[1] > ratios[2] > ratios[3] >= 0.0


def test_argument_errors():
    lib = binding.load_library()
    rep = binding.egtp_sched_report()
    o = np.array([0, 1, 1], dtype=np.int32)
    t = np.array([1, 2, 3], dtype=np.int32)
    p = lambda a: a.ctypes.data_as(ctypes.c_void_p)
    assert lib.egtp_simulate_batches(p(o), p(t), 3, 2, ctypes.byref(rep), None, None) == 3     # not a permutation
    o[:] = [0, 1, 3]
    assert lib.egtp_simulate_batches(p(o), p(t), 3, 2, ctypes.byref(rep), None, None) == 3
    o[:] = [0, 1, 2]
    assert lib.egtp_simulate_batches(p(o), p(t), 3, 0, ctypes.byref(rep), None, None) == 2     # batch size
    t[1] = -1
    assert lib.egtp_simulate_batches(p(o), p(t), 3, 2, ctypes.byref(rep), None, None) == 2     # negative length
    assert lib.egtp_simulate_batches(p(o), p(t), 3, 2, None, None, None) == 1
    assert lib.egtp_sjf_order(None, 3, p(o)) == 1 and lib.egtp_sjf_order(None, -1, None) == 2
