"""Pins of the step-by-step scheduling reference (oracle/sched.py): none of the expected values
below comes from that code."""
import itertools
import math

import numpy as np

from oracle import sched


def test_hand_worked_example():
    # true lengths 5, 2, 9, 2, 7 in order [1, 3, 0, 4, 2], batches of 2:
    #   batch 0 = {1, 3}: lengths 2, 2 -> runs 2 steps, allocated 4, jobs done at step 2, 2
    #   batch 1 = {0, 4}: lengths 5, 7 -> runs 7 steps (2..9), allocated 14, done at 7 and 9
    #   batch 2 = {2}:    length 9     -> runs 9 steps (9..18), allocated 9, done at 18
    r = sched.simulate([1, 3, 0, 4, 2], [5, 2, 9, 2, 7], 2)
    assert r.n_batches == 3
    assert r.actual_tokens == 25 and r.allocated_tokens == 27
    assert r.completion == [7, 2, 18, 2, 9] and r.batch_of == [1, 0, 2, 0, 1]
    assert r.makespan_steps == 18 and r.sum_jct_steps == 38
    assert r.padding_ratio == 2 / 25 and r.avg_jct_steps == 38 / 5 and r.throughput == 5 / 18
    # the same jobs in submission order: batches {0,1} {2,3} {4}: allocated 10 + 18 + 7 = 35
    r = sched.simulate([0, 1, 2, 3, 4], [5, 2, 9, 2, 7], 2)
    assert r.allocated_tokens == 35 and r.padding_ratio == 10 / 25
    assert r.completion == [5, 2, 14, 7, 21]


def test_sjf_order_examples():
    assert sched.sjf_order([3.0, 1.0, 2.0]) == [1, 2, 0]
    assert sched.sjf_order([2.0, 1.0, 2.0, 1.0]) == [1, 3, 0, 2]          # ties keep submission order
    assert sched.sjf_order([float("nan"), 5.0, float("nan"), -1.0]) == [3, 1, 0, 2]
    assert sched.sjf_order([]) == []
    assert sched.sjf_order([float("inf"), float("-inf"), 0.0]) == [1, 2, 0]


def test_equal_lengths_have_no_padding():
    n, L, bs = 10, 7, 4
    r = sched.simulate(list(range(n)), [L] * n, bs)
    assert r.padding_ratio == 0.0 and r.allocated_tokens == r.actual_tokens == n * L
    assert r.n_batches == 3 and r.makespan_steps == 3 * L
    # batches of 4, 4, 2 finishing at L, 2L, 3L
    assert r.sum_jct_steps == 4 * L + 4 * 2 * L + 2 * 3 * L


def test_batch_size_one_closed_forms():
    t = [4, 1, 3, 2]
    r = sched.simulate([0, 1, 2, 3], t, 1)
    assert r.padding_ratio == 0.0 and r.makespan_steps == 10
    assert r.completion == [4, 5, 8, 10]                                    # prefix sums
    r = sched.simulate(sched.sjf_order(t), t, 1)
    # sorted lengths 1, 2, 3, 4: completion 1, 3, 6, 10 -> sum = sum_k (n - k) * t_(k)
    assert r.sum_jct_steps == 20 == 4 * 1 + 3 * 2 + 2 * 3 + 1 * 4


def test_one_batch_pads_to_the_longest():
    t = [3, 10, 1, 6]
    r = sched.simulate([2, 0, 3, 1], t, 8)
    assert r.n_batches == 1 and r.allocated_tokens == 40 and r.actual_tokens == 20
    assert r.padding_ratio == 1.0 and r.completion == t and r.makespan_steps == 10


def test_zero_length_jobs_and_empty_input():
    r = sched.simulate([0, 1, 2], [0, 3, 0], 2)
    assert r.completion == [0, 3, 3] and r.allocated_tokens == 6 and r.actual_tokens == 3
    r = sched.simulate([0, 1], [0, 0], 1)
    assert r.padding_ratio == 0.0 and r.throughput == 0.0 and r.n_batches == 2
    r = sched.simulate([], [], 3)
    assert r.n_batches == 0 and r.avg_jct_steps == 0.0


def test_shortest_first_minimises_mean_completion_brute_force():
    rng = np.random.default_rng(0)
    for _ in range(5):
        t = rng.integers(1, 30, size=6).tolist()
        best = min(sched.simulate(list(p), t, 1).sum_jct_steps for p in itertools.permutations(range(6)))
        assert sched.simulate(sched.sjf_order(t), t, 1).sum_jct_steps == best


def test_sorting_before_cutting_minimises_allocation_brute_force():
    rng = np.random.default_rng(1)
    for bs in (2, 3):
        t = rng.integers(1, 50, size=6).tolist()
        best = min(sched.simulate(list(p), t, bs).allocated_tokens for p in itertools.permutations(range(6)))
        assert sched.simulate(sched.sjf_order(t), t, bs).allocated_tokens == best


def test_allocation_matches_the_definition_on_random_cases():
    # independent evaluation of R_allocated = sum_batches |batch| * max length with numpy
    rng = np.random.default_rng(2)
    for n, bs in ((17, 4), (32, 8), (9, 16)):
        t = rng.integers(0, 200, size=n)
        order = rng.permutation(n)
        r = sched.simulate(order.tolist(), t.tolist(), bs)
        want = sum(len(c) * int(t[c].max()) for c in (order[i:i + bs] for i in range(0, n, bs)))
        assert r.allocated_tokens == want and r.actual_tokens == int(t.sum())
        assert math.isclose(r.padding_ratio, (want - t.sum()) / t.sum(), rel_tol=0, abs_tol=0)
