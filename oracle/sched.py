"""TEST INFRASTRUCTURE -- step-by-step reference of the host-side scheduling model.

A literal discrete-time simulation of the system the end-to-end metrics are defined on
(Section 4.3; appendix on end-to-end system metrics): jobs all submitted at step 0, one engine,
batches of consecutive jobs in the given order, a batch decodes in lock step until its longest
member is done, every member keeps its slot until then.  The simulation advances one decode
step at a time and counts slots and tokens as they happen -- no closed forms -- so that the
library's arithmetic can be checked against the definition.  Plain Python, small inputs only.

Pins (tests/test_oracle_sched_pins.py): a hand-worked example, closed forms for equal lengths
and batch size 1, and brute force over all permutations for the two optimality facts
(shortest-first minimises the mean completion time; sorting before cutting minimises the
allocated slots).
"""
import math
from dataclasses import dataclass
from typing import List, Sequence


def sjf_order(pred: Sequence[float]) -> List[int]:
    """Jobs by ascending predicted length; ties and NaNs keep submission order, NaNs last."""
    def key(i):
        p = float(pred[i])
        return (1, 0.0, i) if math.isnan(p) else (0, p, i)
    return sorted(range(len(pred)), key=key)


@dataclass
class Report:
    n_batches: int
    actual_tokens: int
    allocated_tokens: int
    makespan_steps: int
    sum_jct_steps: int
    padding_ratio: float
    avg_jct_steps: float
    throughput: float
    completion: List[int]
    batch_of: List[int]


def simulate(order: Sequence[int], true_len: Sequence[int], batch_size: int) -> Report:
    n = len(true_len)
    assert sorted(order) == list(range(n)) and batch_size >= 1 and all(t >= 0 for t in true_len)
    completion = [0] * n
    batch_of = [0] * n
    clock = 0            # decode steps elapsed
    allocated = 0        # token slots held, summed over steps
    actual = 0           # tokens really produced
    n_batches = 0
    queue = list(order)
    while queue:
        batch, queue = queue[:batch_size], queue[batch_size:]
        remaining = {j: int(true_len[j]) for j in batch}
        for j in batch:
            batch_of[j] = n_batches
            if remaining[j] == 0:
                completion[j] = clock
        while any(r > 0 for r in remaining.values()):
            clock += 1
            allocated += len(batch)              # every member holds its slot this step
            for j in batch:
                if remaining[j] > 0:
                    remaining[j] -= 1
                    actual += 1
                    if remaining[j] == 0:
                        completion[j] = clock
        n_batches += 1
    sum_jct = sum(completion)
    return Report(n_batches, actual, allocated, clock, sum_jct,
                  (allocated - actual) / actual if actual > 0 else 0.0,
                  sum_jct / n if n > 0 else 0.0,
                  n / clock if clock > 0 else 0.0, completion, batch_of)
