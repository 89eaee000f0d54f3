"""Pins for the oracle's ready-mark / in-order launch model
(Section 4.2 "Autograd Hook"; Section 3.2.3, first and second caveat)."""
import numpy as np
import pytest

import oracle
import workloads
from conftest import read_golden

FP32 = oracle.DT_FP32


def tiny_asg():
    numel = workloads.numel_of(workloads.tiny_shapes())
    return oracle.assign_buckets(numel, [FP32] * 8, 16384)


@pytest.mark.parametrize("case", ["reverse", "forward", "late", "skipped", "partial"])
def test_hand_worked_schedules(case):
    g = read_golden("tiny_schedule.txt")
    order = [int(x) for x in g[case + "_order"].split()]
    want = [tuple(int(v) for v in item.split("@")) for item in g[case + "_log"].split()]
    assert oracle.launch_schedule(tiny_asg(), order) == want


def closed_form(asg, order):
    """launch call of bucket b = latest ready mark among all parameters of
    buckets 0..b (or 'finalize' if one of them is never marked)."""
    pos = {p: i for i, p in enumerate(order)}
    out, worst = [], -1
    for b, bk in enumerate(asg.buckets):
        for p in bk.params:
            worst = max(worst, pos.get(p, len(order)))
        out.append((b, worst))
    return out


@pytest.mark.parametrize("seed", range(25))
def test_random_orders_against_closed_form(seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(1, 60))
    numel = [int(x) for x in rng.integers(1, 400, size=n)]
    asg = oracle.assign_buckets(numel, [FP32] * n, int(rng.integers(0, 3000)))
    order = [int(p) for p in rng.permutation(n)]
    if seed % 2:
        order = order[: int(rng.integers(0, n + 1))]   # some never marked
    log = oracle.launch_schedule(asg, order)
    assert [b for b, _ in log] == list(range(len(asg.buckets)))
    assert log == closed_form(asg, order)


def test_double_mark_and_bad_id_are_errors():
    asg = tiny_asg()
    with pytest.raises(ValueError):
        oracle.launch_schedule(asg, [7, 7])
    with pytest.raises(ValueError):
        oracle.launch_schedule(asg, [8])
    with pytest.raises(ValueError):
        oracle.launch_schedule(asg, [-1])
