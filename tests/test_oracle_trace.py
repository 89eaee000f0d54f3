"""Pins for the oracle's traced-order bucket mapping (Section 6.2.1): the
reduction to the default assignment (itself pinned by the hand-derived Tiny
example and an enumeration), a hand-worked example, partition invariants, a
search over all contiguous partitions of small cases, and the property the
rebuild exists for -- when gradients arrive in the traced order again, every
bucket is launched with the mark of its last gradient."""
import itertools

import numpy as np
import pytest

import oracle
from conftest import read_golden

FP32, FP16, BF16 = 0, 1, 2


def parse_log(text):
    return [tuple(int(x) for x in item.split("@")) for item in text.split()]


def test_hand_worked_rebuild():
    g = read_golden("traced_assignment.txt")
    numel = [int(x) for x in g["numel"].split()]
    cap = int(g["cap_bytes"])
    trace = [int(x) for x in g["trace"].split()]
    dflt = oracle.assign_buckets(numel, [FP32] * 6, cap)
    assert dflt.bucket_of.tolist() == [int(x) for x in g["default_bucket_of"].split()]
    assert dflt.offset_of.tolist() == [int(x) for x in g["default_offset_of"].split()]
    assert oracle.launch_schedule(dflt, trace) == parse_log(g["default_log"])
    visit = oracle.traced_visit_order(trace, 6)
    assert visit == [int(x) for x in g["visit_order"].split()]
    asg = oracle.assign_buckets_in_order(numel, [FP32] * 6, cap, visit)
    assert asg.bucket_of.tolist() == [int(x) for x in g["traced_bucket_of"].split()]
    assert asg.offset_of.tolist() == [int(x) for x in g["traced_offset_of"].split()]
    assert oracle.launch_schedule(asg, trace) == parse_log(g["traced_log"])


def same_assignment(a, b):
    return (a.bucket_of.tolist() == b.bucket_of.tolist() and a.offset_of.tolist() == b.offset_of.tolist()
            and [(bk.params, bk.elems, bk.dtype) for bk in a.buckets]
            == [(bk.params, bk.elems, bk.dtype) for bk in b.buckets])


@pytest.mark.parametrize("seed", range(40))
def test_reverse_registration_order_gives_the_default_assignment(seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(1, 200))
    numel = [int(x) for x in rng.integers(0, 5000, size=n)]
    dtype = [FP32] * n if seed % 2 else [int(x) for x in rng.integers(0, 3, size=n)]
    cap = int(rng.choice([0, 1, 100, 4096, 20000, oracle.CAP_WHOLE_MODEL]))
    want = oracle.assign_buckets(numel, dtype, cap)
    assert same_assignment(oracle.assign_buckets_in_order(numel, dtype, cap, list(range(n - 1, -1, -1))), want)
    # an empty trace leaves everything to the default guess
    assert oracle.traced_visit_order([], n) == list(range(n - 1, -1, -1))


def test_model_shapes_with_identity_trace():
    import workloads
    for name, nb in (("resnet50", 5), ("bert_large", 50)):
        numel = workloads.numel_of(workloads.WORKLOAD_SHAPES[name]())
        n = len(numel)
        visit = oracle.traced_visit_order(list(range(n - 1, -1, -1)), n)
        asg = oracle.assign_buckets_in_order(numel, [FP32] * n, 25 << 20, visit)
        assert len(asg.buckets) == nb
        assert same_assignment(asg, oracle.assign_buckets(numel, [FP32] * n, 25 << 20))


def check_invariants(numel, dtype, cap, visit, asg):
    n = len(numel)
    assert [p for bk in asg.buckets for p in bk.params] == list(visit)      # a contiguous partition of the visit order
    assert sorted(visit) == list(range(n))
    for b, bk in enumerate(asg.buckets):
        assert bk.params
        assert all(dtype[p] == bk.dtype for p in bk.params)
        off = 0
        for p in bk.params:
            assert asg.bucket_of[p] == b and asg.offset_of[p] == off
            off += numel[p]
        assert off == bk.elems
        if len(bk.params) > 1:
            assert bk.nbytes <= cap
        if b + 1 < len(asg.buckets):
            nxt = asg.buckets[b + 1].params[0]
            assert dtype[nxt] != bk.dtype or bk.nbytes + numel[nxt] * oracle.ESIZE[dtype[nxt]] > cap


def fullest_partition_by_search(numel, dtype, cap, visit):
    """Every way to cut the visit order into contiguous groups; of the valid
    ones (one element type, within the cap unless a single parameter) the one
    whose group lengths are lexicographically largest."""
    best = None
    for cuts in itertools.product([0, 1], repeat=len(visit) - 1):
        groups, cur = [], [visit[0]]
        for c, p in zip(cuts, visit[1:]):
            if c:
                groups.append(cur)
                cur = [p]
            else:
                cur.append(p)
        groups.append(cur)
        if any(len({dtype[p] for p in g}) > 1 for g in groups):
            continue
        if any(len(g) > 1 and sum(numel[p] * oracle.ESIZE[dtype[p]] for p in g) > cap for g in groups):
            continue
        key = [len(g) for g in groups]
        if best is None or key > best[0]:
            best = (key, groups)
    return best[1]


@pytest.mark.parametrize("seed", range(40))
def test_small_cases_against_search_and_invariants(seed):
    rng = np.random.default_rng(100 + seed)
    n = int(rng.integers(1, 9))
    numel = [int(x) for x in rng.integers(0, 50, size=n)]
    dtype = [FP32] * n if seed % 3 == 0 else [int(x) for x in rng.choice([FP32, FP16, BF16], size=n)]
    cap = int(rng.choice([0, 1, 16, 64, 100, 200, 1000]))
    trace = [int(p) for p in rng.permutation(n)][: int(rng.integers(0, n + 1))]
    visit = oracle.traced_visit_order(trace, n)
    assert visit[: len(trace)] == trace
    assert visit[len(trace):] == sorted(set(range(n)) - set(trace), reverse=True)
    asg = oracle.assign_buckets_in_order(numel, dtype, cap, visit)
    assert [bk.params for bk in asg.buckets] == fullest_partition_by_search(numel, dtype, cap, visit)
    check_invariants(numel, dtype, cap, visit, asg)


@pytest.mark.parametrize("seed", range(30))
def test_repeating_the_traced_order_launches_every_bucket_with_its_last_gradient(seed):
    rng = np.random.default_rng(200 + seed)
    n = int(rng.integers(1, 150))
    numel = [int(x) for x in rng.integers(0, 4000, size=n)]
    dtype = [FP32] * n if seed % 2 else [int(x) for x in rng.integers(0, 3, size=n)]
    cap = int(rng.choice([0, 1000, 8192, 50000]))
    trace = [int(p) for p in rng.permutation(n)]
    visit = oracle.traced_visit_order(trace, n)
    assert visit == trace
    asg = oracle.assign_buckets_in_order(numel, dtype, cap, visit)
    check_invariants(numel, dtype, cap, visit, asg)
    log = oracle.launch_schedule(asg, trace)
    ends = np.cumsum([len(bk.params) for bk in asg.buckets]) - 1
    assert log == [(b, int(e)) for b, e in enumerate(ends)]
    # no other mapping of the same parameters can launch a bucket's worth of
    # gradients earlier: under the default mapping every gradient is launched
    # no earlier than under the rebuilt one
    dflt = oracle.assign_buckets(numel, dtype, cap)
    dlog = dict(oracle.launch_schedule(dflt, trace))
    tlog = dict(log)
    pos = {p: k for k, p in enumerate(trace)}
    for p in range(n):
        assert dlog[int(dflt.bucket_of[p])] >= pos[p]
        assert tlog[int(asg.bucket_of[p])] >= pos[p]
    # the last launch cannot come before the last mark in either mapping
    assert log[-1][1] == n - 1 and max(dlog.values()) == n - 1


def test_results_do_not_depend_on_the_mapping():
    """The averaged gradients are the same numbers whatever the buckets are."""
    rng = np.random.default_rng(5)
    n, R = 25, 3
    numel = [int(x) for x in rng.integers(0, 300, size=n)]
    reps = [[rng.standard_normal(x).astype(np.float32) for x in numel] for _ in range(R)]
    trace = [int(p) for p in rng.permutation(n)]
    a, _, _ = oracle.synchronize(numel, [FP32] * n, 2000, reps, trace)
    b, asg, log = oracle.synchronize(numel, [FP32] * n, 2000, reps, trace, visit_order=trace)
    assert [bk.params for bk in asg.buckets] != [bk.params for bk in oracle.assign_buckets(numel, [FP32] * n, 2000).buckets]
    for p in range(n):
        assert a[p].tobytes() == b[p].tobytes()


def test_bad_traces_are_rejected():
    with pytest.raises(ValueError):
        oracle.traced_visit_order([0, 0], 3)
    with pytest.raises(ValueError):
        oracle.traced_visit_order([3], 3)
    with pytest.raises(ValueError):
        oracle.assign_buckets_in_order([1, 1], [0, 0], 10, [0, 0])
    with pytest.raises(ValueError):
        oracle.assign_buckets_in_order([1, 1], [0, 0], 10, [0])
