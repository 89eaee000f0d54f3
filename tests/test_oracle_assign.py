"""Pins for the oracle's bucket assignment (Algorithm 1 constructor;
Sections 3.2.3 and 4.2 of the paper)."""
import itertools

import numpy as np
import pytest

import oracle
import workloads
from conftest import read_golden

FP32, FP16, BF16 = oracle.DT_FP32, oracle.DT_FP16, oracle.DT_BF16


def tiny():
    return workloads.numel_of(workloads.tiny_shapes())


def test_tiny_matches_hand_derivation():
    g = read_golden("tiny_assignment.txt")
    asg = oracle.assign_buckets(tiny(), [FP32] * 8, int(g["cap_bytes"]))
    want = [[int(x) for x in grp.split()] for grp in g["buckets"].split("|")]
    assert [bk.params for bk in asg.buckets] == want
    assert [bk.nbytes for bk in asg.buckets] == [int(x) for x in g["bucket_bytes"].split()]
    assert asg.bucket_of.tolist() == [int(x) for x in g["bucket_of"].split()]
    assert asg.offset_of.tolist() == [int(x) for x in g["offset_of"].split()]


def check_invariants(numel, dtype, cap, asg):
    n = len(numel)
    es = oracle.ESIZE
    # every parameter in exactly one bucket
    seen = sorted(p for bk in asg.buckets for p in bk.params)
    assert seen == list(range(n))
    # reverse registration order across and inside buckets
    flat_order = [p for bk in asg.buckets for p in bk.params]
    assert flat_order == list(range(n - 1, -1, -1))
    for b, bk in enumerate(asg.buckets):
        assert bk.params, "empty bucket"
        # one element type per bucket
        assert all(dtype[p] == bk.dtype for p in bk.params)
        # dense, ascending, non-overlapping offsets
        off = 0
        for p in bk.params:
            assert asg.bucket_of[p] == b
            assert asg.offset_of[p] == off
            off += numel[p]
        assert off == bk.elems
        # cap respected unless the bucket is a single parameter
        if len(bk.params) > 1:
            assert bk.nbytes <= cap
        # maximal: the next parameter did not fit (or has another type)
        if b + 1 < len(asg.buckets):
            nxt = asg.buckets[b + 1].params[0]
            assert (dtype[nxt] != bk.dtype
                    or bk.nbytes + numel[nxt] * es[dtype[nxt]] > cap)
    assert sum(bk.elems for bk in asg.buckets) == sum(numel)


def greedy_by_enumeration(numel, dtype, cap):
    """All contiguous partitions of the reversed parameter list; keep the
    valid ones (type-pure, within the cap unless single) and take the one
    whose bucket lengths are lexicographically largest -- 'fill each bucket
    as far as it goes' written as a search."""
    n = len(numel)
    order = list(range(n - 1, -1, -1))
    best = None
    for cuts in itertools.product([0, 1], repeat=n - 1):
        groups, cur = [], [order[0]]
        for c, p in zip(cuts, order[1:]):
            if c:
                groups.append(cur)
                cur = [p]
            else:
                cur.append(p)
        groups.append(cur)
        ok = True
        for g in groups:
            if len({dtype[p] for p in g}) > 1:
                ok = False
            size = sum(numel[p] * oracle.ESIZE[dtype[p]] for p in g)
            if len(g) > 1 and size > cap:
                ok = False
        if not ok:
            continue
        key = [len(g) for g in groups]
        if best is None or key > best[0]:
            best = (key, groups)
    return best[1]


@pytest.mark.parametrize("seed", range(40))
def test_small_cases_against_enumeration(seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(1, 9))
    numel = [int(x) for x in rng.integers(0, 50, size=n)]
    dtype = [int(x) for x in rng.choice([FP32, FP16, BF16], size=n, p=[0.6, 0.3, 0.1])]
    if seed % 3 == 0:
        dtype = [FP32] * n
    cap = int(rng.choice([0, 1, 16, 64, 100, 200, 1000]))
    asg = oracle.assign_buckets(numel, dtype, cap)
    assert [bk.params for bk in asg.buckets] == greedy_by_enumeration(numel, dtype, cap)
    check_invariants(numel, dtype, cap, asg)


@pytest.mark.parametrize("seed", range(30))
def test_random_lists_keep_invariants(seed):
    rng = np.random.default_rng(1000 + seed)
    n = int(rng.integers(1, 300))
    numel = [int(x) for x in rng.integers(0, 5000, size=n)]
    dtype = [FP32] * n if seed % 2 else [int(x) for x in rng.integers(0, 3, size=n)]
    cap = int(rng.integers(0, 40000))
    check_invariants(numel, dtype, cap, oracle.assign_buckets(numel, dtype, cap))


def test_exact_fit_stays_in_bucket():
    # 3 x 16 bytes with cap 32: the second parameter makes the bucket exactly full
    asg = oracle.assign_buckets([4, 4, 4], [FP32] * 3, 32)
    assert [bk.params for bk in asg.buckets] == [[2, 1], [0]]


def test_cap_zero_gives_one_bucket_per_gradient():
    # Section 5.2: zero bucket size means each gradient is communicated on its own
    for shapes in (workloads.tiny_shapes(), workloads.resnet50_shapes()):
        numel = workloads.numel_of(shapes)
        asg = oracle.assign_buckets(numel, [FP32] * len(numel), 0)
        assert [bk.params for bk in asg.buckets] == [[p] for p in range(len(numel) - 1, -1, -1)]
        assert all(o == 0 for o in asg.offset_of)


def test_unbounded_cap_gives_one_bucket():
    numel = workloads.numel_of(workloads.resnet50_shapes())
    asg = oracle.assign_buckets(numel, [FP16] * len(numel), oracle.CAP_WHOLE_MODEL)
    assert len(asg.buckets) == 1 and asg.buckets[0].elems == 25_557_032


def test_type_change_closes_bucket():
    asg = oracle.assign_buckets([8, 8, 8, 8], [FP32, FP16, FP16, FP32], 1 << 20)
    assert [bk.params for bk in asg.buckets] == [[3], [2, 1], [0]]
    assert [bk.dtype for bk in asg.buckets] == [FP32, FP16, FP32]


def test_model_sizes():
    # element counts of the two model-shaped lists (public architecture arithmetic)
    r = workloads.numel_of(workloads.resnet50_shapes())
    b = workloads.numel_of(workloads.bert_large_shapes())
    assert (len(r), sum(r)) == (161, 25_557_032)
    assert (len(b), sum(b)) == (391, 335_141_888)


# Bucket counts worked out separately by hand-arithmetic for the build plan
# (cap in MiB -> number of buckets).  A second derivation, not the paper's.
@pytest.mark.parametrize("name,dt,counts", [
    ("resnet50", FP32, {0: 161, 1: 66, 5: 20, 10: 13, 25: 5, 50: 2, 100: 1}),
    ("resnet50", FP16, {0: 161, 1: 44, 5: 13, 10: 7, 25: 2, 50: 1, 100: 1}),
    ("bert_large", FP32, {0: 391, 1: 293, 5: 171, 10: 123, 25: 50, 50: 26, 100: 14}),
])
def test_bucket_counts_of_model_shapes(name, dt, counts):
    numel = workloads.numel_of(workloads.WORKLOAD_SHAPES[name]())
    for mib, want in counts.items():
        asg = oracle.assign_buckets(numel, [dt] * len(numel), mib << 20)
        assert len(asg.buckets) == want
        check_invariants(numel, [dt] * len(numel), mib << 20, asg)


def test_resnet50_default_cap_layout():
    numel = workloads.numel_of(workloads.resnet50_shapes())
    asg = oracle.assign_buckets(numel, [FP32] * 161, 25 << 20)
    assert [len(bk.params) for bk in asg.buckets] == [13, 9, 15, 48, 76]
    # decimal megabytes give a different BERT split: the unit matters
    numel = workloads.numel_of(workloads.bert_large_shapes())
    assert len(oracle.assign_buckets(numel, [FP32] * 391, 25 * 10**6).buckets) == 73
