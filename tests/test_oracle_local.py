"""Pins for the oracle's per-replica participation path and global bitmap
(Section 3.2.3, last paragraph; Section 4.2 "Globally Unused Parameters";
Section 3.2.4 for the accumulation across no_sync iterations)."""
import numpy as np
import pytest

import oracle
import workloads
from conftest import read_golden

FP32, FP16 = oracle.DT_FP32, oracle.DT_FP16


def test_hand_worked_example():
    g = read_golden("local_unused.txt")
    reps = [[np.array([1, 2], np.float32), np.array([10, 20], np.float32), np.array([100, 200], np.float32)],
            [np.array([3, 6], np.float32), np.array([30, 50], np.float32), np.array([300, 400], np.float32)]]
    marks = [(2, [0, 0]), (1, [0, 1]), (0, [1, 1])]
    outs, asg, log, glob = oracle.synchronize_local([2, 2, 2], [FP32] * 3, 1 << 20, reps, marks, True)
    want = lambda key: [float(x) for x in g[key].split()]
    assert glob.tolist() == [int(x) for x in g["global_used"].split()]
    for r in range(2):
        assert outs[r][0].tolist() == want("p0")
        assert outs[r][1].tolist() == want("p1")
    assert outs[0][2].tolist() == want("p2_replica0_intact")
    assert outs[1][2].tolist() == want("p2_replica1_intact")
    outs, _, _, _ = oracle.synchronize_local([2, 2, 2], [FP32] * 3, 1 << 20, reps, marks, False)
    assert outs[0][2].tolist() == want("p2_zeroed") and outs[1][2].tolist() == want("p2_zeroed")
    # a parameter that is never marked at all is globally unused as well
    outs, _, log, glob = oracle.synchronize_local([2, 2, 2], [FP32] * 3, 1 << 20, reps, marks[1:], True)
    assert glob.tolist() == [1, 1, 0] and outs[1][2].tolist() == [300, 400] and log == [(0, 2)]


def test_all_used_equals_plain_synchronization():
    numel = workloads.numel_of(workloads.tiny_shapes())
    R = 3
    reps = [workloads.gaussian_replica(1, r, 0, numel, 1.0) for r in range(R)]
    order = [3, 0, 7, 1, 2, 6, 5, 4]
    base, _, blog = oracle.synchronize(numel, [FP32] * 8, 16384, reps, order)
    outs, _, log, glob = oracle.synchronize_local(numel, [FP32] * 8, 16384, reps, [(p, [1] * R) for p in order])
    assert log == blog and glob.tolist() == [1] * 8
    for r in range(R):
        for p in range(8):
            assert outs[r][p].tobytes() == base[p].tobytes()


@pytest.mark.parametrize("seed", range(10))
def test_against_the_definition_in_float64(seed):
    """out_p = (1/R) * sum over the replicas that used p, for globally used p;
    untouched otherwise; the bitmap is numpy's any() over the replica axis."""
    rng = np.random.default_rng(seed)
    n, R = int(rng.integers(1, 20)), int(rng.integers(1, 6))
    numel = [int(x) for x in rng.integers(0, 300, size=n)]
    reps = [[workloads.gaussian_grad(30 + seed, r, 0, p, numel[p], 1.0) for p in range(n)] for r in range(R)]
    used = rng.integers(0, 2, size=(R, n))
    marked = [int(p) for p in rng.permutation(n)][: int(rng.integers(0, n + 1))]
    marks = [(p, used[:, p].tolist()) for p in marked]
    eff = np.zeros((R, n), dtype=bool)
    for p in marked:
        eff[:, p] = used[:, p] != 0
    for find_unused in (True, False):
        outs, _, _, glob = oracle.synchronize_local(numel, [FP32] * n, int(rng.integers(0, 2000)), reps, marks, find_unused)
        assert glob.tolist() == eff.any(axis=0).astype(int).tolist()
        for p in range(n):
            exact = sum(reps[r][p].astype(np.float64) for r in range(R) if eff[r, p]) / R if eff[:, p].any() else None
            for r in range(R):
                if exact is not None:
                    assert np.allclose(outs[r][p], exact, rtol=1e-6, atol=1e-7)
                elif find_unused:
                    assert outs[r][p].tobytes() == reps[r][p].tobytes()
                else:
                    assert outs[r][p].tobytes() == np.zeros(numel[p], np.float32).tobytes()


def test_unused_replicas_are_not_read():
    numel = [50, 7, 300]
    R = 3
    reps = [[workloads.gaussian_grad(40, r, 0, p, numel[p], 1.0) for p in range(3)] for r in range(R)]
    clean, _, _, _ = oracle.synchronize_local(numel, [FP32] * 3, 256, reps,
                                              [(2, [1, 0, 1]), (1, [0, 0, 0]), (0, [0, 1, 0])])
    reps[1][2][:] = np.nan
    reps[0][0][:] = np.nan
    reps[2][0][:] = np.nan
    outs, _, _, _ = oracle.synchronize_local(numel, [FP32] * 3, 256, reps,
                                             [(2, [1, 0, 1]), (1, [0, 0, 0]), (0, [0, 1, 0])])
    for r in range(R):
        assert outs[r][2].tobytes() == clean[r][2].tobytes()
        assert outs[r][0].tobytes() == clean[r][0].tobytes()
        assert np.isfinite(outs[r][2]).all() and np.isfinite(outs[r][0]).all()


def test_participation_accumulates_across_no_sync_iterations():
    """A parameter used only in an earlier no_sync iteration still counts as
    used when the next synchronization takes place."""
    numel = [4, 4]
    R = 2
    reps = [[np.full(4, 1.0 + r, np.float32), np.full(4, 10.0 + r, np.float32)] for r in range(R)]
    prior = np.array([[0, 1], [0, 0]], dtype=np.uint8)       # replica 0 used p1 during no_sync
    outs, _, _, glob = oracle.synchronize_local(numel, [FP32] * 2, 1 << 20, reps, [(0, [1, 1])], True, prior)
    assert glob.tolist() == [1, 1]
    assert outs[0][1].tolist() == [5.0] * 4          # (10 + 0) / 2: replica 1 contributes zeros
    assert outs[1][0].tolist() == [1.5] * 4
