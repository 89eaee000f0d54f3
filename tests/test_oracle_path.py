"""Pins for the oracle's pack / unpack / whole-path functions, the
mean-gradient identity, no_sync accumulation and unused parameters."""
import numpy as np
import pytest

import oracle
import workloads

FP32, FP16, BF16 = oracle.DT_FP32, oracle.DT_FP16, oracle.DT_BF16
U = 2.0 ** -24


def tag_replica(r, numel, dtype):
    starts = np.concatenate([[0], np.cumsum(numel)[:-1]])
    return [workloads.tag_grad(r, int(s), int(n), dtype) for s, n in zip(starts, numel)]


# ---- pack / unpack ---------------------------------------------------------
@pytest.mark.parametrize("dtype", [FP32, FP16, BF16])
def test_pack_is_concatenation_in_fill_order(dtype):
    numel = workloads.numel_of(workloads.tiny_shapes())
    asg = oracle.assign_buckets(numel, [dtype] * 8, 16384)
    grads = tag_replica(0, numel, dtype)
    for b, bk in enumerate(asg.buckets):
        flat = oracle.pack_bucket(asg, b, grads)
        want = np.concatenate([grads[p] for p in range(max(bk.params), min(bk.params) - 1, -1)])
        assert flat.tobytes() == want.tobytes()


@pytest.mark.parametrize("dtype", [FP32, FP16, BF16])
@pytest.mark.parametrize("cap", [0, 100, 16384, oracle.CAP_WHOLE_MODEL])
def test_single_replica_round_trip_is_identity(dtype, cap):
    """R = 1: pack, x / 1, unpack must hand every gradient back bit for bit."""
    numel = workloads.numel_of(workloads.tiny_shapes()) + [0, 1, 3]
    grads = tag_replica(0, numel, dtype)
    outs, asg, log = oracle.synchronize(numel, [dtype] * len(numel), cap, [grads])
    for g, o in zip(grads, outs):
        assert o.dtype == g.dtype and o.tobytes() == g.tobytes()
    assert [b for b, _ in log] == list(range(len(asg.buckets)))


def test_unpack_reads_the_parameters_own_slot():
    numel = [5, 7, 3]
    asg = oracle.assign_buckets(numel, [FP32] * 3, 1 << 20)     # one bucket: 2, 1, 0
    avg = np.arange(15, dtype=np.float32)
    outs = [None] * 3
    oracle.unpack_bucket(asg, 0, avg, outs)
    assert outs[2].tolist() == [0, 1, 2]
    assert outs[1].tolist() == [3, 4, 5, 6, 7, 8, 9]
    assert outs[0].tolist() == [10, 11, 12, 13, 14]


# ---- the method equals the plain definition --------------------------------
@pytest.mark.parametrize("cap", [0, 16384, oracle.CAP_WHOLE_MODEL])
def test_tiny_config_against_float64_definition(cap):
    numel = workloads.numel_of(workloads.tiny_shapes())
    R = 2
    reps = [workloads.gaussian_replica(1, r, 0, numel, 1.0) for r in range(R)]
    outs, _, _ = oracle.synchronize(numel, [FP32] * 8, cap, reps)
    exact = oracle.mean_definition_f64(reps, [FP32] * 8)
    gamma = R * U / (1 - R * U)
    for p in range(8):
        scale = sum(np.abs(reps[r][p].astype(np.float64)) for r in range(R)) / R
        assert (np.abs(outs[p].astype(np.float64) - exact[p]) <= gamma * scale).all()


def test_bucketing_does_not_change_values():
    numel = workloads.numel_of(workloads.tiny_shapes())
    reps = [workloads.gaussian_replica(1, r, 0, numel, 1.0) for r in range(5)]
    base, _, _ = oracle.synchronize(numel, [FP32] * 8, 0, reps)
    for cap in (64, 16384, oracle.CAP_WHOLE_MODEL):
        outs, _, _ = oracle.synchronize(numel, [FP32] * 8, cap, reps)
        for a, b in zip(base, outs):
            assert a.tobytes() == b.tobytes()
    order = [3, 0, 7, 1, 2, 6, 5, 4]
    outs, _, _ = oracle.synchronize(numel, [FP32] * 8, 16384, reps, order)
    for a, b in zip(base, outs):
        assert a.tobytes() == b.tobytes()


# ---- mathematical equivalence with local training (Section 3, opening) ------
def mse_grad(X, w, b, y):
    """Gradient of L = mean((X w + b - y)^2) in float64."""
    res = X @ w + b - y
    return 2.0 / len(y) * (X.T @ res), np.array([2.0 / len(y) * res.sum()])


def mse_loss(X, w, b, y):
    return float(np.mean((X @ w + b - y) ** 2))


def test_mean_of_shard_gradients_is_full_batch_gradient():
    """d = 16, batch 64 in R = 2 shards of 32: averaging the shard gradients
    of the mean-squared-error loss over the replicas gives the gradient of
    the loss over the whole batch.  Ground truth: closed form in float64,
    itself checked by central differences."""
    X, w, b, y = workloads.linear_regression_problem(1)
    gw, gb = mse_grad(X, w, b, y)
    h = 1e-6
    for j in range(16):
        e = np.zeros(16)
        e[j] = h
        fd = (mse_loss(X, w + e, b, y) - mse_loss(X, w - e, b, y)) / (2 * h)
        assert abs(fd - gw[j]) < 1e-6 * max(1.0, abs(gw[j]))
    fd = (mse_loss(X, w, b + h, y) - mse_loss(X, w, b - h, y)) / (2 * h)
    assert abs(fd - gb[0]) < 1e-6

    R = 2
    reps = []
    for r in range(R):
        sl = slice(r * 32, (r + 1) * 32)
        sw, sb = mse_grad(X[sl], w, b, y[sl])
        reps.append([sw.astype(np.float32), sb.astype(np.float32)])   # params: w [1,16], b [1]
    outs, _, _ = oracle.synchronize([16, 1], [FP32, FP32], 25 << 20, reps)
    assert np.allclose(outs[0], gw, rtol=1e-6, atol=1e-7)
    assert np.allclose(outs[1], gb, rtol=1e-6, atol=1e-7)
    # the sum (no division by R) or a single shard would be far off
    assert not np.allclose(reps[0][0] + reps[1][0], gw, rtol=1e-3)
    assert not np.allclose(reps[0][0], gw, rtol=1e-3)


# ---- no_sync (Section 3.2.4) -------------------------------------------------
@pytest.mark.parametrize("dtype", [FP32, FP16, BF16])
def test_accumulated_micro_steps_equal_sync_of_their_sum(dtype):
    numel = workloads.numel_of(workloads.tiny_shapes())
    R, K = 3, 4
    micro = [[workloads.gaussian_replica(5, r, k, numel, 1e-2, dtype) for r in range(R)] for k in range(K)]
    acc = [[np.zeros(n, dtype=oracle.STORAGE[dtype]) for n in numel] for _ in range(R)]
    for k in range(K):
        for r in range(R):
            oracle.accumulate(acc[r], micro[k][r], [dtype] * 8)
    got, _, _ = oracle.synchronize(numel, [dtype] * 8, 16384, acc)
    # the same sum formed separately, k ascending, rounding to storage each step
    summed = []
    for r in range(R):
        row = []
        for p in range(8):
            s = oracle.to_f32(np.zeros(numel[p], dtype=oracle.STORAGE[dtype]), dtype)
            for k in range(K):
                s = oracle.to_f32(oracle.from_f32(s + oracle.to_f32(micro[k][r][p], dtype), dtype), dtype)
            row.append(oracle.from_f32(s, dtype))
        summed.append(row)
    want, _, _ = oracle.synchronize(numel, [dtype] * 8, 16384, summed)
    for a, b in zip(got, want):
        assert a.tobytes() == b.tobytes()


def test_accumulation_with_integer_inputs_is_exact():
    numel = [33, 5, 64]
    R, K = 4, 4
    micro = [[[workloads.integer_grad(9, r, k, p, n, 1000) for p, n in enumerate(numel)]
              for r in range(R)] for k in range(K)]
    acc = [[np.zeros(n, dtype=np.float32) for n in numel] for _ in range(R)]
    for k in range(K):
        for r in range(R):
            oracle.accumulate(acc[r], micro[k][r], [FP32] * 3)
    got, _, _ = oracle.synchronize(numel, [FP32] * 3, 128, acc)
    for p in range(3):
        total = sum(micro[k][r][p].astype(np.int64) for k in range(K) for r in range(R))
        assert (got[p].astype(np.float64) == total / R).all()


def test_accumulate_skips_parameters_without_gradient():
    acc = [np.ones(4, np.float32), np.ones(2, np.float32)]
    oracle.accumulate(acc, [None, np.full(2, 2.0, np.float32)], [FP32, FP32])
    assert acc[0].tolist() == [1, 1, 1, 1] and acc[1].tolist() == [3, 3]


# ---- parameters that are never marked ready -----------------------------------
def test_unmarked_parameters_reduce_as_zeros_and_are_not_read():
    numel = workloads.numel_of(workloads.tiny_shapes())
    R = 2
    reps = [workloads.gaussian_replica(1, r, 0, numel, 1.0) for r in range(R)]
    unused = [5, 2]
    for r in range(R):
        for p in unused:
            reps[r][p][:] = np.nan
    order = [p for p in range(7, -1, -1) if p not in unused]
    outs, asg, log = oracle.synchronize(numel, [FP32] * 8, 16384, reps, order)
    for p in unused:
        assert outs[p].tobytes() == np.zeros(numel[p], np.float32).tobytes()   # +0 exactly
    full, _, _ = oracle.synchronize(numel, [FP32] * 8, 16384,
                                    [workloads.gaussian_replica(1, r, 0, numel, 1.0) for r in range(R)])
    for p in range(8):
        if p not in unused:
            assert outs[p].tobytes() == full[p].tobytes()
    assert log == [(0, 6), (1, 6), (2, 6)]


# ---- the pins do catch planted mistakes -----------------------------------------
def _tiny_problem():
    numel = workloads.numel_of(workloads.tiny_shapes())
    reps = [workloads.gaussian_replica(1, r, 0, numel, 1.0) for r in range(2)]
    return numel, reps


def test_planted_mistakes_are_caught(monkeypatch):
    numel, reps = _tiny_problem()
    exact = oracle.mean_definition_f64(reps, [FP32] * 8)
    import oracle.ddp_oracle as mod

    def close(outs):
        return all(np.allclose(o, e, rtol=1e-6, atol=1e-9) for o, e in zip(outs, exact))

    assert close(mod.synchronize(numel, [FP32] * 8, 16384, reps)[0])

    # (1) no division by R
    real_reduce = mod.reduce_average
    monkeypatch.setattr(mod, "reduce_average",
                        lambda flats, dt: (real_reduce(flats, dt) * np.float32(len(flats))).astype(np.float32))
    assert not close(mod.synchronize(numel, [FP32] * 8, 16384, reps)[0])
    monkeypatch.setattr(mod, "reduce_average", real_reduce)

    # (2) unpack with a shifted offset
    real_unpack = mod.unpack_bucket

    def bad_unpack(asg, b, avg, outs):
        real_unpack(asg, b, np.roll(avg, 1), outs)
    monkeypatch.setattr(mod, "unpack_bucket", bad_unpack)
    assert not close(mod.synchronize(numel, [FP32] * 8, 16384, reps)[0])
    monkeypatch.setattr(mod, "unpack_bucket", real_unpack)

    # (3) a replica dropped from the sum
    monkeypatch.setattr(mod, "reduce_average", lambda flats, dt: real_reduce(flats[:-1] + [np.zeros_like(flats[0])], dt))
    assert not close(mod.synchronize(numel, [FP32] * 8, 16384, reps)[0])
