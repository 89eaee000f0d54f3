"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle
on the same seeded inputs.  Indexing (assignment, pack, unpack) must be
bit-exact; reductions must stay within 1e-6 (fp32) / 1e-3 (fp16, bf16) of the
oracle relative to max(|oracle|, mean_r |x_r|) -- and, because both sides add
in the same order, are also expected to agree bit for bit, which is asserted
separately so that a failure tells which bar was missed."""
import numpy as np
import pytest

import oracle
import workloads

pytestmark = pytest.mark.gpu

FP32, FP16, BF16 = 0, 1, 2
TOL = {FP32: 1e-6, FP16: 1e-3, BF16: 1e-3}
STAGED, FUSED = 0, 1


def lib():
    import paper_2006_15704_amd as d
    from paper_2006_15704_amd import harness
    return d, harness


def assert_close(got, want, reps_p, dtype, what):
    """spec tolerance, then bit equality (NaN == NaN, -0 == +0)."""
    g = oracle.to_f32(got, dtype).astype(np.float64)
    w = oracle.to_f32(want, dtype).astype(np.float64)
    scale = np.zeros_like(w)
    for x in reps_p:
        scale += np.abs(oracle.to_f32(x, dtype).astype(np.float64))
    scale /= len(reps_p)
    both_nan = np.isnan(g) & np.isnan(w)
    with np.errstate(invalid="ignore"):
        bad = ~both_nan & ~(np.abs(g - w) <= TOL[dtype] * np.maximum(np.abs(w), scale))
        bad &= ~((g == w))          # covers equal infinities
    assert not bad.any(), f"{what}: {int(bad.sum())} elements outside tolerance"
    same = both_nan | (g == w)
    assert same.all(), f"{what}: {int((~same).sum())} elements differ in bits"


def run_sync(numel, dtypes, reps, cap, pipeline, order=None, skew=None, replica_skew=None,
             write_all=False, one_by_one=False, same_stream=False, check_flat=True, options=()):
    d, harness = lib()
    R = len(reps)
    grads = harness.DeviceGrads(numel, dtypes, R, skew=skew, replica_skew=replica_skew, fill=0xFF)
    for r in range(R):
        grads.upload_replica(r, reps[r])
    want, asg, wlog = oracle.synchronize(numel, dtypes, cap, reps, order)
    with harness.Session(grads, cap, pipeline, write_all, same_stream) as s:
        for opt, val in options:
            d.ddp_set_option(s.ctx, opt, val)
        assert s.n_buckets == len(asg.buckets)
        bucket_of, offset = d.ddp_get_assignment(s.ctx, len(numel))
        assert bucket_of.tolist() == asg.bucket_of.tolist()
        assert offset.tolist() == asg.offset_of.tolist()
        s.sync(order, one_by_one=one_by_one)
        assert d.ddp_get_launch_log(s.ctx, 1) == wlog
        if pipeline == STAGED and check_flat:
            marked = set(range(len(numel))) if order is None else set(order)
            unused = [i for i in range(len(numel)) if i not in marked]
            for b in range(s.n_buckets):
                for r in range(R):
                    flat = s.bucket_bytes(b, r)
                    assert flat.tobytes() == oracle.pack_bucket(asg, b, reps[r], unused).tobytes(), \
                        f"flat bucket {b} replica {r}"
        outs = [[grads.download(r, i) for i in range(len(numel))] for r in range(R if write_all else 1)]
        others = [[grads.download(r, i) for i in range(len(numel))] for r in range(1, R)] if not write_all else []
    for rr, out_r in enumerate(outs):
        for i in range(len(numel)):
            assert_close(out_r[i], want[i], [reps[r][i] for r in range(R)], dtypes[i],
                         f"param {i} replica {rr}")
    return outs, others, want


def gaussian_reps(config_id, numel, R, sigma, dtype=FP32):
    return [workloads.gaussian_replica(config_id, r, 0, numel, sigma, dtype) for r in range(R)]


# ---- config 1: Tiny ----------------------------------------------------------------
@pytest.mark.parametrize("pipeline", [STAGED, FUSED])
def test_tiny_config(pipeline):
    numel = workloads.numel_of(workloads.tiny_shapes())
    reps = gaussian_reps(1, numel, 2, 1.0)
    outs, others, _ = run_sync(numel, [FP32] * 8, reps, 16384, pipeline, one_by_one=True)
    if pipeline == FUSED:
        return
    # W = 1: the other replicas' gradients are inputs only and stay untouched
    for r, row in enumerate(others, start=1):
        for i in range(8):
            assert row[i].tobytes() == reps[r][i].tobytes()


@pytest.mark.parametrize("pipeline", [STAGED, FUSED])
def test_tiny_linear_regression_mean_gradient(pipeline):
    X, w, b, y = workloads.linear_regression_problem(1)
    full_w = 2.0 / 64 * (X.T @ (X @ w + b - y))
    full_b = 2.0 / 64 * (X @ w + b - y).sum()
    reps = []
    for r in range(2):
        sl = slice(r * 32, (r + 1) * 32)
        res = X[sl] @ w + b - y[sl]
        reps.append([(2.0 / 32 * (X[sl].T @ res)).astype(np.float32),
                     np.array([2.0 / 32 * res.sum()], dtype=np.float32)])
    outs, _, _ = run_sync([16, 1], [FP32, FP32], reps, 25 << 20, pipeline)
    assert np.allclose(outs[0][0], full_w, rtol=1e-6, atol=1e-7)
    assert np.allclose(outs[0][1], full_b, rtol=1e-6, atol=1e-7)


# ---- indexing: tags, alignments, odd sizes ----------------------------------------------
@pytest.mark.parametrize("pipeline", [STAGED, FUSED])
@pytest.mark.parametrize("dtype", [FP32, FP16, BF16])
@pytest.mark.parametrize("cap", [0, 1000, 16384, oracle.CAP_WHOLE_MODEL])
def test_single_replica_round_trip_is_identity(pipeline, dtype, cap):
    numel = workloads.numel_of(workloads.tiny_shapes()) + [0, 1, 3, 4099, 7]
    starts = np.concatenate([[0], np.cumsum(numel)[:-1]])
    reps = [[workloads.tag_grad(0, int(s), int(n), dtype) for s, n in zip(starts, numel)]]
    outs, _, _ = run_sync(numel, [dtype] * len(numel), reps, cap, pipeline)
    for i in range(len(numel)):
        assert outs[0][i].tobytes() == reps[0][i].tobytes()


@pytest.mark.parametrize("pipeline", [STAGED, FUSED])
@pytest.mark.parametrize("dtype", [FP32, FP16])
def test_unaligned_gradient_pointers(pipeline, dtype):
    """Tensors that start at every element-aligned offset modulo 16 bytes,
    different per replica, with lengths around the vector and tile sizes."""
    es = 4 if dtype == FP32 else 2
    numel = [1, 2, 3, 5, 8, 13, 2047, 2048, 2049, 4095, 4096, 4097, 8191, 8193, 20000, 33, 64, 1023, 9000]
    skew = [(i * es) % 16 for i in range(len(numel))]
    R = 3
    replica_skew = [0, es, 3 * es]
    reps = gaussian_reps(11, numel, R, 1e-2, dtype)
    for write_all in (False, True):
        run_sync(numel, [dtype] * len(numel), reps, 20000, pipeline, skew=skew,
                 replica_skew=replica_skew, write_all=write_all)


@pytest.mark.parametrize("pipeline", [STAGED, FUSED])
def test_mixed_element_types(pipeline):
    numel = [100, 257, 4100, 33, 64, 9]
    dtypes = [FP32, FP16, FP16, BF16, FP32, FP32]
    R = 4
    reps = [[workloads.gaussian_grad(12, r, 0, p, n, 1e-2, dt) for p, (n, dt) in enumerate(zip(numel, dtypes))]
            for r in range(R)]
    run_sync(numel, dtypes, reps, 1 << 20, pipeline)


@pytest.mark.parametrize("dtype", [FP32, FP16, BF16])
def test_kernel_variants_give_the_same_bits(dtype):
    """Coalesced and single launches, with hinted and plain loads, under every
    cap on resident blocks, on a list that mixes large, tiny, unaligned and
    unmarked tensors."""
    d, _ = lib()
    es = 4 if dtype == FP32 else 2
    numel = [70000, 3, 2048, 4096, 12289, 1, 40000, 64, 9999]
    skew = [0, es, 0, 0, 2 * es, 0, 0, 3 * es, 0]
    R = 5
    reps = gaussian_reps(13, numel, R, 1e-2, dtype)
    order = [8, 7, 6, 4, 3, 2, 0]          # parameters 5 and 1 never marked
    for coalesce in (1 << 62, 0):
        for nt in (1, 0):
            opts = [(d.DDP_OPT_NONTEMPORAL, nt), (d.DDP_OPT_COALESCE, coalesce),
                    # occupancy cap of the reduce kernels: none, one block per unit (the largest
                    # LDS allocation), three
                    (d.DDP_OPT_REDUCE_CAP_MIN_BYTES, 0),
                    (d.DDP_OPT_REDUCE_BLOCKS_PER_CU, (0 if nt else 1) if coalesce else 3)]
            for pipeline in (STAGED, FUSED):
                run_sync(numel, [dtype] * len(numel), reps, 1 << 22, pipeline, order=order, skew=skew,
                         options=opts, write_all=(nt == 0))


# ---- reductions -----------------------------------------------------------------------------
@pytest.mark.parametrize("pipeline", [STAGED, FUSED])
@pytest.mark.parametrize("R", [1, 2, 3, 5, 7, 8, 12, 16, 31, 32, 64])
def test_replica_counts_fp32(pipeline, R):
    numel = [5000, 17, 4096, 1]
    reps = gaussian_reps(20 + R, numel, R, 1e-2)
    run_sync(numel, [FP32] * 4, reps, 8192, pipeline)


@pytest.mark.parametrize("pipeline", [STAGED, FUSED])
@pytest.mark.parametrize("dtype", [FP16, BF16])
@pytest.mark.parametrize("R", [2, 3, 16])
def test_replica_counts_16bit(pipeline, dtype, R):
    numel = [5000, 17, 8192, 1]
    reps = gaussian_reps(40 + R, numel, R, 1e-2, dtype)
    run_sync(numel, [dtype] * 4, reps, 8192, pipeline)


@pytest.mark.parametrize("pipeline", [STAGED, FUSED])
@pytest.mark.parametrize("R", [3, 8])
def test_integer_inputs_equal_exact_arithmetic(pipeline, R):
    numel = [4097, 300]
    reps = [[workloads.integer_grad(3, r, 0, p, n, 100_000) for p, n in enumerate(numel)] for r in range(R)]
    outs, _, _ = run_sync(numel, [FP32] * 2, reps, 1 << 20, pipeline)
    for p in range(2):
        total = sum(reps[r][p].astype(np.int64) for r in range(R))
        assert (outs[0][p] == (total / R).astype(np.float32)).all()


@pytest.mark.parametrize("pipeline", [STAGED, FUSED])
def test_fp16_every_bit_pattern_with_partner(pipeline):
    """All 65,536 fp16 patterns (subnormals, infinities, NaNs) averaged with a
    fixed partner, and alone (R = 1 must hand finite values back unchanged)."""
    bits = np.arange(65536, dtype=np.uint16).view(np.float16)
    partner = np.full(65536, np.float16(0.3711), dtype=np.float16)
    run_sync([65536], [FP16], [[bits], [partner]], 1 << 20, pipeline, check_flat=False)
    outs, _, _ = run_sync([65536], [FP16], [[bits]], 1 << 20, pipeline, check_flat=False)
    finite = np.isfinite(bits)
    assert (outs[0][0].view(np.uint16)[finite] == bits.view(np.uint16)[finite]).all()


@pytest.mark.parametrize("pipeline", [STAGED, FUSED])
def test_bf16_rounding_ties_and_specials(pipeline):
    """Sums that land exactly on bf16 rounding ties: x = k + 0.5 ulp patterns
    built from two bf16 addends, plus infinities and NaN."""
    hi = np.arange(0, 65536, dtype=np.uint16)
    a = hi                                   # every bf16 pattern
    b = (hi & np.uint16(0xFF80))             # same exponent, zero mantissa: sum doubles/rounds
    c = np.full(65536, 0x3B80, dtype=np.uint16)   # 2^-8
    run_sync([65536], [BF16], [[a], [b], [c]], 1 << 20, pipeline, check_flat=False)
    run_sync([65536], [BF16], [[a], [c]], 1 << 20, pipeline, check_flat=False)


@pytest.mark.parametrize("pipeline", [STAGED, FUSED])
def test_nonfinite_and_signed_zero(pipeline):
    x = np.array([np.inf, np.nan, 1.0, -np.inf, -0.0, -0.0, 1e-45, 3e38], dtype=np.float32)
    y = np.array([1.0, 1.0, np.inf, np.inf, -0.0, 0.0, 1e-45, 3e38], dtype=np.float32)
    outs, _, want = run_sync([8], [FP32], [[x], [y]], 1 << 20, pipeline)
    assert np.signbit(outs[0][0][4]) == np.signbit(want[0][4])    # -0 + -0 stays -0
    assert outs[0][0][6] == want[0][6] and want[0][6] > 0           # subnormals are not flushed


# ---- ready order, launch order, absent gradients, iterations ----------------------------
@pytest.mark.parametrize("pipeline", [STAGED, FUSED])
@pytest.mark.parametrize("seed", range(4))
def test_random_ready_orders_with_unmarked_parameters(pipeline, seed):
    rng = np.random.default_rng(seed)
    n = 40
    numel = [int(x) for x in rng.integers(1, 3000, size=n)]
    R = 4
    reps = gaussian_reps(60 + seed, numel, R, 1e-2)
    order = [int(p) for p in rng.permutation(n)]
    never = sorted(order[n - 6:]) if seed % 2 else []
    order = order[: n - 6] if seed % 2 else order
    for r in range(R):
        for p in never:
            reps[r][p][:] = np.nan          # must not be read
    outs, _, _ = run_sync(numel, [FP32] * n, reps, 10000, pipeline, order=order,
                          write_all=bool(seed & 2), one_by_one=True)
    for row in outs:
        for p in never:
            assert row[p].tobytes() == np.zeros(numel[p], np.float32).tobytes()


@pytest.mark.parametrize("pipeline", [STAGED, FUSED])
def test_two_iterations_replenish_pending_counts(pipeline):
    d, harness = lib()
    numel = workloads.numel_of(workloads.tiny_shapes())
    R = 2
    grads = harness.DeviceGrads(numel, [FP32] * 8, R)
    with harness.Session(grads, 16384, pipeline) as s:
        for it, order in enumerate([[7, 6, 5, 4, 3, 2, 1, 0], [0, 1, 2, 3, 4, 5, 6, 7], [7, 6, 5, 4]]):
            reps = [workloads.gaussian_replica(70 + it, r, 0, numel, 1.0) for r in range(R)]
            for r in range(R):
                grads.upload_replica(r, reps[r])
            want, asg, wlog = oracle.synchronize(numel, [FP32] * 8, 16384, reps, order)
            s.sync(order, one_by_one=True)
            assert d.ddp_get_launch_log(s.ctx, 1) == wlog
            for i in range(8):
                assert grads.download(0, i).tobytes() == want[i].tobytes()
        with pytest.raises(d.DdpError) as e:
            d.ddp_mark_ready(s.ctx, 3)
            d.ddp_mark_ready(s.ctx, 3)
        assert e.value.code == d.DDP_ERR_ALREADY_READY
        d.ddp_finalize_backward(s.ctx)
        d.ddp_synchronize(s.ctx)


# ---- no_sync -------------------------------------------------------------------------------
@pytest.mark.parametrize("pipeline", [STAGED, FUSED])
@pytest.mark.parametrize("dtype", [FP32, FP16, BF16])
def test_no_sync_accumulation_then_one_reduction(pipeline, dtype):
    d, harness = lib()
    numel = workloads.numel_of(workloads.tiny_shapes()) + [4099]
    n, R, K = len(numel), 3, 4
    dts = [dtype] * n
    grads = harness.DeviceGrads(numel, dts, R, fill=0)
    micro_dev = harness.DeviceGrads(numel, dts, R, skew=[(i * 2 * (2 if dtype else 4)) % 16 for i in range(n)])
    acc = [[np.zeros(x, dtype=oracle.STORAGE[dtype]) for x in numel] for _ in range(R)]
    skipped = {1: [2, 5]}          # micro-step 1 produces no gradient for parameters 2 and 5
    with harness.Session(grads, 16384, pipeline) as s:
        for k in range(K):
            micro = [workloads.gaussian_replica(80, r, k, numel, 1e-2, dtype) for r in range(R)]
            ptrs = []
            for r in range(R):
                row = list(micro[r])
                for p in skipped.get(k, []):
                    row[p] = None
                oracle.accumulate(acc[r], row, dts)
                for p in range(n):
                    if row[p] is not None:
                        micro_dev.upload(r, p, row[p])
                ptrs += [None if row[p] is None else micro_dev.ptr(r, p) for p in range(n)]
            d.ddp_no_sync_accumulate(s.ctx, ptrs)
            d.ddp_synchronize(s.ctx)
            assert d.ddp_get_launch_log(s.ctx, 0) == []         # no reduction was launched
        for r in range(R):
            for p in range(n):
                assert grads.download(r, p).tobytes() == acc[r][p].tobytes(), f"accumulator r{r} p{p}"
        want, _, _ = oracle.synchronize(numel, dts, 16384, acc)
        s.sync()
        assert d.ddp_get_used_map(s.ctx, n, 1).tolist() == [1] * n
        for p in range(n):
            assert grads.download(0, p).tobytes() == want[p].tobytes()


# ---- overlap plumbing: the reduction must wait for the backward stream ------------------
@pytest.mark.parametrize("pipeline", [STAGED, FUSED])
@pytest.mark.parametrize("tail_on_backward", [1, 0])
def test_reduction_waits_for_gradients_produced_on_the_backward_stream(pipeline, tail_on_backward):
    """Gradient memory starts as NaN; the synthetic backward stream writes the
    real gradients after a delay, parameter by parameter, and marks them ready.
    Any reduction that ran ahead of its inputs would average NaNs."""
    d, harness = lib()
    numel = workloads.numel_of(workloads.tiny_shapes())
    R = 2
    reps = [workloads.gaussian_replica(90, r, 0, numel, 1.0) for r in range(R)]
    grads = harness.DeviceGrads(numel, [FP32] * 8, R, fill=0xFF)
    src = harness.DeviceGrads(numel, [FP32] * 8, R)
    for r in range(R):
        src.upload_replica(r, reps[r])
    want, _, _ = oracle.synchronize(numel, [FP32] * 8, 16384, reps)
    with harness.Session(grads, 16384, pipeline) as s:
        d.ddp_set_option(s.ctx, d.DDP_OPT_TAIL_ON_BACKWARD, tail_on_backward)
        order = list(range(7, -1, -1))
        d.ddp_synth_backward(s.ctx, order, [200_000] * 8, src.ptrs(), True)
        d.ddp_finalize_backward(s.ctx)
        d.ddp_synchronize(s.ctx)
        for i in range(8):
            assert grads.download(0, i).tobytes() == want[i].tobytes()


# ---- degenerate and extreme shapes ------------------------------------------------------------
@pytest.mark.parametrize("pipeline", [STAGED, FUSED])
@pytest.mark.parametrize("numel", [[0, 0, 0], [1], [0, 5, 0], [0], [16, 0, 0, 16]])
def test_empty_and_single_element_tensors(pipeline, numel):
    R = 3
    reps = gaussian_reps(14, numel, R, 1.0)
    for cap in (0, 64, oracle.CAP_WHOLE_MODEL):
        run_sync(numel, [FP32] * len(numel), reps, cap, pipeline, one_by_one=True)


@pytest.mark.parametrize("pipeline", [STAGED, FUSED])
def test_many_small_parameters_with_the_largest_replica_count(pipeline):
    """3000 tensors of 0..700 elements, R = 64 (the library's maximum), a cap
    that gives hundreds of buckets, a random ready order and 5 % of the
    parameters never marked."""
    rng = np.random.default_rng(15)
    n, R = 3000, 64
    numel = [int(x) for x in rng.integers(0, 700, size=n)]
    reps = gaussian_reps(15, numel, R, 1e-2)
    order = [int(p) for p in rng.permutation(n)][: n - 150]
    run_sync(numel, [FP32] * n, reps, 16384, pipeline, order=order, check_flat=False)


# ---- coalesced launches --------------------------------------------------------------------------
@pytest.mark.parametrize("pipeline", [STAGED, FUSED])
def test_coalesced_launches_keep_order_results_and_cover_every_bucket(pipeline):
    """DDP_OPT_COALESCE: buckets completed inside one call go out as one launch
    per run of equal element type.  Same launch log, same bits; the launch ids
    of the timed kernels decode to a partition of the buckets."""
    d, harness = lib()
    numel = [300, 5000, 64, 4096, 9000, 33, 2048, 100, 7000, 12]
    dtypes = [FP32, FP32, FP32, FP16, FP16, FP16, FP32, FP32, BF16, BF16]
    n, R, cap = len(numel), 4, 8192
    reps = [[workloads.gaussian_grad(16, r, 0, p, numel[p], 1e-2, dtypes[p]) for p in range(n)] for r in range(R)]
    order = [9, 8, 7, 6, 4, 3, 2, 1, 0]           # parameter 5 is never marked
    want, asg, wlog = oracle.synchronize(numel, dtypes, cap, reps, order)
    grads = harness.DeviceGrads(numel, dtypes, R)
    for r in range(R):
        grads.upload_replica(r, reps[r])
    with harness.Session(grads, cap, pipeline) as s:
        d.ddp_set_option(s.ctx, d.DDP_OPT_COALESCE, 1 << 62)
        d.ddp_set_option(s.ctx, d.DDP_OPT_TIMING, 1)
        d.ddp_mark_ready_many(s.ctx, order[:5])
        d.ddp_mark_ready_many(s.ctx, order[5:])
        d.ddp_finalize_backward(s.ctx)
        d.ddp_synchronize(s.ctx)
        assert d.ddp_get_launch_log(s.ctx, 1) == wlog
        _, ids = d.ddp_get_kernel_times(s.ctx, d.DDP_K_REDUCE)
        covered = []
        for ident in ids:
            first, extra = int(ident) % 65536, int(ident) // 65536
            covered += list(range(first, first + extra + 1))
            assert len({asg.buckets[b].dtype for b in range(first, first + extra + 1)}) == 1
        assert covered == list(range(len(asg.buckets)))
        assert len(ids) < len(asg.buckets)          # something was in fact coalesced
    for p in range(n):
        assert grads.download(0, p).tobytes() == want[p].tobytes(), f"parameter {p}"


# ---- kernel time stamps ------------------------------------------------------------------------
@pytest.mark.gpu
@pytest.mark.parametrize("pipeline", [STAGED, FUSED])
def test_kernel_time_stamps_cover_every_launch_and_are_plausible(pipeline):
    """DDP_OPT_TIMING = 1: every pack / reduce / unpack / accumulate launch carries its own pair of
    time stamps.  Durations are positive and far below the wall time of the whole step, their number
    matches the launches, and the results are the ones without timing."""
    import time
    d, harness = lib()
    numel = [1 << 20, 300, 1 << 18, 5000, 1 << 19]
    n, R, cap = len(numel), 4, 1 << 21
    dtypes = [FP32] * n
    reps = gaussian_reps(21, numel, R, 1e-2)
    micro = gaussian_reps(22, numel, R, 1e-2)
    acc = [list(reps[r]) for r in range(R)]
    for r in range(R):
        oracle.accumulate(acc[r], micro[r], dtypes)
    want, asg, _ = oracle.synchronize(numel, dtypes, cap, acc)
    grads = harness.DeviceGrads(numel, dtypes, R)
    mg = harness.DeviceGrads(numel, dtypes, R)
    for r in range(R):
        grads.upload_replica(r, reps[r])
        mg.upload_replica(r, micro[r])
    with harness.Session(grads, cap, pipeline) as s:
        d.ddp_set_option(s.ctx, d.DDP_OPT_COALESCE, 0)
        d.ddp_set_option(s.ctx, d.DDP_OPT_TIMING, 1)
        d.ddp_synchronize(s.ctx)
        t0 = time.perf_counter()
        d.ddp_no_sync_accumulate(s.ctx, mg.ptrs())
        for p in range(n - 1, -1, -1):
            d.ddp_mark_ready(s.ctx, p)
        d.ddp_finalize_backward(s.ctx)
        d.ddp_synchronize(s.ctx)
        wall_ms = (time.perf_counter() - t0) * 1e3
        nb = len(asg.buckets)
        expect = {d.DDP_K_ACCUMULATE: 1, d.DDP_K_REDUCE: nb,
                  d.DDP_K_PACK: nb if pipeline == STAGED else 0, d.DDP_K_UNPACK: 1 if pipeline == STAGED else 0}
        for kind, count in expect.items():
            ms, ids = d.ddp_get_kernel_times(s.ctx, kind)
            assert len(ms) == count, f"kind {kind}: {len(ms)} timed launches, expected {count}"
            assert np.all(ms > 0.0) and np.all(ms < wall_ms), f"kind {kind}: durations {ms} ms, wall {wall_ms} ms"
            if count == nb:
                assert ids.tolist() == list(range(nb))
        outs = [grads.download(0, i) for i in range(n)]
    for i in range(n):
        assert outs[i].tobytes() == want[i].tobytes(), f"parameter {i}"


# ---- several reduction streams -----------------------------------------------------------------
@pytest.mark.parametrize("pipeline", [STAGED, FUSED])
@pytest.mark.parametrize("streams", [2, 3, 8])
def test_round_robin_reduction_streams_give_the_same_results(pipeline, streams):
    """DDP_OPT_REDUCE_STREAMS (the one-GPU form of Section 3.3's round-robin
    process groups): same launch log, same bits, for ready marks given one at
    a time, with never-marked parameters, and with coalesced launches."""
    d, _ = lib()
    rng = np.random.default_rng(17)
    n, R = 60, 4
    numel = [int(x) for x in rng.integers(0, 6000, size=n)]
    reps = gaussian_reps(17, numel, R, 1e-2)
    order = [int(p) for p in rng.permutation(n)][: n - 5]
    for extra in ((), ((d.DDP_OPT_COALESCE, 40000),), ((d.DDP_OPT_TIMING, 1),), ((d.DDP_OPT_TIMING, 2),),
                  ((d.DDP_OPT_TAIL_ON_BACKWARD, 0),), ((d.DDP_OPT_TAIL_ON_BACKWARD, 0), (d.DDP_OPT_TIMING, 2))):
        run_sync(numel, [FP32] * n, reps, 12000, pipeline, order=order, one_by_one=not extra,
                 write_all=True, options=((d.DDP_OPT_REDUCE_STREAMS, streams),) + extra)


@pytest.mark.parametrize("pipeline", [STAGED, FUSED])
@pytest.mark.parametrize("same_stream", [False, True])
def test_round_robin_streams_wait_for_the_backward_stream(pipeline, same_stream):
    """Gradient memory starts as NaN and is written by the synthetic backward
    stream after a delay; every reduction stream has to wait for it, over
    several iterations enqueued without host synchronization in between."""
    d, harness = lib()
    numel = workloads.numel_of(workloads.tiny_shapes()) + [5000, 300, 4096, 77]
    n, R, cap = len(numel), 3, 4096
    grads = harness.DeviceGrads(numel, [FP32] * n, R, fill=0xFF)
    srcs, wants = [], []
    for it in range(3):
        reps = [workloads.gaussian_replica(91 + it, r, 0, numel, 1.0) for r in range(R)]
        src = harness.DeviceGrads(numel, [FP32] * n, R)
        for r in range(R):
            src.upload_replica(r, reps[r])
        srcs.append(src)
        wants.append(oracle.synchronize(numel, [FP32] * n, cap, reps)[0])
    keep = harness.DeviceGrads(numel, [FP32] * n, 3, fill=0)       # copies of each iteration's result
    import torch
    with harness.Session(grads, cap, pipeline, same_stream=same_stream) as s:
        d.ddp_set_option(s.ctx, d.DDP_OPT_REDUCE_STREAMS, 4)
        order = list(range(n - 1, -1, -1))
        for it in range(3):
            d.ddp_synth_backward(s.ctx, order, [100_000] * n, srcs[it].ptrs(), True)
            d.ddp_finalize_backward(s.ctx)
            # work enqueued on the backward stream after finalize sees the averaged gradients
            with torch.cuda.stream(s.backward_stream):
                keep.bufs[it].copy_(grads.bufs[0], non_blocking=True)
        d.ddp_synchronize(s.ctx)
        torch.cuda.synchronize()
        for it in range(3):
            for i in range(n):
                assert keep.download(it, i).tobytes() == wants[it][i].tobytes(), f"iteration {it} parameter {i}"


# ---- graph capture ------------------------------------------------------------------------------
@pytest.mark.parametrize("two_streams", [False, True])
def test_a_captured_step_replays_correctly(two_streams):
    """One whole step (ready marks + finalize, fused pipeline) captured into a
    HIP graph on the backward stream and replayed on new gradients several
    times, with eager work and synchronizations between the replays; every
    replay is compared with the oracle.  With two_streams the buckets are
    launched one call at a time, so all but the last go to the reduction
    stream and the capture forks and joins across streams."""
    import torch
    d, harness = lib()
    numel = workloads.numel_of(workloads.tiny_shapes()) + [9000, 2048, 77]
    n, R, cap = len(numel), 3, 16384
    grads = harness.DeviceGrads(numel, [FP32] * n, R)
    order = list(range(n - 1, -1, -1))
    with harness.Session(grads, cap, FUSED) as s:
        reps = gaussian_reps(95, numel, R, 1.0)
        for r in range(R):
            grads.upload_replica(r, reps[r])
        s.sync()                                   # an eager step first (also builds every lazy resource)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=s.backward_stream):
            if two_streams:
                for p in order:
                    d.ddp_mark_ready(s.ctx, p)
            else:
                d.ddp_mark_ready_many(s.ctx, order)
            d.ddp_finalize_backward(s.ctx)
        torch.cuda.synchronize()
        for it in range(4):
            reps = gaussian_reps(96 + it, numel, R, 1.0)
            for r in range(R):
                grads.upload_replica(r, reps[r])
            torch.cuda.synchronize()
            want, _, _ = oracle.synchronize(numel, [FP32] * n, cap, reps)
            g.replay()
            torch.cuda.synchronize()
            for i in range(n):
                assert grads.download(0, i).tobytes() == want[i].tobytes(), f"replay {it} parameter {i}"
        del g
