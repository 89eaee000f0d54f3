"""GPU parity for per-replica participation and the global unused-parameter
bitmap (Section 3.2.3, last paragraph; Section 4.2 "Globally Unused
Parameters"): the HIP path, through the C ABI, against the oracle's
synchronize_local on the same seeded inputs.  Tensors of replicas that did not
use a parameter hold NaN patterns, so a kernel that read one of them, or a
mask applied to the wrong replica or parameter, poisons the result."""
import numpy as np
import pytest

import oracle
import workloads

pytestmark = pytest.mark.gpu

FP32, FP16, BF16 = 0, 1, 2
STAGED, FUSED = 0, 1
NAN_BITS = {FP32: np.float32(np.nan), FP16: np.float16(np.nan), BF16: np.uint16(0x7FC1)}


def lib():
    import paper_2006_15704_amd as d
    from paper_2006_15704_amd import harness
    return d, harness


def poison(arr, dtype):
    arr[...] = NAN_BITS[dtype]


def random_case(seed, n, R, dtype, max_numel, p_used=0.6, n_nobody=3, n_unmarked=3):
    """numel, dtypes, gradients, ready marks with masks; replicas whose final
    flag is 0 get NaN tensors."""
    rng = np.random.default_rng(seed)
    numel = [int(x) for x in rng.integers(0, max_numel, size=n)]
    numel[int(rng.integers(0, n))] = 3 * 2048 + 5          # several whole tiles and a ragged tail
    dtypes = [dtype] * n if dtype is not None else [int(x) for x in rng.integers(0, 3, size=n)]
    reps = [[workloads.gaussian_grad(500 + seed, r, 0, p, numel[p], 1e-2, dtypes[p]) for p in range(n)]
            for r in range(R)]
    order = [int(p) for p in rng.permutation(n)]
    unmarked = set(order[n - n_unmarked:]) if n_unmarked else set()
    order = order[: n - n_unmarked] if n_unmarked else order
    nobody = set(order[:n_nobody])
    marks = []
    for p in order:
        used = [0] * R if p in nobody else [int(rng.random() < p_used) for _ in range(R)]
        if p % 7 == 0 and p not in nobody:
            used = [1] * R
        marks.append((p, used))
    flag = np.zeros((R, n), dtype=np.uint8)
    for p, used in marks:
        flag[:, p] = used
    for r in range(R):
        for p in range(n):
            if not flag[r, p]:
                poison(reps[r][p], dtypes[p])
    return numel, dtypes, reps, marks, flag, {int(p) for p in np.flatnonzero(~flag.any(axis=0))}


def check_against_oracle(numel, dtypes, reps, marks, cap, pipeline, write_all, find_unused,
                         options=(), skew=None, replica_skew=None, use_plain_mark_for_full=True):
    d, harness = lib()
    n, R = len(numel), len(reps)
    want, asg, wlog, glob = oracle.synchronize_local(numel, dtypes, cap, reps, marks, find_unused=find_unused)
    grads = harness.DeviceGrads(numel, dtypes, R, skew=skew, replica_skew=replica_skew, fill=0xFF)
    for r in range(R):
        grads.upload_replica(r, reps[r])
    with harness.Session(grads, cap, pipeline, write_all) as s:
        d.ddp_set_option(s.ctx, d.DDP_OPT_FIND_UNUSED, 1 if find_unused else 0)
        for opt, val in options:
            d.ddp_set_option(s.ctx, opt, val)
        for p, used in marks:
            if all(used) and use_plain_mark_for_full:
                d.ddp_mark_ready(s.ctx, p)
            else:
                d.ddp_mark_ready_local(s.ctx, p, used)
        d.ddp_finalize_backward(s.ctx)
        d.ddp_synchronize(s.ctx)
        assert d.ddp_get_launch_log(s.ctx, 1) == wlog
        assert d.ddp_get_global_used(s.ctx, n).tolist() == glob.tolist()
        assert d.ddp_get_used_map(s.ctx, n, 1).tolist() == glob.tolist()
        written = range(R) if write_all else range(1)
        for r in range(R):
            for p in range(n):
                got = grads.download(r, p)
                if r in written:
                    assert got.tobytes() == want[r][p].tobytes(), f"replica {r} parameter {p}"
                else:       # W = 1: the other replicas' tensors are inputs only
                    assert got.tobytes() == reps[r][p].tobytes(), f"replica {r} parameter {p} was written"
    return want, glob


@pytest.mark.parametrize("pipeline", [STAGED, FUSED])
@pytest.mark.parametrize("write_all", [False, True])
@pytest.mark.parametrize("find_unused", [False, True])
@pytest.mark.parametrize("seed", range(3))
def test_partial_participation_matches_oracle(pipeline, write_all, find_unused, seed):
    R = [5, 8, 3][seed]
    numel, dtypes, reps, marks, flag, nobody = random_case(seed, 36, R, FP32, 5000)
    want, glob = check_against_oracle(numel, dtypes, reps, marks, 20000, pipeline, write_all, find_unused)
    assert sorted(p for p in range(len(numel)) if not glob[p]) == sorted(nobody)
    for p in range(len(numel)):
        if glob[p]:
            assert not np.isnan(want[0][p]).any()          # the case is built so that NaNs are never read
        elif find_unused:
            assert np.isnan(want[0][p]).all()              # kept as it was
        else:
            assert want[0][p].tobytes() == np.zeros(numel[p], np.float32).tobytes()


@pytest.mark.parametrize("pipeline", [STAGED, FUSED])
@pytest.mark.parametrize("dtype", [FP16, BF16, None])
def test_partial_participation_16bit_and_mixed_types(pipeline, dtype):
    numel, dtypes, reps, marks, _, _ = random_case(10 + (dtype or 0), 30, 6, dtype, 9000)
    check_against_oracle(numel, dtypes, reps, marks, 16384, pipeline, True, True)
    check_against_oracle(numel, dtypes, reps, marks, 16384, pipeline, False, False)


@pytest.mark.parametrize("pipeline", [STAGED, FUSED])
def test_partial_participation_with_misaligned_tensors(pipeline):
    """Tensors at different offsets modulo 16 bytes per parameter and per
    replica: masked replicas on the element-wise path and on tile edges."""
    n, R = 24, 4
    numel, dtypes, reps, marks, _, _ = random_case(20, n, R, FP32, 7000)
    skew = [(4 * i) % 16 for i in range(n)]
    check_against_oracle(numel, dtypes, reps, marks, 30000, pipeline, True, False, skew=skew)
    check_against_oracle(numel, dtypes, reps, marks, 30000, pipeline, False, True, skew=skew,
                         replica_skew=[0, 4, 8, 12])


@pytest.mark.parametrize("pipeline", [STAGED, FUSED])
def test_participation_with_coalesced_launches_and_kernel_variants(pipeline):
    d, _ = lib()
    numel, dtypes, reps, marks, _, _ = random_case(30, 40, 8, FP32, 6000)
    for options in ([(d.DDP_OPT_COALESCE, 1 << 62)], [(d.DDP_OPT_COALESCE, 0), (d.DDP_OPT_REDUCE_STREAMS, 1)],
                    [(d.DDP_OPT_COALESCE, 1 << 62), (d.DDP_OPT_REDUCE_BLOCKS_PER_CU, 1), (d.DDP_OPT_REDUCE_CAP_MIN_BYTES, 0)],
                    [(d.DDP_OPT_NONTEMPORAL, 0)]):
        check_against_oracle(numel, dtypes, reps, marks, 20000, pipeline, False, True, options=options)


@pytest.mark.parametrize("pipeline", [STAGED, FUSED])
def test_largest_replica_count_with_single_participants(pipeline):
    """R = 64: every mask bit position is exercised -- parameter p is used by
    replica p alone (and a few by the last two replicas)."""
    R = 64
    n = 70
    numel = [100 + 37 * p for p in range(n)]
    reps = [[workloads.gaussian_grad(40, r, 0, p, numel[p], 1.0, FP32) for p in range(n)] for r in range(R)]
    marks = []
    for p in range(n - 1, -1, -1):
        used = [0] * R
        if p < R:
            used[p] = 1
        else:
            used[62] = used[63] = 1
        marks.append((p, used))
        for r in range(R):
            if not used[r]:
                poison(reps[r][p], FP32)
    want, glob = check_against_oracle(numel, [FP32] * n, reps, marks, 4096, pipeline, False, True)
    assert glob.all()
    for p in range(R):          # one participant: the result is its gradient divided by 64, exactly
        assert want[0][p].tobytes() == (reps[p][p] / np.float32(64)).astype(np.float32).tobytes()


@pytest.mark.parametrize("pipeline", [STAGED, FUSED])
def test_iterations_alternate_between_masked_and_full_participation(pipeline):
    """Three synchronizations on one context: masks, then everybody (no flag
    table travels), then other masks -- flags, staging buffers and the bitmap
    must not leak from one iteration into the next."""
    d, harness = lib()
    n, R, cap = 30, 4, 16384
    base = random_case(50, n, R, FP32, 5000)
    numel, dtypes = base[0], base[1]
    grads = harness.DeviceGrads(numel, dtypes, R, fill=0xFF)
    with harness.Session(grads, cap, pipeline, True) as s:
        d.ddp_set_option(s.ctx, d.DDP_OPT_FIND_UNUSED, 1)
        for it in range(4):
            rng = np.random.default_rng(60 + it)
            reps = [[workloads.gaussian_grad(60 + it, r, 0, p, numel[p], 1e-2, FP32) for p in range(n)]
                    for r in range(R)]
            order = [int(p) for p in rng.permutation(n)]
            if it % 2 == 0:
                marks = [(p, [int(rng.random() < 0.5) for _ in range(R)]) for p in order[: n - 4]]
            else:
                marks = [(p, [1] * R) for p in order]
            flag = np.zeros((R, n), dtype=np.uint8)
            for p, used in marks:
                flag[:, p] = used
            for r in range(R):
                for p in range(n):
                    if not flag[r, p]:
                        poison(reps[r][p], FP32)
                grads.upload_replica(r, reps[r])
            want, _, wlog, glob = oracle.synchronize_local(numel, dtypes, cap, reps, marks, find_unused=True)
            for p, used in marks:
                d.ddp_mark_ready_local(s.ctx, p, used)
            d.ddp_finalize_backward(s.ctx)
            if it != 2:      # once, the bitmap is fetched while the reductions may still run
                d.ddp_synchronize(s.ctx)
            assert d.ddp_get_launch_log(s.ctx, 1) == wlog
            assert d.ddp_get_global_used(s.ctx, n).tolist() == glob.tolist()
            d.ddp_synchronize(s.ctx)
            for r in range(R):
                for p in range(n):
                    assert grads.download(r, p).tobytes() == want[r][p].tobytes(), f"iteration {it} r{r} p{p}"


@pytest.mark.parametrize("pipeline", [STAGED, FUSED])
@pytest.mark.parametrize("find_unused", [False, True])
def test_no_sync_participation_accumulates_into_the_bitmap(pipeline, find_unused):
    """Section 3.2.4: what no_sync iterations used still counts at the next
    synchronization.  A (replica, parameter) pair takes part if any micro-step
    or the final ready mark used it; pairs that never did hold NaNs."""
    d, harness = lib()
    rng = np.random.default_rng(70)
    n, R, K, cap = 20, 3, 3, 16384
    numel = [int(x) for x in rng.integers(1, 5000, size=n)]
    dts = [FP32] * n
    micro_used = rng.random((K, R, n)) < 0.4
    micro_used[:, :, 0] = False                      # parameter 0: only the final mark uses it
    micro_used[:, :, 1] = False                      # parameter 1: nobody, ever
    final_used = (rng.random((R, n)) < 0.4).astype(np.uint8)
    final_used[:, 1] = 0
    final_used[:, 0] = [1, 0, 0]
    order = [p for p in range(n - 1, -1, -1) if p != 5]     # parameter 5 gets no ready mark
    prior = micro_used.any(axis=0).astype(np.uint8)
    ever = prior | final_used
    ever[:, 5] = prior[:, 5]

    grads = harness.DeviceGrads(numel, dts, R, fill=0)
    micro_dev = harness.DeviceGrads(numel, dts, R)
    acc = [[np.zeros(x, dtype=np.float32) for x in numel] for _ in range(R)]
    for r in range(R):
        for p in range(n):
            if not ever[r, p]:
                poison(acc[r][p], FP32)
                grads.upload(r, p, acc[r][p])
    with harness.Session(grads, cap, pipeline, True) as s:
        d.ddp_set_option(s.ctx, d.DDP_OPT_FIND_UNUSED, 1 if find_unused else 0)
        for k in range(K):
            micro = [workloads.gaussian_replica(71, r, k, numel, 1e-2, FP32) for r in range(R)]
            ptrs = []
            for r in range(R):
                row = [micro[r][p] if micro_used[k, r, p] else None for p in range(n)]
                oracle.accumulate(acc[r], row, dts)
                for p in range(n):
                    if row[p] is not None:
                        micro_dev.upload(r, p, row[p])
                ptrs += [None if row[p] is None else micro_dev.ptr(r, p) for p in range(n)]
            d.ddp_no_sync_accumulate(s.ctx, ptrs)
            d.ddp_synchronize(s.ctx)
        # the final iteration's own gradients are already in the accumulators
        # (its backward pass added them); only its participation is new
        final = [workloads.gaussian_replica(72, r, 0, numel, 1e-2, FP32) for r in range(R)]
        for r in range(R):
            for p in range(n):
                if final_used[r, p] and p != 5:
                    if prior[r, p]:
                        acc[r][p] = (acc[r][p] + final[r][p]).astype(np.float32)
                    else:
                        acc[r][p] = final[r][p].copy()
                    grads.upload(r, p, acc[r][p])
        marks = [(p, final_used[:, p].tolist()) for p in order]
        want, _, wlog, glob = oracle.synchronize_local(numel, dts, cap, acc, marks, find_unused=find_unused,
                                                       prior_used=prior)
        assert glob.tolist() == ever.any(axis=0).astype(np.uint8).tolist()
        for p, used in marks:
            d.ddp_mark_ready_local(s.ctx, p, used)
        d.ddp_finalize_backward(s.ctx)
        d.ddp_synchronize(s.ctx)
        assert d.ddp_get_launch_log(s.ctx, 1) == wlog
        assert d.ddp_get_global_used(s.ctx, n).tolist() == glob.tolist()
        for r in range(R):
            for p in range(n):
                assert grads.download(r, p).tobytes() == want[r][p].tobytes(), f"r{r} p{p}"
        # the next synchronization starts from a clean bitmap
        d.ddp_finalize_backward(s.ctx)
        d.ddp_synchronize(s.ctx)
        assert d.ddp_get_global_used(s.ctx, n).tolist() == [0] * n


@pytest.mark.parametrize("pipeline", [STAGED, FUSED])
def test_participation_with_several_reduction_streams(pipeline):
    """Flag tables travel on whichever stream launches the bucket; four
    iterations with different masks are enqueued with no host synchronization
    between them (only the result of the last one can be checked then, plus
    the bitmap of each)."""
    d, harness = lib()
    n, R, cap = 40, 4, 9000
    numel, dtypes, reps, _, _, _ = random_case(80, n, R, FP32, 6000, n_unmarked=0, n_nobody=0)
    reps = [[workloads.gaussian_grad(80, r, 0, p, numel[p], 1e-2, FP32) for p in range(n)] for r in range(R)]
    grads = harness.DeviceGrads(numel, dtypes, R)
    for r in range(R):
        grads.upload_replica(r, reps[r])
    state = [[x.copy() for x in row] for row in reps]
    with harness.Session(grads, cap, pipeline, True) as s:
        d.ddp_set_option(s.ctx, d.DDP_OPT_REDUCE_STREAMS, 3)
        d.ddp_set_option(s.ctx, d.DDP_OPT_FIND_UNUSED, 1)
        for it in range(4):
            d.ddp_set_option(s.ctx, d.DDP_OPT_TAIL_ON_BACKWARD, it & 1)
            rng = np.random.default_rng(81 + it)
            order = [int(p) for p in rng.permutation(n)][: n - 3]
            marks = [(p, [int(rng.random() < 0.6) for _ in range(R)]) for p in order]
            state, _, wlog, glob = oracle.synchronize_local(numel, dtypes, cap, state, marks, find_unused=True)
            for p, used in marks:
                d.ddp_mark_ready_local(s.ctx, p, used)
            d.ddp_finalize_backward(s.ctx)
            assert d.ddp_get_launch_log(s.ctx, 1) == wlog
            assert d.ddp_get_global_used(s.ctx, n).tolist() == glob.tolist()
        d.ddp_synchronize(s.ctx)
        for r in range(R):
            for p in range(n):
                assert grads.download(r, p).tobytes() == state[r][p].tobytes(), f"r{r} p{p}"


def test_wholly_unused_buckets_are_not_launched():
    """Section 6.2.2, skipping at the bucket level: with find_unused a bucket
    whose parameters nobody used keeps its gradients and needs no kernel; the
    launch log (the schedule) still lists it, the timed launches do not."""
    d, harness = lib()
    n, R, cap = 12, 3, 8000                       # 1000 fp32 elements each: two parameters per bucket
    numel = [1000] * n
    dtypes = [FP32] * n
    reps = [[workloads.gaussian_grad(90, r, 0, p, numel[p], 1.0, FP32) for p in range(n)] for r in range(R)]
    asg = oracle.assign_buckets(numel, dtypes, cap)
    assert [bk.params for bk in asg.buckets] == [[11, 10], [9, 8], [7, 6], [5, 4], [3, 2], [1, 0]]
    dead = {9, 8, 3, 2}                           # buckets 1 and 4; parameter 5 alone does not empty bucket 3
    marks = []
    for p in range(n - 1, -1, -1):
        used = [0] * R if (p in dead or p == 5) else [1, int(p % 2), 1]
        marks.append((p, used))
        for r in range(R):
            if not used[r]:
                poison(reps[r][p], FP32)
    want, _, wlog, glob = oracle.synchronize_local(numel, dtypes, cap, reps, marks, find_unused=True)
    grads = harness.DeviceGrads(numel, dtypes, R)
    for r in range(R):
        grads.upload_replica(r, reps[r])
    for find_unused, expect in ((1, [0, 2, 3, 5]), (0, [0, 1, 2, 3, 4, 5])):
        with harness.Session(grads, cap, FUSED, True) as s:
            d.ddp_set_option(s.ctx, d.DDP_OPT_FIND_UNUSED, find_unused)
            d.ddp_set_option(s.ctx, d.DDP_OPT_COALESCE, 0)
            d.ddp_set_option(s.ctx, d.DDP_OPT_TIMING, 1)
            for p, used in marks:
                d.ddp_mark_ready_local(s.ctx, p, used)
            d.ddp_finalize_backward(s.ctx)
            d.ddp_synchronize(s.ctx)
            assert d.ddp_get_launch_log(s.ctx, 1) == wlog
            assert d.ddp_get_global_used(s.ctx, n).tolist() == glob.tolist()
            _, ids = d.ddp_get_kernel_times(s.ctx, d.DDP_K_REDUCE)
            assert [int(x) for x in ids] == expect
            if find_unused:
                for r in range(R):
                    for p in range(n):
                        assert grads.download(r, p).tobytes() == want[r][p].tobytes(), f"r{r} p{p}"
