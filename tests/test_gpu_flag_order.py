"""GPU parity for the ordering of bucket launches after the backward stream
through device flags (an announcement kernel on the backward stream, a gate
kernel in front of every bucket kernel, a repair launch at finalize), against
the oracle on the same seeded inputs.  Gradient memory starts as NaN and is
written by the synthetic backward stream after a delay, so a bucket kernel that
ran ahead of its gate, or a launch that was skipped and not repaired, shows in
the result.  A gate wait of 0 makes every gate give up without waiting (the
condition is forced from the host; every kernel still ends normally), which
sends everything through the repair launch."""
import numpy as np
import pytest

import oracle
import workloads

pytestmark = pytest.mark.gpu

FP32, FP16, BF16 = 0, 1, 2
FUSED = 1
NAN_BITS = {FP32: np.float32(np.nan), FP16: np.float16(np.nan), BF16: np.uint16(0x7FC1)}


def lib():
    import paper_2006_15704_amd as d
    from paper_2006_15704_amd import harness
    return d, harness


def ragged(seed, n, max_elems):
    rng = np.random.default_rng(seed)
    numel = [int(x) for x in rng.integers(1, max_elems, size=n)]
    numel[0] = 5
    numel[n // 2] = 3 * 4096 + 7          # whole tiles and a ragged tail
    return numel


def session_with_flags(d, harness, grads, cap, streams, write_all=False):
    s = harness.Session(grads, cap, FUSED, write_all)
    d.ddp_set_option(s.ctx, d.DDP_OPT_COALESCE, 0)             # one launch (and one gate) per bucket
    d.ddp_set_option(s.ctx, d.DDP_OPT_REDUCE_STREAMS, streams)
    if not d.ddp_get_option(s.ctx, d.DDP_OPT_FLAG_ORDER):
        s.close()
        pytest.skip("no pair of streams on separate hardware queues was found: launches are ordered by events")
    return s


@pytest.mark.parametrize("dtype", [FP32, FP16])
@pytest.mark.parametrize("streams", [1, 2])
@pytest.mark.parametrize("gate_wait_us", [100000, 0])
def test_flag_ordered_launches_wait_for_the_backward_stream(dtype, streams, gate_wait_us):
    d, harness = lib()
    import torch
    numel = ragged(31, 14, 9000)
    n, R, cap = len(numel), 3, 32 << 10
    dtypes = [dtype] * n
    grads = harness.DeviceGrads(numel, dtypes, R, fill=0xFF)
    keep = harness.DeviceGrads(numel, dtypes, 3, fill=0)
    srcs, wants = [], []
    for it in range(3):
        reps = [workloads.gaussian_replica(600 + it, r, 0, numel, 1.0, dtype) for r in range(R)]
        src = harness.DeviceGrads(numel, dtypes, R)
        for r in range(R):
            src.upload_replica(r, reps[r])
        srcs.append(src)
        wants.append(oracle.synchronize(numel, dtypes, cap, reps))
    s = session_with_flags(d, harness, grads, cap, streams)
    with s:
        d.ddp_set_option(s.ctx, d.DDP_OPT_GATE_WAIT_US, gate_wait_us)
        before = d.ddp_get_option(s.ctx, d.DDP_STAT_REPAIRED_LAUNCHES)
        order = list(range(n - 1, -1, -1))
        for it in range(3):       # three iterations enqueued without host synchronization in between
            d.ddp_synth_backward(s.ctx, order, [150_000] * n, srcs[it].ptrs(), True)
            d.ddp_finalize_backward(s.ctx)
            assert d.ddp_get_launch_log(s.ctx, 1) == wants[it][2]
            with torch.cuda.stream(s.backward_stream):      # work after finalize sees the averages
                keep.bufs[it].copy_(grads.bufs[0], non_blocking=True)
        d.ddp_synchronize(s.ctx)
        torch.cuda.synchronize()
        repaired = d.ddp_get_option(s.ctx, d.DDP_STAT_REPAIRED_LAUNCHES) - before
        nb = s.n_buckets
    for it in range(3):
        for i in range(n):
            assert keep.download(it, i).tobytes() == wants[it][0][i].tobytes(), f"iteration {it} parameter {i}"
    if gate_wait_us == 0:
        # the delay kernels are far longer than a single look: all gated launches were repaired
        # (every bucket but the ones launched by the call that completes the iteration)
        assert repaired >= 3 * (nb - 2), (repaired, nb)
    else:
        assert repaired == 0


@pytest.mark.parametrize("find_unused", [False, True])
@pytest.mark.parametrize("gate_wait_us", [100000, 0])
def test_flag_ordering_with_partial_participation_and_all_writers(find_unused, gate_wait_us):
    """Per-replica participation flags travel to the device while the backward
    stream is busy; the repair launch sees the whole bitmap."""
    d, harness = lib()
    rng = np.random.default_rng(77)
    numel = ragged(32, 12, 7000)
    n, R, cap = len(numel), 4, 24 << 10
    dtypes = [FP32] * n
    reps = [[workloads.gaussian_grad(640, r, 0, p, numel[p], 1e-2, FP32) for p in range(n)] for r in range(R)]
    order = [int(p) for p in rng.permutation(n)]
    marks = []
    for k, p in enumerate(order[:-1]):                       # the last one is never marked
        used = [0] * R if k == 2 else [int(rng.random() < 0.6) for _ in range(R)]
        if k % 3 == 0 and k != 2:
            used = [1] * R
        marks.append((p, used))
    flag = np.zeros((R, n), dtype=np.uint8)
    for p, used in marks:
        flag[:, p] = used
    for r in range(R):
        for p in range(n):
            if not flag[r, p]:
                reps[r][p][...] = NAN_BITS[FP32]
    want, _, wlog, glob = oracle.synchronize_local(numel, dtypes, cap, reps, marks, find_unused=find_unused)
    grads = harness.DeviceGrads(numel, dtypes, R, fill=0xFF)
    for r in range(R):
        grads.upload_replica(r, reps[r])
    s = session_with_flags(d, harness, grads, cap, 2, write_all=True)
    with s:
        d.ddp_set_option(s.ctx, d.DDP_OPT_FIND_UNUSED, 1 if find_unused else 0)
        d.ddp_set_option(s.ctx, d.DDP_OPT_GATE_WAIT_US, gate_wait_us)
        for p, used in marks:
            # a delay kernel keeps the backward stream busy, so the mark that follows orders its launches
            d.ddp_synth_backward(s.ctx, [p], [200_000], None, False)
            d.ddp_mark_ready_local(s.ctx, p, used)
        d.ddp_finalize_backward(s.ctx)
        d.ddp_synchronize(s.ctx)
        assert d.ddp_get_launch_log(s.ctx, 1) == wlog
        assert d.ddp_get_global_used(s.ctx, n).tolist() == glob.tolist()
        for r in range(R):
            for i in range(n):
                assert grads.download(r, i).tobytes() == want[r][i].tobytes(), f"replica {r} parameter {i}"


def test_flag_ordering_with_mixed_element_types_and_gates_that_give_up():
    d, harness = lib()
    numel = ragged(33, 10, 6000)
    n, R, cap = len(numel), 2, 16 << 10
    dtypes = [FP32, FP32, FP16, FP16, FP16, BF16, FP32, BF16, BF16, FP32]
    reps = [[workloads.gaussian_grad(650, r, 0, p, numel[p], 1.0, dtypes[p]) for p in range(n)] for r in range(R)]
    want, _, wlog = oracle.synchronize(numel, dtypes, cap, reps)
    grads = harness.DeviceGrads(numel, dtypes, R, fill=0xFF)
    src = harness.DeviceGrads(numel, dtypes, R)
    for r in range(R):
        src.upload_replica(r, reps[r])
    s = session_with_flags(d, harness, grads, cap, 1)
    with s:
        d.ddp_set_option(s.ctx, d.DDP_OPT_GATE_WAIT_US, 0)
        d.ddp_synth_backward(s.ctx, list(range(n - 1, -1, -1)), [150_000] * n, src.ptrs(), True)
        d.ddp_finalize_backward(s.ctx)
        d.ddp_synchronize(s.ctx)
        assert d.ddp_get_launch_log(s.ctx, 1) == wlog
        assert d.ddp_get_option(s.ctx, d.DDP_STAT_REPAIRED_LAUNCHES) >= 1
        for i in range(n):
            assert grads.download(0, i).tobytes() == want[i].tobytes(), f"parameter {i}"


def test_events_and_flags_give_the_same_bits_and_options_are_validated():
    d, harness = lib()
    numel = ragged(34, 9, 5000)
    n, R, cap = len(numel), 2, 16 << 10
    reps = [workloads.gaussian_replica(660, r, 0, numel, 1.0, FP32) for r in range(R)]
    want, _, _ = oracle.synchronize(numel, [FP32] * n, cap, reps)
    for flag_order in (0, -1):
        grads = harness.DeviceGrads(numel, [FP32] * n, R, fill=0xFF)
        src = harness.DeviceGrads(numel, [FP32] * n, R)
        for r in range(R):
            src.upload_replica(r, reps[r])
        with harness.Session(grads, cap, FUSED) as s:
            d.ddp_set_option(s.ctx, d.DDP_OPT_FLAG_ORDER, flag_order)
            if flag_order == 0:
                assert d.ddp_get_option(s.ctx, d.DDP_OPT_FLAG_ORDER) == 0
            for bad in (1, 2, -2):
                with pytest.raises(d.DdpError) as e:
                    d.ddp_set_option(s.ctx, d.DDP_OPT_FLAG_ORDER, bad)
                assert e.value.code == d.DDP_ERR_ARG
            with pytest.raises(d.DdpError) as e:
                d.ddp_set_option(s.ctx, d.DDP_OPT_GATE_WAIT_US, -1)
            assert e.value.code == d.DDP_ERR_ARG
            d.ddp_mark_ready(s.ctx, n - 1)
            with pytest.raises(d.DdpError) as e:             # only between iterations
                d.ddp_set_option(s.ctx, d.DDP_OPT_FLAG_ORDER, 0)
            assert e.value.code == d.DDP_ERR_STATE
            d.ddp_finalize_backward(s.ctx)
            d.ddp_synchronize(s.ctx)
            d.ddp_synth_backward(s.ctx, list(range(n - 1, -1, -1)), [100_000] * n, src.ptrs(), True)
            d.ddp_finalize_backward(s.ctx)
            d.ddp_synchronize(s.ctx)
            for i in range(n):
                assert grads.download(0, i).tobytes() == want[i].tobytes(), f"flag_order {flag_order} parameter {i}"


@pytest.mark.parametrize("hold", [2, 6, 1000])
@pytest.mark.parametrize("flag_order", [-1, 0])
def test_launch_hold_under_a_running_backward_pass(hold, flag_order):
    """DDP_OPT_LAUNCH_HOLD: launchable buckets wait for a few more marks and share launches;
    the ordering after the backward stream, the launch log and the bits stay what they are.
    Marks arrive through the synthetic backward pass (NaN until produced) in a seeded random
    order with three parameters never marked."""
    d, harness = lib()
    import torch
    rng = np.random.default_rng(40 + hold)
    numel = ragged(35, 30, 5000)
    n, R, cap = len(numel), 3, 20 << 10
    dtypes = [FP32] * n
    order = [int(p) for p in rng.permutation(n)][: n - 3]
    reps = [workloads.gaussian_replica(670, r, 0, numel, 1.0, FP32) for r in range(R)]
    want, asg, wlog = oracle.synchronize(numel, dtypes, cap, reps, order)
    grads = harness.DeviceGrads(numel, dtypes, R, fill=0xFF)
    src = harness.DeviceGrads(numel, dtypes, R)
    for r in range(R):
        src.upload_replica(r, reps[r])
    with harness.Session(grads, cap, FUSED) as s:
        d.ddp_set_option(s.ctx, d.DDP_OPT_FLAG_ORDER, flag_order)
        d.ddp_set_option(s.ctx, d.DDP_OPT_LAUNCH_HOLD, hold)
        for it in range(2):
            for p in order:                    # one call per parameter: produce it, then mark it
                d.ddp_synth_backward(s.ctx, [p], [60_000], src.ptrs(), False)
                d.ddp_mark_ready(s.ctx, p)
            d.ddp_finalize_backward(s.ctx)
            d.ddp_synchronize(s.ctx)
            assert d.ddp_get_launch_log(s.ctx, 1) == wlog
            for i in range(n):
                assert grads.download(0, i).tobytes() == want[i].tobytes(), f"iteration {it} parameter {i}"
            for r in range(R):                 # back to NaN for the next iteration
                grads.bufs[r].fill_(0xFF)
            torch.cuda.synchronize()
