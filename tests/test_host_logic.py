"""CPU-only tests of the library's host logic through the C ABI, on a
plan-only context (no device, nothing computed): bucket assignment and the
ready/launch state machine must agree with the oracle exactly; error paths
return codes instead of hanging or aborting; the shared library exports every
symbol the header declares."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
import workloads

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def d():
    import paper_2006_15704_amd as lib
    return lib


def plan(d, numel, dtype, cap, R=2):
    ctx = d.ddp_create(R, d.DDP_DEVICE_NONE)
    d.ddp_register_params(ctx, numel, dtype, None)
    nb = d.ddp_build_buckets(ctx, cap)
    return ctx, nb


def test_library_exports_every_declared_symbol(d):
    header = open(os.path.join(ROOT, "include", "ddp_gfx950.h")).read()
    declared = set(re.findall(r"\b(ddp_[a-z_]+)\s*\(", header))
    declared.discard("ddp_ctx")
    assert declared, "no declarations found"
    lib = ctypes.CDLL(d.binding.LIB_PATH)
    for name in sorted(declared):
        assert hasattr(lib, name), f"{name} is declared but not exported"
    assert declared == set(d.binding.EXPORTS)
    for name in d.binding.EXPORTS:
        assert callable(getattr(d, name)), f"binding lacks {name}"


@pytest.mark.parametrize("name,dt,caps", [
    ("tiny", 0, [0, 100, 16384, 1 << 20]),
    ("resnet50", 0, [0, 1 << 20, 5 << 20, 10 << 20, 25 << 20, 50 << 20, 100 << 20]),
    ("resnet50", 1, [0, 1 << 20, 5 << 20, 25 << 20]),
    ("bert_large", 0, [0, 1 << 20, 25 << 20, 25 * 10**6, 100 << 20]),
])
def test_assignment_matches_oracle(d, name, dt, caps):
    numel = workloads.numel_of(workloads.WORKLOAD_SHAPES[name]())
    n = len(numel)
    for cap in caps + [d.DDP_CAP_WHOLE_MODEL]:
        asg = oracle.assign_buckets(numel, [dt] * n, cap)
        ctx, nb = plan(d, numel, [dt] * n, cap)
        try:
            assert nb == len(asg.buckets)
            bucket_of, offset = d.ddp_get_assignment(ctx, n)
            assert bucket_of.tolist() == asg.bucket_of.tolist()
            assert offset.tolist() == asg.offset_of.tolist()
            for b, bk in enumerate(asg.buckets):
                assert d.ddp_get_bucket_info(ctx, b) == (bk.elems, len(bk.params), bk.dtype)
        finally:
            d.ddp_destroy(ctx)


@pytest.mark.parametrize("seed", range(30))
def test_random_assignment_and_schedule_match_oracle(d, seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(1, 120))
    numel = [int(x) for x in rng.integers(0, 5000, size=n)]
    dtype = [0] * n if seed % 2 else [int(x) for x in rng.integers(0, 3, size=n)]
    cap = int(rng.choice([0, 64, 1000, 8192, 100000]))
    asg = oracle.assign_buckets(numel, dtype, cap)
    order = [int(p) for p in rng.permutation(n)]
    if seed % 3 == 0:
        order = order[: int(rng.integers(0, n + 1))]
    ctx, nb = plan(d, numel, dtype, cap)
    try:
        bucket_of, offset = d.ddp_get_assignment(ctx, n)
        assert bucket_of.tolist() == asg.bucket_of.tolist()
        assert offset.tolist() == asg.offset_of.tolist()
        for it in range(2):          # pending counts must be replenished
            d.ddp_set_option(ctx, d.DDP_OPT_COALESCE, it << 40)      # the log does not depend on it
            if it == 1 and order:
                d.ddp_mark_ready_many(ctx, order[: len(order) // 2])
                rest = order[len(order) // 2:]
            else:
                rest = order
            for p in rest:
                d.ddp_mark_ready(ctx, p)
            running = d.ddp_get_launch_log(ctx, 0)
            d.ddp_finalize_backward(ctx)
            want = oracle.launch_schedule(asg, order)
            assert d.ddp_get_launch_log(ctx, 1) == want
            assert running == [x for x in want if x[1] < len(order)]
            used = d.ddp_get_used_map(ctx, n, 1)
            assert used.tolist() == [1 if p in set(order) else 0 for p in range(n)]
    finally:
        d.ddp_destroy(ctx)


def test_cap_arithmetic_does_not_wrap(d):
    # sizes close to 2^63 bytes: the running total must not overflow into "fits"
    huge = (1 << 60)
    ctx, nb = plan(d, [huge, huge, huge], [0, 0, 0], d.DDP_CAP_WHOLE_MODEL - 5)
    try:
        assert nb == len(oracle.assign_buckets([huge] * 3, [0] * 3, d.DDP_CAP_WHOLE_MODEL - 5).buckets)
    finally:
        d.ddp_destroy(ctx)


def test_error_codes(d):
    with pytest.raises(d.DdpError) as e:
        d.ddp_create(0, d.DDP_DEVICE_NONE)
    assert e.value.code == d.DDP_ERR_ARG
    with pytest.raises(d.DdpError) as e:
        d.ddp_create(d.DDP_MAX_REPLICAS + 1, d.DDP_DEVICE_NONE)
    assert e.value.code == d.DDP_ERR_UNSUPPORTED

    ctx = d.ddp_create(2, d.DDP_DEVICE_NONE)
    try:
        for call in (lambda: d.ddp_build_buckets(ctx, 100), lambda: d.ddp_mark_ready(ctx, 0),
                     lambda: d.ddp_finalize_backward(ctx)):
            with pytest.raises(d.DdpError) as e:
                call()
            assert e.value.code == d.DDP_ERR_STATE
        with pytest.raises(d.DdpError) as e:
            d.ddp_register_params(ctx, [4, 4], [0, 7], None)
        assert e.value.code == d.DDP_ERR_ARG
        with pytest.raises(d.DdpError) as e:
            d.ddp_register_params(ctx, [4, -1], [0, 0], None)
        assert e.value.code == d.DDP_ERR_ARG
        d.ddp_register_params(ctx, [4, 4, 4], [0, 0, 0], None)
        with pytest.raises(d.DdpError) as e:
            d.ddp_register_params(ctx, [4], [0], None)
        assert e.value.code == d.DDP_ERR_STATE
        assert d.ddp_build_buckets(ctx, 32) == 2
        with pytest.raises(d.DdpError) as e:
            d.ddp_build_buckets(ctx, 32)
        assert e.value.code == d.DDP_ERR_STATE
        with pytest.raises(d.DdpError) as e:
            d.ddp_set_option(ctx, d.DDP_OPT_PIPELINE, d.DDP_PIPELINE_FUSED)
        assert e.value.code == d.DDP_ERR_STATE
        for bad in (-1, 3, 1000):
            with pytest.raises(d.DdpError) as e:
                d.ddp_mark_ready(ctx, bad)
            assert e.value.code == d.DDP_ERR_ARG
        d.ddp_mark_ready(ctx, 2)
        with pytest.raises(d.DdpError) as e:
            d.ddp_mark_ready(ctx, 2)
        assert e.value.code == d.DDP_ERR_ALREADY_READY
        assert "already marked" in d.ddp_last_error(ctx)
        # the failed call changed nothing: bucket 0 = {2, 1} still waits for parameter 1
        assert d.ddp_get_launch_log(ctx, 0) == []
        d.ddp_mark_ready(ctx, 1)
        assert d.ddp_get_launch_log(ctx, 0) == [(0, 1)]
        for call in (lambda: d.ddp_synchronize(ctx),
                     lambda: d.ddp_synth_backward(ctx, [0]), lambda: d.ddp_get_bucket_ptr(ctx, 0, 0),
                     lambda: d.ddp_get_kernel_times(ctx, 1)):
            with pytest.raises(d.DdpError) as e:
                call()
            assert e.value.code == d.DDP_ERR_NO_DEVICE
        # no_sync covers whole iterations: refused once the running one has taken a ready mark
        # (its buckets may already be reducing the gradient tensors in place)
        with pytest.raises(d.DdpError) as e:
            d.ddp_no_sync_accumulate(ctx, [None] * 6)
        assert e.value.code == d.DDP_ERR_STATE
        assert "middle of a synchronizing iteration" in d.ddp_last_error(ctx)
        d.ddp_finalize_backward(ctx)      # parameter 0 never marked: no hang, launched by finalize
        assert d.ddp_get_launch_log(ctx, 1) == [(0, 1), (1, 2)]
        with pytest.raises(d.DdpError) as e:      # between iterations the call is in order again
            d.ddp_no_sync_accumulate(ctx, [None] * 6)
        assert e.value.code == d.DDP_ERR_NO_DEVICE
    finally:
        d.ddp_destroy(ctx)


@pytest.mark.parametrize("seed", range(12))
def test_participation_bitmap_host_logic_matches_oracle(d, seed):
    """Per-replica ready marks on a plan-only context: launch log, used map and
    the global bitmap (here the host's OR, no device involved) against the
    oracle's, over two iterations so that the flags are seen to reset."""
    rng = np.random.default_rng(1000 + seed)
    n, R = int(rng.integers(1, 60)), int(rng.integers(1, 9))
    numel = [int(x) for x in rng.integers(0, 3000, size=n)]
    dtype = [int(x) for x in rng.integers(0, 3, size=n)]
    cap = int(rng.choice([0, 1000, 8192]))
    ctx = d.ddp_create(R, d.DDP_DEVICE_NONE)
    try:
        d.ddp_register_params(ctx, numel, dtype, None)
        d.ddp_build_buckets(ctx, cap)
        d.ddp_set_option(ctx, d.DDP_OPT_FIND_UNUSED, seed & 1)
        for it in range(2):
            order = [int(p) for p in rng.permutation(n)][: int(rng.integers(0, n + 1))]
            marks = [(p, [int(x) for x in rng.integers(0, 2, size=R)]) for p in order]
            grads = [[np.zeros(x, dtype=oracle.STORAGE[t]) for x, t in zip(numel, dtype)] for _ in range(R)]
            _, asg, wlog, glob = oracle.synchronize_local(numel, dtype, cap, grads, marks)
            for p, used in marks:
                if all(used) and (p & 1):
                    d.ddp_mark_ready(ctx, p)
                else:
                    d.ddp_mark_ready_local(ctx, p, used)
            d.ddp_finalize_backward(ctx)
            assert d.ddp_get_launch_log(ctx, 1) == wlog
            assert d.ddp_get_global_used(ctx, n).tolist() == glob.tolist()
            assert d.ddp_get_used_map(ctx, n, 1).tolist() == glob.tolist()
    finally:
        d.ddp_destroy(ctx)


def test_participation_argument_errors(d):
    ctx = d.ddp_create(3, d.DDP_DEVICE_NONE)
    try:
        with pytest.raises(d.DdpError) as e:
            d.ddp_mark_ready_local(ctx, 0, [1, 1, 1])
        assert e.value.code == d.DDP_ERR_STATE
        d.ddp_register_params(ctx, [4, 4], [0, 0], None)
        with pytest.raises(d.DdpError) as e:
            d.ddp_get_global_used(ctx, 2)
        assert e.value.code == d.DDP_ERR_STATE
        d.ddp_build_buckets(ctx, 0)
        with pytest.raises(ValueError):
            d.ddp_mark_ready_local(ctx, 0, [1, 1])             # two flags for three replicas
        raw = d.binding._lib.ddp_mark_ready_local
        assert raw(ctx, 0, None) == d.DDP_ERR_ARG              # null flag array
        with pytest.raises(d.DdpError) as e:
            d.ddp_mark_ready_local(ctx, 2, [1, 0, 1])
        assert e.value.code == d.DDP_ERR_ARG
        d.ddp_mark_ready_local(ctx, 1, [0, 0, 1])
        with pytest.raises(d.DdpError) as e:
            d.ddp_mark_ready_local(ctx, 1, [1, 1, 1])
        assert e.value.code == d.DDP_ERR_ALREADY_READY
        d.ddp_finalize_backward(ctx)
        assert d.ddp_get_global_used(ctx, 2).tolist() == [0, 1]
        d.ddp_finalize_backward(ctx)                            # nothing marked at all
        assert d.ddp_get_global_used(ctx, 2).tolist() == [0, 0]
    finally:
        d.ddp_destroy(ctx)


def test_reduction_stream_option_is_validated(d):
    ctx, _ = plan(d, [4, 4, 4], [0, 0, 0], 0)
    try:
        for opt, bad in ((d.DDP_OPT_REDUCE_BLOCKS_PER_CU, -2), (d.DDP_OPT_REDUCE_BLOCKS_PER_CU, 17),
                         (d.DDP_OPT_REDUCE_CAP_MIN_BYTES, -1), (d.DDP_OPT_COALESCE, -2), (99, 0)):
            with pytest.raises(d.DdpError) as e:
                d.ddp_set_option(ctx, opt, bad)
            assert e.value.code == d.DDP_ERR_ARG
        d.ddp_set_option(ctx, d.DDP_OPT_REDUCE_BLOCKS_PER_CU, 0)
        d.ddp_set_option(ctx, d.DDP_OPT_REDUCE_CAP_MIN_BYTES, 1 << 40)
        for bad in (0, -2, 9):
            with pytest.raises(d.DdpError) as e:
                d.ddp_set_option(ctx, d.DDP_OPT_REDUCE_STREAMS, bad)
            assert e.value.code == d.DDP_ERR_ARG
        d.ddp_set_option(ctx, d.DDP_OPT_REDUCE_STREAMS, 8)
        d.ddp_mark_ready(ctx, 2)
        with pytest.raises(d.DdpError) as e:                 # not in the middle of an iteration
            d.ddp_set_option(ctx, d.DDP_OPT_REDUCE_STREAMS, 2)
        assert e.value.code == d.DDP_ERR_STATE
        d.ddp_finalize_backward(ctx)
        d.ddp_set_option(ctx, d.DDP_OPT_REDUCE_STREAMS, 2)
        assert d.ddp_get_launch_log(ctx, 1) == [(0, 0), (1, 1), (2, 1)]
    finally:
        d.ddp_destroy(ctx)


@pytest.mark.parametrize("seed", range(20))
def test_rebuild_from_trace_matches_oracle(d, seed):
    """Section 6.2.1 on a plan-only context: the trace the library records is
    the ready order; the rebuilt mapping and the following iteration's launch
    log equal the oracle's; a second rebuild follows the newer trace."""
    rng = np.random.default_rng(3000 + seed)
    n = int(rng.integers(1, 100))
    numel = [int(x) for x in rng.integers(0, 4000, size=n)]
    dtype = [0] * n if seed % 2 else [int(x) for x in rng.integers(0, 3, size=n)]
    cap = int(rng.choice([0, 1000, 8192, 60000]))
    ctx, nb = plan(d, numel, dtype, cap, R=3)
    try:
        assert d.ddp_get_ready_order(ctx, 1) == []
        for it in range(3):
            order = [int(p) for p in rng.permutation(n)]
            if (seed + it) % 3 == 0:
                order = order[: int(rng.integers(0, n + 1))]
            for k, p in enumerate(order):
                d.ddp_mark_ready(ctx, p)
                if k == 0:
                    assert d.ddp_get_ready_order(ctx, 0) == [p]
            d.ddp_finalize_backward(ctx)
            assert d.ddp_get_ready_order(ctx, 1) == order
            assert d.ddp_get_ready_order(ctx, 0) == []
            cap2 = int(rng.choice([cap, 500, 20000]))
            visit = oracle.traced_visit_order(order, n)
            asg = oracle.assign_buckets_in_order(numel, dtype, cap2, visit)
            assert d.ddp_rebuild_buckets(ctx, cap2) == len(asg.buckets)
            bucket_of, offset = d.ddp_get_assignment(ctx, n)
            assert bucket_of.tolist() == asg.bucket_of.tolist()
            assert offset.tolist() == asg.offset_of.tolist()
            for b, bk in enumerate(asg.buckets):
                assert d.ddp_get_bucket_info(ctx, b) == (bk.elems, len(bk.params), bk.dtype)
            assert d.ddp_get_launch_log(ctx, 1) == []            # old bucket numbers are gone
            assert d.ddp_get_ready_order(ctx, 1) == order        # the trace stays
            # the same backward order again: every bucket goes out with its last gradient
            d.ddp_mark_ready_many(ctx, order)
            d.ddp_finalize_backward(ctx)
            assert d.ddp_get_launch_log(ctx, 1) == oracle.launch_schedule(asg, order)
    finally:
        d.ddp_destroy(ctx)


def test_rebuild_state_errors_and_empty_trace(d):
    ctx = d.ddp_create(2, d.DDP_DEVICE_NONE)
    try:
        d.ddp_register_params(ctx, [100, 200, 50, 400, 25, 300], [0] * 6, None)
        with pytest.raises(d.DdpError) as e:
            d.ddp_rebuild_buckets(ctx, 1600)
        assert e.value.code == d.DDP_ERR_STATE
        assert d.ddp_build_buckets(ctx, 1600) == 3
        # no iteration closed yet: the trace is empty and the mapping stays the default one
        assert d.ddp_rebuild_buckets(ctx, 1600) == 3
        assert d.ddp_get_assignment(ctx, 6)[0].tolist() == [2, 2, 2, 1, 0, 0]
        d.ddp_mark_ready(ctx, 4)
        with pytest.raises(d.DdpError) as e:
            d.ddp_rebuild_buckets(ctx, 1600)
        assert e.value.code == d.DDP_ERR_STATE
        for p in (5, 1, 3):
            d.ddp_mark_ready(ctx, p)
        d.ddp_finalize_backward(ctx)
        assert d.ddp_get_launch_log(ctx, 1) == [(0, 1), (1, 3), (2, 4)]
        assert d.ddp_rebuild_buckets(ctx, 1600) == 4
        bucket_of, offset = d.ddp_get_assignment(ctx, 6)
        assert bucket_of.tolist() == [3, 1, 3, 2, 0, 0] and offset.tolist() == [50, 0, 0, 0, 0, 25]
        for p in (4, 5, 1, 3):
            d.ddp_mark_ready(ctx, p)
        d.ddp_finalize_backward(ctx)
        assert d.ddp_get_launch_log(ctx, 1) == [(0, 1), (1, 2), (2, 3), (3, 4)]
        assert d.ddp_get_used_map(ctx, 6, 1).tolist() == [0, 1, 0, 1, 1, 1]
    finally:
        d.ddp_destroy(ctx)


def test_compute_context_without_gpu_fails_loudly(d):
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    with pytest.raises(d.DdpError) as e:
        d.ddp_create(2, 0)
    assert e.value.code == d.DDP_ERR_HIP


def test_options_read_back_on_a_plan_only_context(d):
    ctx, nb = plan(d, [100, 200, 300], [0, 0, 0], 1 << 20)
    try:
        assert d.ddp_get_option(ctx, d.DDP_OPT_REDUCE_STREAMS) == -1      # chosen per launch
        assert d.ddp_get_option(ctx, d.DDP_OPT_GATE_WAIT_US) == 100000
        d.ddp_set_option(ctx, d.DDP_OPT_GATE_WAIT_US, 5)
        assert d.ddp_get_option(ctx, d.DDP_OPT_GATE_WAIT_US) == 5
        # nothing can be ordered through device flags without a device
        assert d.ddp_get_option(ctx, d.DDP_OPT_FLAG_ORDER) == 0
        assert d.ddp_get_option(ctx, d.DDP_STAT_REPAIRED_LAUNCHES) == 0
        assert d.ddp_get_option(ctx, d.DDP_OPT_COALESCE) > 0          # the limit chosen from R
        # every option that can be set can be read
        for opt, val in ((d.DDP_OPT_NONTEMPORAL, 0), (d.DDP_OPT_EMIT_BUSY_BLOCKS, 7), (d.DDP_OPT_REDUCE_BLOCKS_PER_CU, 3),
                         (d.DDP_OPT_REDUCE_CAP_MIN_BYTES, 12345), (d.DDP_OPT_ACCUMULATE_BLOCKS_PER_CU, 4),
                         (d.DDP_OPT_CHAIN_LAUNCHES, 0)):
            d.ddp_set_option(ctx, opt, val)
            assert d.ddp_get_option(ctx, opt) == val
        with pytest.raises(d.DdpError) as e:
            d.ddp_get_option(ctx, 9999)
        assert e.value.code == d.DDP_ERR_ARG
        for bad in (1, -2):
            with pytest.raises(d.DdpError) as e:
                d.ddp_set_option(ctx, d.DDP_OPT_FLAG_ORDER, bad)
            assert e.value.code == d.DDP_ERR_ARG
    finally:
        d.ddp_destroy(ctx)


def test_outputs_for_16_bit_gradients_on_a_plan_only_context(d):
    ctx = d.ddp_create(2, d.DDP_DEVICE_NONE)
    try:
        with pytest.raises(d.DdpError) as e:
            d.ddp_set_outputs(ctx, None)
        assert e.value.code == d.DDP_ERR_STATE
        d.ddp_register_params(ctx, [1000, 2000, 3000], [1, 1, 2], None)
        d.ddp_set_outputs(ctx, None)           # a plan has no memory: the pointers are not looked at
        # buckets are capped by the 16-bit bytes: 2000 + 1000 elements of 2 bytes fit 6000 bytes
        assert d.ddp_build_buckets(ctx, 6000) == 2
        assert d.ddp_get_assignment(ctx, 3)[0].tolist() == oracle.assign_buckets([1000, 2000, 3000], [1, 1, 2], 6000).bucket_of.tolist()
        with pytest.raises(d.DdpError) as e:
            d.ddp_set_outputs(ctx, None)
        assert e.value.code == d.DDP_ERR_STATE
    finally:
        d.ddp_destroy(ctx)
    ctx = d.ddp_create(2, d.DDP_DEVICE_NONE)
    try:
        d.ddp_register_params(ctx, [10, 10], [0, 1], None)
        with pytest.raises(d.DdpError) as e:
            d.ddp_set_outputs(ctx, None)
        assert e.value.code == d.DDP_ERR_ARG
    finally:
        d.ddp_destroy(ctx)


@pytest.mark.parametrize("hold", [1, 3, 50])
def test_launch_hold_changes_neither_the_buckets_nor_the_launch_log(d, hold):
    """DDP_OPT_LAUNCH_HOLD only postpones when a launchable bucket is enqueued; which bucket
    became launchable after which mark is what the log records."""
    rng = np.random.default_rng(hold)
    numel = [int(x) for x in rng.integers(1, 400, size=60)]
    order = [int(p) for p in rng.permutation(60)][:55]          # five never marked
    ctx, nb = plan(d, numel, [0] * 60, 2000)
    try:
        d.ddp_set_option(ctx, d.DDP_OPT_LAUNCH_HOLD, hold)
        assert d.ddp_get_option(ctx, d.DDP_OPT_LAUNCH_HOLD) == hold
        asg = oracle.assign_buckets(numel, [0] * 60, 2000)
        want = oracle.launch_schedule(asg, order)
        for k, p in enumerate(order):
            d.ddp_mark_ready(ctx, p)
            assert d.ddp_get_launch_log(ctx, 0) == [x for x in want if x[1] <= k]
        with pytest.raises(d.DdpError) as e:                    # only between iterations
            d.ddp_set_option(ctx, d.DDP_OPT_LAUNCH_HOLD, 0)
        assert e.value.code == d.DDP_ERR_STATE
        d.ddp_finalize_backward(ctx)
        assert d.ddp_get_launch_log(ctx, 1) == want
        with pytest.raises(d.DdpError) as e:
            d.ddp_set_option(ctx, d.DDP_OPT_LAUNCH_HOLD, -1)
        assert e.value.code == d.DDP_ERR_ARG
    finally:
        d.ddp_destroy(ctx)
