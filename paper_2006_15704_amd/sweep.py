"""Bucket-size sweep with a synthetic backward pass (one GPU).

The one-GPU analogue of the paper's bucket-size experiment (Section 5.2) and of
its overlap measurement (Section 5.1): ResNet-50-shaped fp16 gradients, R = 16
replica copies, bucket caps from 0 (every gradient alone) to the whole model.
A synthetic backward stream stands in for autograd: for every parameter, in
reverse registration order, it runs a kernel that waits a fixed delay and then
the parameter is marked ready, so buckets are reduced on the reduction stream
while "backward" is still running.

For every cap and delay the script reports
    t_backward   the backward pass alone (no ready marks)
    t_sync       the synchronization alone (ready marks without delay)
    t_total      backward with ready marks + finalize, until the averaged
                 gradients are complete
(all three are GPU times between two events on the backward stream)
    exposed      t_total - t_backward: synchronization time not hidden
    after_marks  the part of t_total after everything ddp_synth_backward enqueued
                 on the backward stream (an event between it and finalize); with
                 DDP_OPT_TAIL_ON_BACKWARD that includes the last buckets
    overlap      1 - exposed / t_sync
one JSON object per line.  Run:  python -m paper_2006_15704_amd.sweep

`python -m paper_2006_15704_amd.sweep --knobs` runs the sweeps that the
library's launch defaults rest on instead (see knob_sweep).
"""
from __future__ import annotations

import argparse
import itertools
import json
import os
import statistics
import sys
import time

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

MIB = 1 << 20


def timed(fn, sync, reps, torch, stream):
    """Median GPU time of fn(): the work is bracketed by two events recorded on
    the backward stream.  ddp_finalize_backward makes that stream wait for the
    reductions, so the closing event marks the completion of everything."""
    out = []
    for _ in range(reps):
        sync()
        a = torch.cuda.Event(enable_timing=True)
        b = torch.cuda.Event(enable_timing=True)
        a.record(stream)
        fn()
        b.record(stream)
        sync()
        b.synchronize()
        out.append(a.elapsed_time(b))
    return statistics.median(out)


def timed_exposed(backward, finalize, sync, reps, torch, stream):
    """Median GPU times of backward() followed by finalize(): the whole thing,
    and the part after everything backward() enqueued on the stream (an event
    between the two calls)."""
    total, exposed = [], []
    for _ in range(reps):
        sync()
        a, m, b = (torch.cuda.Event(enable_timing=True) for _ in range(3))
        a.record(stream)
        backward()
        m.record(stream)
        finalize()
        b.record(stream)
        sync()
        b.synchronize()
        total.append(a.elapsed_time(b))
        exposed.append(m.elapsed_time(b))
    return statistics.median(total), statistics.median(exposed)


def knob_sweep(args) -> int:
    """The measurements behind the library's launch defaults, one JSON object per
    line: resident reduce blocks per compute unit, launch size (coalescing
    limit) against the number of replicas, and the non-temporal hint, on the
    BERT-large- and ResNet-50-shaped lists in binary32.  All marks of a step
    arrive in one call; GPU time between two events around the timed steps."""
    import torch
    import workloads
    import paper_2006_15704_amd as lib
    from paper_2006_15704_amd import harness

    def rate(workload, R, options, steps, replica_skew=None, per_call=False, bf16_to_binary32=False):
        if workload == "uniform":          # 40 tensors of 25 MiB: every tile is interior
            numel = [25 * MIB // 4] * 40
        else:
            numel = workloads.numel_of(workloads.WORKLOAD_SHAPES[workload]())
        n = len(numel)
        dtype = 2 if bf16_to_binary32 else 0
        grads = harness.DeviceGrads(numel, [dtype] * n, R, replica_skew=replica_skew)
        outputs = harness.DeviceGrads(numel, [0] * n, 1) if bf16_to_binary32 else None
        gen = torch.Generator(device="cuda")
        gen.manual_seed(7)
        for r in range(R):
            b = grads.bufs[r]
            if bf16_to_binary32:
                b[: b.numel() // 2 * 2].view(torch.bfloat16).normal_(0.0, 1e-3, generator=gen)
            else:
                b[: b.numel() // 4 * 4].view(torch.float32).normal_(0.0, 1e-3, generator=gen)
        order = list(range(n - 1, -1, -1))

        def step(ctx):
            if per_call:
                for p in order:
                    lib.ddp_mark_ready(ctx, p)
            else:
                lib.ddp_mark_ready_many(ctx, order)
            lib.ddp_finalize_backward(ctx)

        with harness.Session(grads, 25 * MIB, lib.DDP_PIPELINE_FUSED, outputs=outputs) as s:
            for opt, val in options:
                lib.ddp_set_option(s.ctx, opt, val)
            for _ in range(2):
                step(s.ctx)
            lib.ddp_synchronize(s.ctx)
            runs = []
            for _ in range(3):          # the median of three runs: the box stalls a process now and then
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record(s.backward_stream)
                for _ in range(steps):
                    step(s.ctx)
                b.record(s.backward_stream)
                lib.ddp_synchronize(s.ctx)
                torch.cuda.synchronize()
                runs.append(a.elapsed_time(b) / steps)
            ms = statistics.median(runs)
        total = (R * 2 + 4) * sum(numel) if bf16_to_binary32 else (R + 1) * sum(numel) * 4
        return round(ms, 4), round(total / ms / 1e6 / 8000.0, 4)

    def emit(**kw):
        print(json.dumps(kw), flush=True)

    for workload, steps in (("resnet50", 40), ("bert_large", 8)):
        for blocks in (0, 1, 2, 3, 4):
            ms, frac = rate(workload, 8, ((lib.DDP_OPT_REDUCE_BLOCKS_PER_CU, blocks), (lib.DDP_OPT_REDUCE_CAP_MIN_BYTES, 0)), steps)
            emit(sweep="blocks_per_cu", workload=workload, R=8, blocks_per_cu=blocks, ms_per_sync=ms, frac_of_hbm_peak=frac)
    for R in (2, 4, 8, 16, 32):
        for mib in (25, 50, 70, 100, 240, 400):
            ms, frac = rate("bert_large", R, ((lib.DDP_OPT_COALESCE, mib * MIB),), 4 if R >= 16 else 8)
            emit(sweep="launch_size", workload="bert_large", R=R, coalesce_mib=mib, ms_per_sync=ms, frac_of_hbm_peak=frac)
        ms, frac = rate("bert_large", R, (), 4 if R >= 16 else 8)
        emit(sweep="launch_size", workload="bert_large", R=R, coalesce_mib="default", ms_per_sync=ms, frac_of_hbm_peak=frac)
    for workload, steps in (("resnet50", 40), ("bert_large", 8)):
        for nt in (1, 0):
            ms, frac = rate(workload, 8, ((lib.DDP_OPT_NONTEMPORAL, nt),), steps)
            emit(sweep="nontemporal", workload=workload, R=8, nontemporal=nt, ms_per_sync=ms, frac_of_hbm_peak=frac)
    # one launch per 25 MiB bucket, one ready mark per call: from which launch size on the cap on resident
    # blocks pays and a second reduction stream no longer does (DDP_OPT_REDUCE_CAP_MIN_BYTES)
    for R in (8, 16, 32):
        for what, opts in (("short launch: no cap, two reduction streams", ((lib.DDP_OPT_REDUCE_CAP_MIN_BYTES, 1 << 50),)),
                           ("long launch: cap, one reduction stream", ((lib.DDP_OPT_REDUCE_CAP_MIN_BYTES, 0),)),
                           ("library default", ())):
            ms, frac = rate("bert_large", R, opts, 4 if R >= 16 else 8, per_call=True)
            emit(sweep="long_launch", workload="bert_large", R=R, treated_as=what, ms_per_sync=ms, frac_of_hbm_peak=frac)
    # 16-bit gradients in, binary32 averages out (ddp_set_outputs): resident blocks per compute unit
    for blocks in (0, 2, 3, 4, 5, -1):
        ms, frac = rate("bert_large", 8, ((lib.DDP_OPT_REDUCE_BLOCKS_PER_CU, blocks),) + (((lib.DDP_OPT_REDUCE_CAP_MIN_BYTES, 0),) if blocks >= 0 else ()),
                        8, bf16_to_binary32=True)
        emit(sweep="blocks_per_cu_binary32_outputs", workload="bert_large bf16 -> binary32", R=8,
             blocks_per_cu="default" if blocks < 0 else blocks, ms_per_sync=ms, frac_of_hbm_peak=frac)
    # replicas whose tensors sit at different offsets modulo 16 bytes
    for what, skew in (("all replicas alike modulo 16 bytes", None),
                       ("replica r shifted by 4 * (r mod 4) bytes", [4 * (r % 4) for r in range(8)])):
        ms, frac = rate("uniform", 8, (), 8, replica_skew=skew)
        emit(sweep="replica_alignment", workload="40 tensors of 25 MiB", R=8, placement=what, ms_per_sync=ms,
             frac_of_hbm_peak=frac)
    return 0


def main() -> int:
    if "--knobs" in sys.argv:
        return knob_sweep(None)
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="resnet50", choices=["resnet50", "bert_large"])
    ap.add_argument("--dtype", default="f16", choices=["f32", "f16", "bf16"])
    ap.add_argument("--replicas", type=int, default=16)
    ap.add_argument("--caps-mib", default="0,1,5,10,25,50,100,-1",
                    help="comma list of caps in MiB; -1 = whole model")
    ap.add_argument("--delays-us", default="0,10,50")
    ap.add_argument("--pipelines", default="fused,staged")
    ap.add_argument("--reps", type=int, default=20)
    ap.add_argument("--busy-blocks", type=int, default=0,
                    help="delay kernels use this many thread blocks doing arithmetic instead of "
                         "one sleeping block")
    ap.add_argument("--streams", default="1",
                    help="comma list: numbers of reduction streams (DDP_OPT_REDUCE_STREAMS)")
    ap.add_argument("--coalesce-mib", type=float, default=0,
                    help="DDP_OPT_COALESCE in MiB (0 = off, negative = no limit)")
    ap.add_argument("--hold", type=int, default=0,
                    help="DDP_OPT_LAUNCH_HOLD: a launchable bucket waits for this many further ready marks so "
                         "that its successors can share its launch (needs --coalesce-mib other than 0)")
    ap.add_argument("--chain", type=int, default=1, choices=[0, 1],
                    help="DDP_OPT_CHAIN_LAUNCHES: 1 = a launch behind a long one on another stream starts as that one drains")
    ap.add_argument("--shuffle-blocks", type=int, default=0,
                    help="backward order = reverse registration order cut into blocks of this many "
                         "parameters, the blocks shuffled (0 = plain reverse order).  Every "
                         "configuration is then measured twice: with the default mapping and after "
                         "ddp_rebuild_buckets has followed the traced order (Section 6.2.1)")
    ap.add_argument("--flag-order", type=int, default=-1, choices=[-1, 0],
                    help="DDP_OPT_FLAG_ORDER: -1 = bucket launches are ordered after the backward stream "
                         "through device flags where the streams allow it, 0 = through events")
    ap.add_argument("--produce", action="store_true",
                    help="the synthetic backward also writes every gradient (copies it from a "
                         "source buffer after the delay), which keeps the memory system busy "
                         "the way a real backward pass does")
    args = ap.parse_args()

    import torch
    import workloads
    import paper_2006_15704_amd as lib
    from paper_2006_15704_amd import harness

    dtype = {"f32": 0, "f16": 1, "bf16": 2}[args.dtype]
    numel = workloads.numel_of(workloads.WORKLOAD_SHAPES[args.workload]())
    n, R = len(numel), args.replicas
    es = harness.ESIZE[dtype]
    B = sum(numel) * es
    grads = harness.DeviceGrads(numel, [dtype] * n, R)
    for r in range(R):
        grads.upload_replica(r, workloads.gaussian_replica(4, r, 0, numel, 1e-2, dtype))
    src_ptrs = None
    if args.produce:
        src = harness.DeviceGrads(numel, [dtype] * n, R, fill=0)
        src_ptrs = src.ptrs()
    torch.cuda.synchronize()
    order = list(range(n - 1, -1, -1))
    if args.shuffle_blocks > 0:
        import numpy as np
        blocks = [order[i:i + args.shuffle_blocks] for i in range(0, n, args.shuffle_blocks)]
        perm = np.random.default_rng(1).permutation(len(blocks))
        order = [p for b in perm for p in blocks[int(b)]]
    caps = [int(x) for x in args.caps_mib.split(",")]
    delays = [int(x) for x in args.delays_us.split(",")]

    stream_counts = [int(x) for x in args.streams.split(",")]
    for pipe, n_streams in itertools.product(args.pipelines.split(","), stream_counts):
        code = lib.DDP_PIPELINE_FUSED if pipe == "fused" else lib.DDP_PIPELINE_STAGED
        for cap_mib in caps:
            cap = lib.DDP_CAP_WHOLE_MODEL if cap_mib < 0 else cap_mib * MIB
            with harness.Session(grads, cap, code) as s:
                ctx = s.ctx
                lib.ddp_set_option(ctx, lib.DDP_OPT_EMIT_BUSY_BLOCKS, args.busy_blocks)
                lib.ddp_set_option(ctx, lib.DDP_OPT_REDUCE_STREAMS, n_streams)
                lib.ddp_set_option(ctx, lib.DDP_OPT_FLAG_ORDER, args.flag_order)
                by_flags = bool(lib.ddp_get_option(ctx, lib.DDP_OPT_FLAG_ORDER))
                lib.ddp_set_option(ctx, lib.DDP_OPT_COALESCE,
                                   (1 << 62) if args.coalesce_mib < 0 else int(args.coalesce_mib * MIB))
                lib.ddp_set_option(ctx, lib.DDP_OPT_LAUNCH_HOLD, args.hold)
                lib.ddp_set_option(ctx, lib.DDP_OPT_CHAIN_LAUNCHES, args.chain)

                def sync():
                    lib.ddp_synchronize(ctx)

                def sync_alone():
                    lib.ddp_synth_backward(ctx, order, None, None, True)
                    lib.ddp_finalize_backward(ctx)

                for mapping in (("default", "rebuilt") if args.shuffle_blocks > 0 else ("default",)):
                    if mapping == "rebuilt":
                        sync_alone()                       # leaves the trace of this order
                        sync()
                        n_buckets = lib.ddp_rebuild_buckets(ctx, cap)
                    else:
                        n_buckets = s.n_buckets
                    for _ in range(3):
                        sync_alone()
                    t_sync = timed(sync_alone, sync, args.reps, torch, s.backward_stream)
                    for d_us in delays:
                        dl = [d_us * 1000] * n

                        def backward_alone():
                            lib.ddp_synth_backward(ctx, order, dl, src_ptrs, False)

                        def backward_with_marks():
                            lib.ddp_synth_backward(ctx, order, dl, src_ptrs, True)

                        def finalize():
                            lib.ddp_finalize_backward(ctx)

                        t_bwd = timed(backward_alone, sync, args.reps, torch, s.backward_stream) if (d_us > 0 or src_ptrs) else 0.0
                        t_tot, after_marks = timed_exposed(backward_with_marks, finalize, sync, args.reps, torch,
                                                           s.backward_stream)
                        exposed = t_tot - t_bwd
                        print(json.dumps({
                            "workload": args.workload, "dtype": args.dtype, "R": R, "pipeline": pipe,
                            "cap_mib": cap_mib, "n_buckets": n_buckets, "streams": n_streams,
                            "coalesce_mib": args.coalesce_mib, "launch_hold": args.hold, "delay_us_per_param": d_us,
                            "order": f"blocks of {args.shuffle_blocks} shuffled" if args.shuffle_blocks else "reverse",
                            "mapping": mapping, "ordered_by": "flags" if by_flags else "events",
                            "backward_writes_gradients": bool(src_ptrs), "busy_blocks": args.busy_blocks,
                            "t_backward_ms": round(t_bwd, 4), "t_sync_ms": round(t_sync, 4),
                            "t_total_ms": round(t_tot, 4), "exposed_ms": round(exposed, 4),
                            "after_marks_ms": round(after_marks, 4),
                            "overlap": round(1.0 - exposed / t_sync, 3) if t_sync > 0 else None,
                            "sync_gbps_alg": round((R + 1) * B / t_sync / 1e6, 1),
                        }), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
