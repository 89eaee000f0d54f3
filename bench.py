#!/usr/bin/env python3
"""Benchmark of bucketed gradient synchronization on one MI355X.

One "step" is one pass of the whole hot path over one batch of synthetic
gradients, through the C ABI: ready marks for every parameter in reverse
registration order (each bucket is launched as soon as it is complete and its
predecessors have been launched), then the finalizing step.  The marks of a
step arrive in one call, so with the library's defaults consecutive buckets
share a kernel launch up to 100 MiB (DDP_OPT_COALESCE); the
`one_launch_per_bucket` and `two_streams` sub-objects report the same steps
with a launch per bucket.  Inputs are resident in HBM before the timed region
starts.  The default pipeline is the
one-pass (fused) one; `--pipeline staged` times the literal pack / reduce /
unpack pipeline instead, and the default run also reports the staged
pipeline's per-kernel rates in a `staged` sub-object.

Prints ONE JSON line.
  value     (R + W) * B / ms_per_step: every replica gradient read once, the
            average written W = 1 times -- the algorithmic end-to-end bytes of
            one synchronization divided by the measured step time.
  roofline  the reduce kernel (the dominant one) against the 8 TB/s HBM peak:
            algorithmic bytes per launch = (R + 1) * bytes of the buckets the
            launch covers, divided by the average launch duration: the time
            between two HIP events around the timed region (on the stream the
            launches run on or are waited for by) divided by the launches.
  cpu_baseline  the CPU oracle on the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0     # MI355X published HBM3E bandwidth

WORKLOADS = {
    # name: (shape list, config id, R, sigma, dtype code, cap bytes)
    "resnet50": ("resnet50", 2, 8, 1e-2, 0, 25 << 20),
    "bert_large": ("bert_large", 3, 8, 1e-3, 0, 25 << 20),
    "resnet50_fp16_r16": ("resnet50", 4, 16, 1e-2, 1, 25 << 20),      # the bucket-size sweep's configuration
    "bert_large_bf16": ("bert_large", 3, 8, 1e-3, 2, 25 << 20),        # diagnostic: 16-bit storage at BERT size
    "bert_large_r32": ("bert_large", 5, 32, 1e-3, 0, 25 << 20),        # configuration 5's reduction (R = 32)
    "tiny": ("tiny", 1, 2, 1.0, 0, 16384),
    "uniform": ("uniform", 9, 8, 1e-2, 0, 25 << 20),     # diagnostic: 40 single-tensor 25 MiB buckets
}


def generate_replicas(config_id, numel, R, sigma, dtype, threads=16):
    import workloads
    jobs = [(r, p) for r in range(R) for p in range(len(numel))]
    with ThreadPoolExecutor(max_workers=threads) as pool:
        flat = list(pool.map(
            lambda rp: workloads.gaussian_grad(config_id, rp[0], 0, rp[1], numel[rp[1]], sigma, dtype), jobs))
    n = len(numel)
    return [flat[r * n:(r + 1) * n] for r in range(R)]


def read_traffic(workload, pipeline):
    """HBM bytes per reduce launch from the committed counter summary, if any."""
    path = os.path.join(ROOT, "profiles", f"reduce_traffic_{workload}_{pipeline}.json")
    try:
        with open(path) as fh:
            return json.load(fh).get("traffic_bytes_per_launch")
    except Exception:
        return None


def measure(lib, harness, torch, grads, cap, pipeline_code, order, steps, warmup, timing_mode, args):
    """Runs warmup + `steps` timed steps on a fresh context; returns a dict."""
    with harness.Session(grads, cap, pipeline_code, same_stream=args.same_stream) as s:
        ctx = s.ctx
        if args.reduce_blocks is not None:
            lib.ddp_set_option(ctx, lib.DDP_OPT_REDUCE_BLOCKS, args.reduce_blocks)
        if args.plain_loads:
            lib.ddp_set_option(ctx, lib.DDP_OPT_NONTEMPORAL, 0)
        if args.unroll is not None:
            lib.ddp_set_option(ctx, lib.DDP_OPT_REDUCE_UNROLL, args.unroll)
        if args.copy_nt_store:
            lib.ddp_set_option(ctx, lib.DDP_OPT_COPY_NT_STORE, 1)
        if args.coalesce_mib is not None:
            lib.ddp_set_option(ctx, lib.DDP_OPT_COALESCE,
                               (1 << 62) if args.coalesce_mib < 0 else int(args.coalesce_mib * (1 << 20)))
        if args.streams is not None:
            lib.ddp_set_option(ctx, lib.DDP_OPT_REDUCE_STREAMS, args.streams)
        if args.tail_on_backward is not None:
            lib.ddp_set_option(ctx, lib.DDP_OPT_TAIL_ON_BACKWARD, args.tail_on_backward)
        if args.blocks_per_cu is not None:
            lib.ddp_set_option(ctx, lib.DDP_OPT_REDUCE_BLOCKS_PER_CU, args.blocks_per_cu)
        if args.copy_blocks_per_cu is not None:
            lib.ddp_set_option(ctx, lib.DDP_OPT_COPY_BLOCKS_PER_CU, args.copy_blocks_per_cu)
        if args.cap_min_mib is not None:
            lib.ddp_set_option(ctx, lib.DDP_OPT_REDUCE_CAP_MIN_BYTES, int(args.cap_min_mib * (1 << 20)))
        if args.pair_min_mib is not None:
            lib.ddp_set_option(ctx, lib.DDP_OPT_PAIR_MIN_BYTES, int(args.pair_min_mib * (1 << 20)))

        def step():
            lib.ddp_mark_ready_many(ctx, order)
            lib.ddp_finalize_backward(ctx)

        for _ in range(warmup):
            step()
        lib.ddp_synchronize(ctx)
        torch.cuda.synchronize()

        launches_per_step = None
        if timing_mode == "region":
            # one more untimed step with the library's per-iteration events, to count the launches
            lib.ddp_set_option(ctx, lib.DDP_OPT_TIMING, 2)
            step()
            lib.ddp_synchronize(ctx)
            launches_per_step = int(lib.ddp_get_kernel_times(ctx, lib.DDP_K_ITERATION)[1].sum())
            lib.ddp_set_option(ctx, lib.DDP_OPT_TIMING, 0)

        # timed region: `steps` steps.  "launch" / "iteration": the library's HIP events, one pair
        # per launch / per iteration, on the stream the kernels run on.  "region": one pair of HIP
        # events around all the steps on the backward stream -- every launch either runs on that
        # stream or is waited for by it in ddp_finalize_backward -- and no events in between.
        lib.ddp_set_option(ctx, lib.DDP_OPT_TIMING, {"launch": 1, "iteration": 2, "region": 0}[timing_mode])
        torch.cuda.synchronize()
        ev_a = torch.cuda.Event(enable_timing=True)
        ev_b = torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        ev_a.record(s.backward_stream)
        for _ in range(steps):
            step()
        ev_b.record(s.backward_stream)
        t_enq = time.perf_counter()
        lib.ddp_synchronize(ctx)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        res = {"ms_per_step": (t1 - t0) * 1e3 / steps,
               "host_enqueue_ms_per_step": (t_enq - t0) * 1e3 / steps,
               "region_ms": ev_a.elapsed_time(ev_b), "launches_per_step": launches_per_step}
        res["reduce"] = lib.ddp_get_kernel_times(ctx, lib.DDP_K_REDUCE)
        res["pack"] = lib.ddp_get_kernel_times(ctx, lib.DDP_K_PACK)
        res["unpack"] = lib.ddp_get_kernel_times(ctx, lib.DDP_K_UNPACK)
        res["iteration"] = lib.ddp_get_kernel_times(ctx, lib.DDP_K_ITERATION)
        lib.ddp_set_option(ctx, lib.DDP_OPT_TIMING, 0)
        res["bucket_elems"] = [lib.ddp_get_bucket_info(ctx, b)[0] for b in range(s.n_buckets)]
        res["n_buckets"] = s.n_buckets
    return res


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="resnet50", choices=sorted(WORKLOADS))
    ap.add_argument("--pipeline", default="fused", choices=["staged", "fused"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-staged-leg", action="store_true",
                    help="skip the extra measurement of the staged pipeline's kernels")
    ap.add_argument("--no-coalesce-leg", action="store_true",
                    help="skip the extra measurement with one launch per bucket")
    ap.add_argument("--no-streams-leg", action="store_true",
                    help="skip the extra measurement with two reduction streams")
    ap.add_argument("--no-accumulate-leg", action="store_true",
                    help="skip the extra measurement of the no_sync accumulation kernel")
    ap.add_argument("--reduce-blocks", type=int, default=None)
    ap.add_argument("--plain-loads", action="store_true")
    ap.add_argument("--unroll", type=int, default=None, choices=[1, 2, 4])
    ap.add_argument("--pair-min-mib", type=float, default=None,
                    help="fused pipeline: bucket size from which blocks take two tiles")
    ap.add_argument("--coalesce-mib", type=float, default=None,
                    help="buckets completed by one call share a launch up to this many MiB "
                         "(DDP_OPT_COALESCE; 0 = one launch per bucket, negative = no limit; "
                         "default: the library's, 100 MiB)")
    ap.add_argument("--streams", type=int, default=None,
                    help="reduction streams taken in turn by the bucket launches (DDP_OPT_REDUCE_STREAMS)")
    ap.add_argument("--tail-on-backward", type=int, default=None, choices=[0, 1],
                    help="DDP_OPT_TAIL_ON_BACKWARD: 1 (library default) = the launches of the call that "
                         "completes an iteration go to the backward stream; 0 = always a reduction stream")
    ap.add_argument("--blocks-per-cu", type=int, default=None,
                    help="reduce kernels: resident thread blocks per compute unit "
                         "(DDP_OPT_REDUCE_BLOCKS_PER_CU; 0 = no cap)")
    ap.add_argument("--copy-blocks-per-cu", type=int, default=None,
                    help="pack / unpack / accumulate kernels: resident blocks per compute unit "
                         "(DDP_OPT_COPY_BLOCKS_PER_CU; 0 = no cap)")
    ap.add_argument("--acc-blocks-per-cu", type=int, default=None,
                    help="accumulate kernel: resident blocks per compute unit "
                         "(DDP_OPT_ACCUMULATE_BLOCKS_PER_CU; 0 = no cap)")
    ap.add_argument("--cap-min-mib", type=float, default=None,
                    help="launch size from which that cap applies (DDP_OPT_REDUCE_CAP_MIN_BYTES)")
    ap.add_argument("--copy-nt-store", action="store_true",
                    help="staged pipeline: pack/unpack store with the non-temporal hint")
    ap.add_argument("--same-stream", action="store_true",
                    help="use one stream for backward and reduction (no event plumbing)")
    ap.add_argument("--timing", default=None, choices=["launch", "iteration", "region"],
                    help="HIP-event granularity in the timed region: one pair per kernel launch "
                         "(default for staged), one pair around each iteration's bucket launches, or "
                         "one pair around all the steps (default for fused, where the reduce launches "
                         "are the only kernels: no event between them)")
    ap.add_argument("--cap-mib", type=float, default=None,
                    help="override the bucket cap (MiB; negative = whole model)")
    ap.add_argument("--replicas", type=int, default=None,
                    help="diagnostic: override the workload's number of replicas R")
    ap.add_argument("--uniform", default=None,
                    help="diagnostic workload 'count,elems': that many equal tensors (with --workload uniform)")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run a plain 1 GiB device copy (for scaling profiler counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the R replicas are R buffers in one GPU's "
              "HBM); --gpus above 1 is not supported and nothing was measured", file=sys.stderr)
        return 2

    import torch
    import workloads
    import __graft_entry__
    __graft_entry__.ensure_built()          # a fresh checkout has no library yet
    import paper_2006_15704_amd as lib
    from paper_2006_15704_amd import harness

    shape_name, config_id, R, sigma, dtype, cap = WORKLOADS[args.workload]
    if args.replicas is not None:
        R = args.replicas
    if args.cap_mib is not None:
        cap = lib.DDP_CAP_WHOLE_MODEL if args.cap_mib < 0 else int(args.cap_mib * (1 << 20))
    if args.workload == "uniform" and args.uniform:
        count, elems = (int(x) for x in args.uniform.split(","))
        numel = workloads.numel_of(workloads.uniform_shapes(count, elems))
    else:
        numel = workloads.numel_of(workloads.WORKLOAD_SHAPES[shape_name]())
    n = len(numel)
    es = harness.ESIZE[dtype]
    B = sum(numel) * es
    W = 1
    codes = {"staged": lib.DDP_PIPELINE_STAGED, "fused": lib.DDP_PIPELINE_FUSED}
    timing = args.timing or ("region" if args.pipeline == "fused" else "launch")

    reps = generate_replicas(config_id, numel, R, sigma, dtype)
    grads = harness.DeviceGrads(numel, [dtype] * n, R)
    for r in range(R):
        grads.upload_replica(r, reps[r])
    torch.cuda.synchronize()

    if args.calibration_copy:
        src = torch.zeros(1 << 30, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    order = list(range(n - 1, -1, -1))
    m = measure(lib, harness, torch, grads, cap, codes[args.pipeline], order, args.steps, args.warmup,
                timing, args)
    ms_per_step = m["ms_per_step"]
    bucket_elems, n_buckets = m["bucket_elems"], m["n_buckets"]
    red_ms, red_ids = m["reduce"]
    iter_ms, iter_launches = m["iteration"]

    def launch_elems(ident):
        """elements covered by a launch id (first bucket + 65536 * further buckets)"""
        first, extra = int(ident) % 65536, int(ident) // 65536
        return sum(bucket_elems[first:first + extra + 1])

    # reduce kernel: algorithmic bytes per launch = (R + 1) * bucket bytes
    per_bucket = {}
    if timing == "launch":
        launches = len(red_ms)
        total_alg = float(sum((R + 1) * launch_elems(b) * es for b in red_ids))
        total_ms = float(red_ms.sum())
        for b in range(n_buckets):
            sel = red_ms[red_ids == b]
            if len(sel):
                per_bucket[str(b)] = round((R + 1) * bucket_elems[b] * es / float(np.median(sel)) / 1e6, 1)
    elif timing == "iteration":
        # one interval per iteration holding all its bucket launches; in the
        # fused pipeline they are the only kernels inside it
        launches = int(iter_launches.sum())
        total_alg = float((R + 1) * B * len(iter_ms))
        total_ms = float(iter_ms.sum())
    else:
        # one interval around all the steps (fused pipeline: the reduce launches are its only
        # kernels); the gaps between consecutive launches are part of it
        launches = m["launches_per_step"] * args.steps
        total_alg = float((R + 1) * B * args.steps)
        total_ms = float(m["region_ms"])
    avg_launch_ms = total_ms / max(launches, 1)
    achieved = total_alg / max(total_ms, 1e-12) / 1e6          # bytes / ms -> GB/s

    value = (R + W) * B / ms_per_step / 1e6
    out = {
        "metric": "bucketed grad-sync throughput ((R+W)*B per synchronization)",
        "value": round(value, 2),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": {0: "f32", 1: "f16", 2: "bf16"}[dtype],
        "data": "synthetic",
        "config": {"workload": f"{args.workload}: {n} tensors, {sum(numel)} elements, R={R}, "
                               f"cap={cap} B, {n_buckets} buckets, ready order = reverse registration",
                   "pipeline": args.pipeline, "R": R, "W": W, "bucket_cap_bytes": cap},
        "pct_hbm_peak_end_to_end": round(100.0 * value / HBM_PEAK_GBPS, 2),
        "host_enqueue_ms_per_step": round(m["host_enqueue_ms_per_step"], 4),
        "kernel_ms_per_step": {
            "pack": round(float(m["pack"][0].sum()) / args.steps, 4),
            "reduce": round(total_ms / args.steps, 4),
            "unpack": round(float(m["unpack"][0].sum()) / args.steps, 4),
        },
        "roofline": {
            "kernel": "flat_reduce_kernel" if args.pipeline == "staged" else "fused_reduce_kernel",
            "bound": "hbm",
            "achieved": round(achieved, 1),
            "peak": HBM_PEAK_GBPS,
            "unit": "GB/s",
            "frac": round(achieved / HBM_PEAK_GBPS, 4),
            "avg_launch_ms": round(avg_launch_ms, 5),
            "launches": launches,
            "timing": ("one HIP event pair around the timed region" if timing == "region"
                       else "HIP event pair per " + timing),
            "interval_ms": ({"median": round(float(np.median(iter_ms)), 5), "min": round(float(iter_ms.min()), 5),
                             "max": round(float(iter_ms.max()), 5), "what": "one iteration's launches"}
                            if timing == "iteration" and len(iter_ms) else
                            {"median": round(float(np.median(red_ms)), 5), "min": round(float(red_ms.min()), 5),
                             "max": round(float(red_ms.max()), 5), "what": "one launch"}
                            if timing == "launch" and len(red_ms) else None),
            "algorithmic_bytes_per_launch": round(total_alg / max(launches, 1)),
            "traffic": read_traffic(args.workload, args.pipeline),
        },
    }
    if per_bucket:
        out["reduce_gbps_per_bucket"] = per_bucket
    if timing == "region":
        # a short second pass with one event pair per iteration, for the spread
        it = measure(lib, harness, torch, grads, cap, codes[args.pipeline], order, max(10, args.steps // 5), 2,
                     "iteration", args)
        it_ms, it_launches = it["iteration"]
        out["roofline"]["per_iteration_pass"] = {
            "interval_ms": {"median": round(float(np.median(it_ms)), 5), "min": round(float(it_ms.min()), 5),
                            "max": round(float(it_ms.max()), 5)},
            "reduce_gbps": round((R + 1) * B * len(it_ms) / float(it_ms.sum()) / 1e6, 1),
            "what": "one HIP event pair per iteration around its launches (the pairs cost a few us each)",
        }

    if args.pipeline == "fused" and not args.no_staged_leg:
        # the literal three-kernel pipeline on the same data, one event pair per launch
        steps2 = max(5, args.steps // 2)
        st = measure(lib, harness, torch, grads, cap, codes["staged"], order, steps2, 2, "launch", args)
        s_red_ms, s_red_ids = st["reduce"]
        red_alg = float(sum((R + 1) * launch_elems(b) * es for b in s_red_ids))
        out["staged"] = {
            "ms_per_step": round(st["ms_per_step"], 4),
            "value_gbps": round((R + W) * B / st["ms_per_step"] / 1e6, 1),
            "pack_gbps": round(2.0 * R * B * steps2 / float(st["pack"][0].sum()) / 1e6, 1),
            "reduce_gbps": round(red_alg / float(s_red_ms.sum()) / 1e6, 1),
            "unpack_gbps": round((1.0 + W) * B * steps2 / float(st["unpack"][0].sum()) / 1e6, 1),
            "bytes": "pack 2RB, reduce (R+1)B, unpack (1+W)B per step",
            "steps": steps2,
        }

    if args.pipeline == "fused" and args.coalesce_mib is None and not args.no_coalesce_leg:
        # the same steps with one launch per bucket on the reduction stream (DDP_OPT_COALESCE = 0,
        # DDP_OPT_TAIL_ON_BACKWARD = 0), as when the ready marks arrive in separate calls during a
        # real backward pass
        args.coalesce_mib = 0.0
        keep_tail, args.tail_on_backward = args.tail_on_backward, 0
        pb = measure(lib, harness, torch, grads, cap, codes["fused"], order, args.steps, 2, "iteration", args)
        args.coalesce_mib, args.tail_on_backward = None, keep_tail
        pb_ms, pb_launches = pb["iteration"]
        per_bucket_gbps = None
        if n_buckets <= 64:
            # a few more steps with one event pair per launch: the rate of every bucket
            args.coalesce_mib, args.tail_on_backward = 0.0, 0
            pl = measure(lib, harness, torch, grads, cap, codes["fused"], order, max(5, args.steps // 5), 2, "launch", args)
            args.coalesce_mib, args.tail_on_backward = None, keep_tail
            l_ms, l_ids = pl["reduce"]
            per_bucket_gbps = {str(b): round((R + 1) * bucket_elems[b] * es / float(np.median(l_ms[l_ids == b])) / 1e6, 1)
                               for b in range(n_buckets) if (l_ids == b).any()}
        out["one_launch_per_bucket"] = {
            "reduce_gbps_per_bucket": per_bucket_gbps,
            "per_bucket_note": "median over steps, one HIP event pair per launch (the pair adds about 3 us to each)",
            "ms_per_step": round(pb["ms_per_step"], 4),
            "value_gbps": round((R + W) * B / pb["ms_per_step"] / 1e6, 1),
            "launches_per_step": int(pb_launches.sum()) // args.steps,
            "reduce_gbps": round((R + 1) * B * len(pb_ms) / float(pb_ms.sum()) / 1e6, 1),
            "frac_of_hbm_peak": round((R + 1) * B * len(pb_ms) / float(pb_ms.sum()) / 1e6 / HBM_PEAK_GBPS, 4),
        }

    if args.pipeline == "fused" and args.streams is None and not args.no_streams_leg:
        # one launch per bucket, the launches alternating between two reduction streams
        # (DDP_OPT_REDUCE_STREAMS): neighbouring buckets overlap, so only the iteration as a
        # whole has a duration
        args.streams = 2
        keep_coalesce, args.coalesce_mib = args.coalesce_mib, 0.0
        keep_tail, args.tail_on_backward = args.tail_on_backward, 0
        rr = measure(lib, harness, torch, grads, cap, codes["fused"], order, args.steps, 2, "iteration", args)
        args.streams, args.coalesce_mib, args.tail_on_backward = None, keep_coalesce, keep_tail
        rr_ms, _ = rr["iteration"]
        out["two_streams"] = {
            "ms_per_step": round(rr["ms_per_step"], 4),
            "value_gbps": round((R + W) * B / rr["ms_per_step"] / 1e6, 1),
            "reduce_gbps": round((R + 1) * B * len(rr_ms) / float(rr_ms.sum()) / 1e6, 1),
            "frac_of_hbm_peak": round((R + 1) * B * len(rr_ms) / float(rr_ms.sum()) / 1e6 / HBM_PEAK_GBPS, 4),
            "note": "one launch per bucket; (R+1)*B per iteration / time from the first launch to the join of both streams",
        }

    if not args.no_accumulate_leg:
        # no_sync micro-step: grad[r][i] += micro[r][i] for all replicas, 3*R*B bytes
        micro = harness.DeviceGrads(numel, [dtype] * n, R, fill=0)
        ptrs = micro.ptrs()
        with harness.Session(grads, cap, codes[args.pipeline]) as s:
            if args.acc_blocks_per_cu is not None:
                lib.ddp_set_option(s.ctx, lib.DDP_OPT_ACCUMULATE_BLOCKS_PER_CU, args.acc_blocks_per_cu)
            for _ in range(2):
                lib.ddp_no_sync_accumulate(s.ctx, ptrs)
            lib.ddp_synchronize(s.ctx)
            lib.ddp_set_option(s.ctx, lib.DDP_OPT_TIMING, 1)
            reps_acc = 10
            for _ in range(reps_acc):
                lib.ddp_no_sync_accumulate(s.ctx, ptrs)
            lib.ddp_synchronize(s.ctx)
            acc_ms, _ = lib.ddp_get_kernel_times(s.ctx, lib.DDP_K_ACCUMULATE)
        out["no_sync_accumulate"] = {
            "ms_per_micro_step": round(float(acc_ms.mean()), 4),
            "gbps": round(3.0 * R * B / float(acc_ms.mean()) / 1e6, 1),
            "bytes": "3*R*B per micro-step (read gradient and micro-gradient, write gradient)",
        }
        del micro

    if not args.no_cpu_baseline:
        import oracle
        t0 = time.perf_counter()
        done = 0
        while True:
            oracle.synchronize(numel, [dtype] * n, cap, reps)
            done += 1
            if time.perf_counter() - t0 > 10.0 or done >= 20:
                break
        cpu_ms = (time.perf_counter() - t0) * 1e3 / done
        out["cpu_baseline"] = {
            "value": round((R + W) * B / cpu_ms / 1e6, 3),
            "unit": "GB/s",
            "cores": 1,
            "kind": "oracle",
            "ms_per_step": round(cpu_ms, 2),
            "sample": f"{done} full synchronizations of the same {args.workload} workload "
                      f"(all {n_buckets} buckets, R={R}) by the numpy oracle, single thread",
            "host_cores_visible": os.cpu_count(),
            "numpy": np.__version__,
        }
    else:
        out["cpu_baseline"] = None
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
