#!/usr/bin/env python3
"""Benchmark of bucketed gradient synchronization on one MI355X.

One "step" is one pass of the whole hot path over one batch of synthetic
gradients, through the C ABI, the way a backward pass drives it (Algorithm 1):
one ddp_mark_ready call per parameter, in reverse registration order -- every
bucket is launched by the call that completes it, on the reduction streams --
and then ddp_finalize_backward.  Library defaults throughout.  Inputs are
resident in HBM before the timed region starts, and consecutive steps work on
different sets of replica gradients (four sets, several GB), so that the
256 MB Infinity Cache cannot serve a step from what the previous one left.

Prints ONE JSON line.
  value     (R + W) * B / ms_per_step for the ResNet-50-shaped list (R = 8):
            every replica gradient read once, the average written W = 1 times,
            divided by the wall-clock time of a step.
  roofline  the reduce kernel (fused_reduce_kernel, the dominant one) against
            the 8 TB/s HBM peak: algorithmic bytes per launch = (R + 1) * bytes
            of the bucket(s) a launch covers; average launch duration = the time
            between two HIP events around the timed steps (on the backward
            stream, which every launch runs on or is joined to by finalize)
            divided by the number of launches -- the launches of a step run on
            two reduction streams and overlap at their ends, so this is the
            duration that adds up to the whole, gates, joins and gaps included.
  bert_large    the same measurement on the BERT-large-shaped list (the metric
            is quoted on both shapes).
  marks_in_one_call   both shapes again with all marks of a step in ONE
            ddp_mark_ready_many call (consecutive buckets then share launches).
  overlap   configuration 4 in short: ResNet-50 shape in fp16, R = 16, a synthetic
            backward stream of one 10 us kernel per parameter; exposed time of
            the synchronization per bucket cap.
  bert_large_r32   configuration 5's reduction (R = 32) and no_sync accumulation.
  cpu_baseline  the CPU oracle on a bounded sample of the headline workload,
            one thread and all host cores.
"""
from __future__ import annotations

import argparse
import json
import os
import statistics
import sys
import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0     # MI355X published HBM3E bandwidth
MIB = 1 << 20

WORKLOADS = {
    # name: (shape list, config id, R, sigma, dtype code, cap bytes)
    "resnet50": ("resnet50", 2, 8, 1e-2, 0, 25 * MIB),
    "bert_large": ("bert_large", 3, 8, 1e-3, 0, 25 * MIB),
    "resnet50_fp16_r16": ("resnet50", 4, 16, 1e-2, 1, 25 * MIB),      # the bucket-size sweep's configuration
    "bert_large_r32": ("bert_large", 5, 32, 1e-3, 0, 25 * MIB),        # configuration 5's reduction (R = 32)
    "bert_large_bf16": ("bert_large", 3, 8, 1e-3, 2, 25 * MIB),        # 16-bit transport of BERT-large's gradients
}
ALL_LEGS = ["headline", "bert_large", "one_call", "hold", "single_set", "per_bucket", "overlap", "r32", "transport",
            "staged", "accumulate", "cpu"]
DT_NAME = {0: "f32", 1: "f16", 2: "bf16"}


def device_grads(harness, torch, numel, dtype, R, sigma, seed, fill_noise=True):
    """R replica buffers with seeded Gaussian gradients generated on the device
    (the same distribution as the host recipe of the parity tests; the bits
    differ, which no throughput figure depends on)."""
    n = len(numel)
    g = harness.DeviceGrads(numel, [dtype] * n, R)
    if fill_noise:
        gen = torch.Generator(device="cuda")
        gen.manual_seed(seed)
        for r in range(R):
            buf = g.bufs[r]
            usable = buf.numel() // 4 * 4
            if dtype == 0:
                buf[:usable].view(torch.float32).normal_(0.0, sigma, generator=gen)
            elif dtype == 1:
                buf[:usable].view(torch.float16).normal_(0.0, sigma, generator=gen)
            else:
                buf[:usable].view(torch.bfloat16).normal_(0.0, sigma, generator=gen)
    return g


def read_traffic(workload, mode):
    """HBM bytes per reduce launch from the committed counter summary, if any."""
    path = os.path.join(ROOT, "profiles", f"reduce_traffic_{workload}_{mode}.txt")
    try:
        with open(path) as fh:
            return json.load(fh).get("traffic_bytes_per_launch")
    except Exception:
        return None


def spread(values):
    v = [float(x) for x in values]
    return {"median": round(statistics.median(v), 5), "min": round(min(v), 5), "max": round(max(v), 5), "n": len(v)}


class Rig:
    """`sets` independent sets of replica gradients of one workload, one context
    per set, all contexts on the same pair of streams."""

    every_rig_options = ()        # (option, value) pairs applied to every context (--launch-ordering)

    def __init__(self, lib, harness, torch, workload, sets, pipeline, options=(), same_stream=False,
                 binary32_outputs=False):
        self.lib, self.torch = lib, torch
        shape_name, self.config_id, self.R, self.sigma, self.dtype, self.cap = WORKLOADS[workload]
        import workloads
        self.numel = workloads.numel_of(workloads.WORKLOAD_SHAPES[shape_name]())
        self.n = len(self.numel)
        self.es = harness.ESIZE[self.dtype]
        self.B = sum(self.numel) * self.es
        self.order = list(range(self.n - 1, -1, -1))
        self.grads = [device_grads(harness, torch, self.numel, self.dtype, self.R, self.sigma, 1000 * self.config_id + k)
                      for k in range(sets)]
        # bytes a synchronization has to move: every replica gradient read once, the average written once
        self.alg_bytes = (self.R + 1) * self.B
        self.outputs = [None] * sets
        if binary32_outputs:         # 16-bit gradients in, binary32 averages out (Section 6.2.3)
            self.outputs = [harness.DeviceGrads(self.numel, [0] * self.n, 1) for _ in range(sets)]
            self.alg_bytes = self.R * self.B + 4 * sum(self.numel)
        self.sessions = []
        streams = None
        for g, o in zip(self.grads, self.outputs):
            s = harness.Session(g, self.cap, pipeline, same_stream=same_stream, streams=streams, outputs=o)
            streams = (s.reduce_stream, s.backward_stream)
            for opt, val in tuple(Rig.every_rig_options) + tuple(options):
                lib.ddp_set_option(s.ctx, opt, val)
            self.sessions.append(s)
        self.backward_stream = self.sessions[0].backward_stream
        self.n_buckets = self.sessions[0].n_buckets
        self.bucket_elems = [lib.ddp_get_bucket_info(self.sessions[0].ctx, b)[0] for b in range(self.n_buckets)]
        self.flag_order = bool(lib.ddp_get_option(self.sessions[0].ctx, lib.DDP_OPT_FLAG_ORDER))

    def close(self):
        for s in self.sessions:
            s.close()
        self.sessions, self.grads, self.outputs = [], [], []

    def step(self, k, per_call):
        ctx = self.sessions[k % len(self.sessions)].ctx
        lib = self.lib
        if per_call:
            mark = lib.ddp_mark_ready
            for p in self.order:
                mark(ctx, p)
        else:
            lib.ddp_mark_ready_many(ctx, self.order)
        lib.ddp_finalize_backward(ctx)

    def sync(self):
        for s in self.sessions:
            self.lib.ddp_synchronize(s.ctx)
        self.torch.cuda.synchronize()

    def measure(self, steps, warmup, per_call, spread_iters=20):
        """warmup + `steps` timed steps; then a pass with one HIP event pair per
        iteration for the spread.  Returns a dict."""
        lib, torch = self.lib, self.torch
        S = len(self.sessions)
        for k in range(max(warmup, S)):
            self.step(k, per_call)
        self.sync()
        # launches per step, counted by the library's per-iteration events on one untimed step
        ctx0 = self.sessions[0].ctx
        lib.ddp_set_option(ctx0, lib.DDP_OPT_TIMING, 2)
        self.step(0, per_call)
        self.sync()
        launches_per_step = int(lib.ddp_get_kernel_times(ctx0, lib.DDP_K_ITERATION)[1].sum())
        lib.ddp_set_option(ctx0, lib.DDP_OPT_TIMING, 0)
        # The timed region: exactly `steps` steps between two host synchronizations, no event
        # between the steps.  It is run three times and the median run is reported (all three are
        # listed): the box now and then stalls a process for tens of milliseconds, which would
        # otherwise decide a figure that is a fraction of a millisecond per step.
        runs = []
        for _ in range(3):
            ev_a = torch.cuda.Event(enable_timing=True)
            ev_b = torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            ev_a.record(self.backward_stream)
            for k in range(steps):
                self.step(k, per_call)
            ev_b.record(self.backward_stream)
            t_enq = time.perf_counter()
            self.sync()
            t1 = time.perf_counter()
            runs.append((t1 - t0, t_enq - t0, ev_a.elapsed_time(ev_b)))
        all_runs_ms = [round(r[0] * 1e3 / steps, 4) for r in runs]
        wall_s, enq_s, region_ms = sorted(runs)[1]
        t0, t1, t_enq = 0.0, wall_s, enq_s
        # spread: one event pair per iteration (each pair costs a few microseconds)
        for s in self.sessions:
            lib.ddp_set_option(s.ctx, lib.DDP_OPT_TIMING, 2)
        for k in range(spread_iters):
            self.step(k, per_call)
        self.sync()
        it_ms = np.concatenate([lib.ddp_get_kernel_times(s.ctx, lib.DDP_K_ITERATION)[0] for s in self.sessions])
        # the reduce kernel by itself: every launch carries an event pair stamped with its start and end
        for s in self.sessions:
            lib.ddp_set_option(s.ctx, lib.DDP_OPT_TIMING, 1)
        for k in range(spread_iters):
            self.step(k, per_call)
        self.sync()
        k_ms = np.concatenate([lib.ddp_get_kernel_times(s.ctx, lib.DDP_K_REDUCE)[0] for s in self.sessions])
        for s in self.sessions:
            lib.ddp_set_option(s.ctx, lib.DDP_OPT_TIMING, 0)
        alg = self.alg_bytes
        ms_per_step = (t1 - t0) * 1e3 / steps
        launches = launches_per_step * steps
        # The launches of an iteration run on two reduction streams and overlap each other at
        # their ends, so "the duration of a launch" that sums up to the time of the whole is
        # the time of the timed region divided by its launches; what one launch takes between
        # its own two events (it shares the memory system with its neighbour meanwhile) is
        # reported next to it.
        avg_launch_ms = region_ms / max(launches, 1)
        achieved = alg * steps / region_ms / 1e6
        return {
            "ms_per_step": round(ms_per_step, 4),
            "ms_per_step_all_runs": all_runs_ms,
            "value_gbps": round(alg / ms_per_step / 1e6, 1),
            "pct_hbm_peak_end_to_end": round(100.0 * alg / ms_per_step / 1e6 / HBM_PEAK_GBPS, 2),
            "host_enqueue_ms_per_step": round((t_enq - t0) * 1e3 / steps, 4),
            "launches_per_step": launches_per_step,
            "repaired_launches": int(sum(lib.ddp_get_option(s.ctx, lib.DDP_STAT_REPAIRED_LAUNCHES) for s in self.sessions)),
            "roofline": {
                "kernel": "fused_reduce_kernel",
                "bound": "hbm",
                "achieved": round(achieved, 1),
                "peak": HBM_PEAK_GBPS,
                "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBPS, 4),
                "avg_launch_ms": round(avg_launch_ms, 5),
                "launches": launches,
                "algorithmic_bytes_per_launch": round(alg / max(launches_per_step, 1)),
                "timing": "one HIP event pair around the timed steps on the backward stream (every launch runs on it "
                          "or is joined to it by finalize), divided by the launches: kernels, gates, joins and gaps",
                "per_launch_event_pairs": {
                    "what": f"every launch carries a pair of HIP events stamped with the kernel's own start and end "
                            f"(third pass of {spread_iters} steps); launches on the two reduction streams overlap, each "
                            "then takes longer than its share",
                    "launch_ms": spread(k_ms),
                    "mean_ms": round(float(k_ms.mean()), 5)},
                "iteration_ms": spread(it_ms),
                "iteration_what": "first bucket launch to the end of the iteration, one HIP event pair per "
                                  "iteration (second pass; the pairs cost a few us each)",
            },
        }

    def per_bucket(self, steps):
        """Every bucket in a launch of its own, the launches back to back on one reduction stream
        (all marks of a step in one call, so that no host latency sits between the launches; the
        stream is ordered behind the backward stream by one event per step, so that no gate kernel
        sits between the bucket kernels).  Every launch carries a pair of HIP events that the
        runtime stamps with the kernel's own start and end; the iteration as a whole is timed
        once more without any per-launch events."""
        lib, torch = self.lib, self.torch
        one_stream = ((lib.DDP_OPT_REDUCE_STREAMS, 1), (lib.DDP_OPT_COALESCE, 0),
                      (lib.DDP_OPT_TAIL_ON_BACKWARD, 0), (lib.DDP_OPT_FLAG_ORDER, 0))
        defaults = ((lib.DDP_OPT_REDUCE_STREAMS, -1), (lib.DDP_OPT_COALESCE, -1),
                    (lib.DDP_OPT_TAIL_ON_BACKWARD, 1), (lib.DDP_OPT_FLAG_ORDER, -1)) + tuple(Rig.every_rig_options)
        for s in self.sessions:
            for o, v in one_stream:
                lib.ddp_set_option(s.ctx, o, v)
        for k in range(len(self.sessions)):
            self.step(k, False)
        self.sync()
        region = []
        for _ in range(3):
            a = torch.cuda.Event(enable_timing=True)
            b = torch.cuda.Event(enable_timing=True)
            a.record(self.backward_stream)
            for k in range(steps):
                self.step(k, False)
            b.record(self.backward_stream)
            self.sync()
            region.append(a.elapsed_time(b) / steps)
        it_ms = sorted(region)[1]
        for s in self.sessions:
            lib.ddp_set_option(s.ctx, lib.DDP_OPT_TIMING, 1)
        for k in range(steps):
            self.step(k, False)
        self.sync()
        ms = np.concatenate([lib.ddp_get_kernel_times(s.ctx, lib.DDP_K_REDUCE)[0] for s in self.sessions])
        ids = np.concatenate([lib.ddp_get_kernel_times(s.ctx, lib.DDP_K_REDUCE)[1] for s in self.sessions])
        for s in self.sessions:
            lib.ddp_set_option(s.ctx, lib.DDP_OPT_TIMING, 0)
            for o, v in defaults:
                lib.ddp_set_option(s.ctx, o, v)
        out, us = {}, {}
        for b in range(self.n_buckets):
            sel = ms[ids == b]
            if len(sel):
                out[str(b)] = round((self.R + 1) * self.bucket_elems[b] * self.es / float(np.median(sel)) / 1e6, 1)
                us[str(b)] = round(float(np.median(sel)) * 1e3, 2)
        total = self.alg_bytes * steps / float(ms.sum()) / 1e6
        return {"reduce_gbps_per_bucket": out, "kernel_us_per_bucket": us, "reduce_gbps": round(total, 1),
                "frac_of_hbm_peak": round(total / HBM_PEAK_GBPS, 4),
                "iteration_ms": round(it_ms, 4),
                "iteration_gbps": round(self.alg_bytes / it_ms / 1e6, 1),
                "iteration_frac_of_hbm_peak": round(self.alg_bytes / it_ms / 1e6 / HBM_PEAK_GBPS, 4),
                "bucket_mib": [round(e * self.es / MIB, 2) for e in self.bucket_elems],
                "note": "one reduction stream ordered by events, one launch per bucket, launches queued back to back. "
                        "reduce_gbps*: from the kernels' own start and end stamps (median over steps per bucket; "
                        "reduce_gbps over the sum of all kernel durations). iteration_*: the same steps without "
                        "per-launch events, HIP events on the backward stream around the timed steps (median of three "
                        "regions): kernels, the gaps between them, the cross-stream order at the start of a step and "
                        "the join at its end"}


def shape_leg(lib, harness, torch, workload, sets, steps, warmup, legs, traffic_mode, options=()):
    """The per-call measurement of one workload plus its optional sub-legs."""
    rig = Rig(lib, harness, torch, workload, sets, lib.DDP_PIPELINE_FUSED, options=options)
    try:
        res = rig.measure(steps, warmup, per_call=True)
        res["roofline"]["traffic"] = read_traffic(workload, traffic_mode)
        res["config"] = {"workload": f"{workload}: {rig.n} tensors, {sum(rig.numel)} elements, R={rig.R}, "
                                     f"cap={rig.cap} B, {rig.n_buckets} buckets, ready order = reverse registration, "
                                     f"one ddp_mark_ready call per parameter",
                         "pipeline": "fused", "R": rig.R, "W": 1, "bucket_cap_bytes": rig.cap,
                         "replica_sets_rotated": sets,
                         "working_set_gb": round(sets * rig.R * rig.B / 1e9, 2),
                         "launch_ordering": "device flags" if rig.flag_order else "events"}
        if "one_call" in legs:
            one = rig.measure(steps, warmup, per_call=False)
            one["what"] = "all marks of a step in one ddp_mark_ready_many call: consecutive buckets share launches"
            res["marks_in_one_call"] = one
        if "hold" in legs:
            for s in rig.sessions:
                lib.ddp_set_option(s.ctx, lib.DDP_OPT_LAUNCH_HOLD, 16)
            held = rig.measure(steps, warmup, per_call=True)
            for s in rig.sessions:
                lib.ddp_set_option(s.ctx, lib.DDP_OPT_LAUNCH_HOLD, 0)
            held["what"] = ("one ddp_mark_ready call per parameter with DDP_OPT_LAUNCH_HOLD = 16: a launchable bucket waits "
                            "for up to 16 further marks so that its successors can share its launch")
            res["marks_one_by_one_hold_16"] = held
        if "per_bucket" in legs and rig.n_buckets <= 64:
            res["one_launch_per_bucket"] = rig.per_bucket(max(5, steps // 2))
    finally:
        rig.close()
    if "single_set" in legs:
        rig = Rig(lib, harness, torch, workload, 1, lib.DDP_PIPELINE_FUSED)
        try:
            one = rig.measure(steps, warmup, per_call=True)
            res["single_replica_set"] = {k: one[k] for k in ("ms_per_step", "value_gbps")}
            res["single_replica_set"]["reduce_frac"] = one["roofline"]["frac"]
            res["single_replica_set"]["what"] = ("every step works on the same addresses: part of a step is served "
                                                 "from the Infinity Cache")
        finally:
            rig.close()
    return res


def overlap_leg(lib, harness, torch, reps=10, delay_us=10):
    """Configuration 4 in short (Section 5.1 / 5.2 in one-GPU form): exposed time of the synchronization
    under a synthetic backward pass of one `delay_us` kernel per parameter."""
    import workloads
    shape_name, config_id, R, sigma, dtype, _ = WORKLOADS["resnet50_fp16_r16"]
    numel = workloads.numel_of(workloads.WORKLOAD_SHAPES[shape_name]())
    n = len(numel)
    B = sum(numel) * harness.ESIZE[dtype]
    grads = device_grads(harness, torch, numel, dtype, R, sigma, 4000)
    order = list(range(n - 1, -1, -1))
    delays = [delay_us * 1000] * n
    rows = []
    for cap_mib in (1, 5, 10, 25, -1):
        cap = lib.DDP_CAP_WHOLE_MODEL if cap_mib < 0 else cap_mib * MIB
        with harness.Session(grads, cap, lib.DDP_PIPELINE_FUSED) as s:
            ctx, stream = s.ctx, s.backward_stream
            lib.ddp_set_option(ctx, lib.DDP_OPT_COALESCE, 0)          # one launch per bucket

            def timed(fn):
                out = []
                for _ in range(reps):
                    lib.ddp_synchronize(ctx)
                    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    a.record(stream)
                    fn()
                    b.record(stream)
                    lib.ddp_synchronize(ctx)
                    b.synchronize()
                    out.append(a.elapsed_time(b))
                return statistics.median(out)

            def sync_alone():
                lib.ddp_synth_backward(ctx, order, None, None, True)
                lib.ddp_finalize_backward(ctx)

            def backward_alone():
                lib.ddp_synth_backward(ctx, order, delays, None, False)

            def backward_and_sync():
                lib.ddp_synth_backward(ctx, order, delays, None, True)
                lib.ddp_finalize_backward(ctx)

            for _ in range(3):
                sync_alone()
            t_sync, t_bwd, t_tot = timed(sync_alone), timed(backward_alone), timed(backward_and_sync)
            row = {"cap_mib": cap_mib, "buckets": s.n_buckets, "sync_alone_ms": round(t_sync, 4),
                   "backward_alone_ms": round(t_bwd, 4), "exposed_ms": round(t_tot - t_bwd, 4),
                   "overlap": round(1.0 - (t_tot - t_bwd) / t_sync, 3),
                   "ordered_by": "flags" if lib.ddp_get_option(ctx, lib.DDP_OPT_FLAG_ORDER) else "events"}
            if s.n_buckets > 4:
                # many small buckets: the same with a launch hold of 8 marks and launches shared up to the default limit
                lib.ddp_set_option(ctx, lib.DDP_OPT_COALESCE, -1)
                lib.ddp_set_option(ctx, lib.DDP_OPT_LAUNCH_HOLD, 8)
                t_hold = timed(backward_and_sync)
                row["exposed_ms_hold_8"] = round(t_hold - t_bwd, 4)
            rows.append(row)
    return {"workload": f"resnet50 shape, fp16, R={R}, {n} parameters, {delay_us} us of synthetic backward per parameter",
            "algorithmic_bytes": (R + 1) * B, "reps": reps,
            "what": "GPU time between two events on the backward stream, median; exposed = t(backward + sync) - "
                    "t(backward alone); overlap = 1 - exposed / sync_alone; one launch per bucket",
            "per_cap": rows}


def r32_leg(lib, harness, torch, steps=8):
    """Configuration 5's two kernels at full size: the R = 32 reduction and one no_sync micro-step."""
    rig = Rig(lib, harness, torch, "bert_large_r32", 1, lib.DDP_PIPELINE_FUSED)
    try:
        res = rig.measure(steps, 2, per_call=True, spread_iters=20)
        out = {"reduce": {"ms_per_sync": res["ms_per_step"], "gbps": res["roofline"]["achieved"],
                          "frac_of_hbm_peak": res["roofline"]["frac"], "bytes_per_sync": (rig.R + 1) * rig.B,
                          "launches_per_step": res["launches_per_step"], "iteration_ms": res["roofline"]["iteration_ms"]}}
        micro = device_grads(harness, torch, rig.numel, rig.dtype, rig.R, rig.sigma, 5001)
        ptrs = micro.ptrs()
        ctx = rig.sessions[0].ctx
        for _ in range(2):
            lib.ddp_no_sync_accumulate(ctx, ptrs)
        lib.ddp_synchronize(ctx)
        lib.ddp_set_option(ctx, lib.DDP_OPT_TIMING, 1)
        for _ in range(max(steps, 20)):
            lib.ddp_no_sync_accumulate(ctx, ptrs)
        lib.ddp_synchronize(ctx)
        acc_ms, _ = lib.ddp_get_kernel_times(ctx, lib.DDP_K_ACCUMULATE)
        lib.ddp_set_option(ctx, lib.DDP_OPT_TIMING, 0)
        out["no_sync_accumulate"] = {"ms_per_micro_step": spread(acc_ms),
                                     "gbps": round(3.0 * rig.R * rig.B / float(np.median(acc_ms)) / 1e6, 1),
                                     "frac_of_hbm_peak": round(3.0 * rig.R * rig.B / float(np.median(acc_ms)) / 1e6 / HBM_PEAK_GBPS, 4),
                                     "bytes_per_micro_step": 3 * rig.R * rig.B}
        out["workload"] = (f"bert_large shape, fp32, R={rig.R}: {rig.R * rig.B / 1e9:.1f} GB of replica gradients "
                           f"and as much of micro-step gradients resident")
        del micro
    finally:
        rig.close()
    return out


def transport_leg(lib, harness, torch, steps):
    """Section 6.2.3 in the form 16-bit gradients in, binary32 averages out: BERT-large's gradients
    as bf16 copies, R = 8.  Bytes per synchronization: R x 2 bytes + 4 bytes per element, i.e.
    (R/2 + 1) x the binary32 model instead of (R + 1) x."""
    rig = Rig(lib, harness, torch, "bert_large_bf16", 2, lib.DDP_PIPELINE_FUSED, binary32_outputs=True)
    try:
        res = rig.measure(steps, 2, per_call=True)
        one = rig.measure(steps, 2, per_call=False)
        elems = sum(rig.numel)
        return {"workload": f"bert_large shape, bf16 gradients of R={rig.R} replicas, binary32 averages to separate tensors",
                "bytes_per_sync": rig.alg_bytes, "bytes_per_sync_all_binary32": (rig.R + 1) * 4 * elems,
                "ms_per_sync": res["ms_per_step"], "gbps": res["roofline"]["achieved"],
                "frac_of_hbm_peak": res["roofline"]["frac"], "launches_per_step": res["launches_per_step"],
                "iteration_ms": res["roofline"]["iteration_ms"],
                "marks_in_one_call": {"ms_per_sync": one["ms_per_step"], "gbps": one["roofline"]["achieved"],
                                      "frac_of_hbm_peak": one["roofline"]["frac"],
                                      "launches_per_step": one["launches_per_step"]}}
    finally:
        rig.close()


def staged_leg(lib, harness, torch, steps):
    """The literal three-kernel pipeline (pack, reduce, unpack) on the headline workload."""
    rig = Rig(lib, harness, torch, "resnet50", 1, lib.DDP_PIPELINE_STAGED)
    try:
        ctx = rig.sessions[0].ctx
        for k in range(2):
            rig.step(k, False)
        rig.sync()
        lib.ddp_set_option(ctx, lib.DDP_OPT_TIMING, 1)
        t0 = time.perf_counter()
        for k in range(steps):
            rig.step(k, False)
        rig.sync()
        ms_per_step = (time.perf_counter() - t0) * 1e3 / steps
        R, B = rig.R, rig.B
        pack, red, unpack = (lib.ddp_get_kernel_times(ctx, k)[0] for k in (lib.DDP_K_PACK, lib.DDP_K_REDUCE, lib.DDP_K_UNPACK))
        return {"ms_per_step": round(ms_per_step, 4),
                "value_gbps": round((R + 1) * B / ms_per_step / 1e6, 1),
                "pack_gbps": round(2.0 * R * B * steps / float(pack.sum()) / 1e6, 1),
                "reduce_gbps": round((R + 1) * B * steps / float(red.sum()) / 1e6, 1),
                "unpack_gbps": round(2.0 * B * steps / float(unpack.sum()) / 1e6, 1),
                "bytes": "pack 2RB, reduce (R+1)B, unpack (1+W)B per step", "steps": steps}
    finally:
        rig.close()


def accumulate_leg(lib, harness, torch, iters=20):
    rig = Rig(lib, harness, torch, "resnet50", 1, lib.DDP_PIPELINE_FUSED)
    try:
        micro = device_grads(harness, torch, rig.numel, rig.dtype, rig.R, rig.sigma, 2001)
        ptrs, ctx = micro.ptrs(), rig.sessions[0].ctx
        for _ in range(2):
            lib.ddp_no_sync_accumulate(ctx, ptrs)
        lib.ddp_synchronize(ctx)
        lib.ddp_set_option(ctx, lib.DDP_OPT_TIMING, 1)
        for _ in range(iters):
            lib.ddp_no_sync_accumulate(ctx, ptrs)
        lib.ddp_synchronize(ctx)
        acc_ms, _ = lib.ddp_get_kernel_times(ctx, lib.DDP_K_ACCUMULATE)
        return {"ms_per_micro_step": spread(acc_ms),
                "gbps": round(3.0 * rig.R * rig.B / float(np.median(acc_ms)) / 1e6, 1),
                "bytes": "3*R*B per micro-step (read gradient and micro-gradient, write gradient)"}
    finally:
        rig.close()


def cpu_baseline_leg(workload="resnet50", budget_s=12.0):
    """The CPU oracle as it stands, on the headline workload: whole synchronizations on one thread,
    then with every bucket's element range split over all host cores (the same oracle functions
    on slices: identical bits)."""
    import oracle
    import workloads
    shape_name, config_id, R, sigma, dtype, cap = WORKLOADS[workload]
    numel = workloads.numel_of(workloads.WORKLOAD_SHAPES[shape_name]())
    n = len(numel)
    B = sum(numel) * workloads.ESIZE[dtype]
    cores = min(os.cpu_count() or 1, 16)        # a one-GPU machine's share of the host
    with ThreadPoolExecutor(max_workers=cores) as pool:
        flat = list(pool.map(lambda rp: workloads.gaussian_grad(config_id, rp[0], 0, rp[1], numel[rp[1]], sigma, dtype),
                             [(r, p) for r in range(R) for p in range(n)]))
    reps = [flat[r * n:(r + 1) * n] for r in range(R)]
    dtypes = [dtype] * n

    t0 = time.perf_counter()
    done = 0
    while True:
        ref, asg, _ = oracle.synchronize(numel, dtypes, cap, reps)
        done += 1
        if time.perf_counter() - t0 > budget_s or done >= 400:
            break
    single_ms = (time.perf_counter() - t0) * 1e3 / done

    def one_sync_all_cores(pool):
        outs = [None] * n
        for b in range(len(asg.buckets)):
            flats = [oracle.pack_bucket(asg, b, reps[r]) for r in range(R)]
            elems = len(flats[0])
            cuts = [elems * k // cores for k in range(cores + 1)]
            parts = list(pool.map(lambda k: oracle.reduce_average([f[cuts[k]:cuts[k + 1]] for f in flats], asg.buckets[b].dtype),
                                  range(cores)))
            oracle.unpack_bucket(asg, b, np.concatenate(parts), outs)
        return outs

    with ThreadPoolExecutor(max_workers=cores) as pool:
        outs = one_sync_all_cores(pool)
        same = all(outs[i].tobytes() == ref[i].tobytes() for i in range(n))
        t0 = time.perf_counter()
        done_mt = 0
        while True:
            one_sync_all_cores(pool)
            done_mt += 1
            if time.perf_counter() - t0 > budget_s or done_mt >= 400:
                break
        multi_ms = (time.perf_counter() - t0) * 1e3 / done_mt
    return {
        "value": round((R + 1) * B / multi_ms / 1e6, 3),
        "unit": "GB/s",
        "cores": cores,
        "kind": "oracle",
        "ms_per_step": round(multi_ms, 2),
        "sample": f"{done_mt} whole synchronizations of the {workload} workload (all {len(asg.buckets)} buckets, R={R}, "
                  f"host-generated gradients of the parity tests' recipe) by the numpy oracle, every bucket's "
                  f"element range split over {cores} threads calling the unchanged oracle functions "
                  f"(bit-identical to the single-thread result: {same})",
        "single_thread": {"value": round((R + 1) * B / single_ms / 1e6, 3), "unit": "GB/s", "cores": 1,
                          "ms_per_step": round(single_ms, 2), "sample": f"{done} whole synchronizations, one thread"},
        "host_cores_visible": os.cpu_count(),
        "numpy": np.__version__,
    }


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=40)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--legs", default=",".join(ALL_LEGS),
                    help="comma list of " + ", ".join(ALL_LEGS) + " (headline is always run)")
    ap.add_argument("--workload", default="resnet50", choices=["resnet50", "bert_large"],
                    help="the workload of the headline measurement (the default run reports bert_large as a "
                         "sub-object; this switch is for profiling one shape alone)")
    ap.add_argument("--sets", type=int, default=4,
                    help="independent sets of replica gradients taken in turn by consecutive steps")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--launch-ordering", default="default", choices=["default", "events"],
                    help="events: order the launches behind the backward stream by HIP events instead of device "
                         "flags (for runs under the profiler's counter collection, which serializes all kernels, "
                         "so that a launch never finds the flag it waits for being set meanwhile)")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run a plain 1 GiB device copy (for scaling profiler counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the R replicas are R buffers in one GPU's "
              "HBM); --gpus above 1 is not supported and nothing was measured", file=sys.stderr)
        return 2
    legs = set(x for x in args.legs.split(",") if x)
    unknown = legs - set(ALL_LEGS)
    if unknown:
        print(f"bench.py: unknown legs {sorted(unknown)}", file=sys.stderr)
        return 2
    if args.no_cpu_baseline:
        legs.discard("cpu")

    import torch
    import __graft_entry__
    __graft_entry__.ensure_built()          # a fresh checkout has no library yet
    import paper_2006_15704_amd as lib
    from paper_2006_15704_amd import harness

    if args.calibration_copy:
        src = torch.zeros(1 << 30, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    sets = args.sets if args.workload == "resnet50" else min(args.sets, 2)
    if args.launch_ordering == "events":
        Rig.every_rig_options = ((lib.DDP_OPT_FLAG_ORDER, 0),)
    head = shape_leg(lib, harness, torch, args.workload, sets, args.steps, args.warmup, legs, "per_call")
    _, _, R, _, dtype, _ = WORKLOADS[args.workload]
    out = {
        "metric": "bucketed grad-sync throughput ((R+W)*B per synchronization)",
        "value": head["value_gbps"],
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"],
        "ms_per_step_all_runs": head["ms_per_step_all_runs"],
        "timed_runs": "the timed region of `steps` steps is run three times; value, ms_per_step and roofline are the median run",
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": DT_NAME[dtype],
        "data": "synthetic",
        "config": head.pop("config"),
        "pct_hbm_peak_end_to_end": head["pct_hbm_peak_end_to_end"],
        "host_enqueue_ms_per_step": head["host_enqueue_ms_per_step"],
        "launches_per_step": head["launches_per_step"],
        "repaired_launches": head["repaired_launches"],
        "roofline": head["roofline"],
    }
    for key in ("marks_in_one_call", "marks_one_by_one_hold_16", "one_launch_per_bucket", "single_replica_set"):
        if key in head:
            out[key] = head[key]
    if "bert_large" in legs and args.workload != "bert_large":
        # 12 GB per step already: two sets are far beyond any cache
        bert = shape_leg(lib, harness, torch, "bert_large", 2, max(10, args.steps // 2), 2,
                         legs - {"single_set"}, "per_call")
        bert["value"] = bert.pop("value_gbps")
        bert["unit"] = "GB/s"
        out["bert_large"] = bert
    if "overlap" in legs:
        out["overlap"] = overlap_leg(lib, harness, torch)
    if "r32" in legs:
        out["bert_large_r32"] = r32_leg(lib, harness, torch)
    if "transport" in legs:
        out["bf16_transport"] = transport_leg(lib, harness, torch, max(10, args.steps // 2))
    if "staged" in legs:
        out["staged"] = staged_leg(lib, harness, torch, max(5, args.steps // 4))
    if "accumulate" in legs:
        out["no_sync_accumulate"] = accumulate_leg(lib, harness, torch)
    torch.cuda.synchronize()
    if "cpu" in legs:
        out["cpu_baseline"] = cpu_baseline_leg()
    else:
        out["cpu_baseline"] = None
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
