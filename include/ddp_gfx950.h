/*
 * ddp_gfx950 -- bucketed gradient synchronization for one MI355X (gfx950).
 *
 * C ABI of the data-parallel hot path of "PyTorch Distributed: Experiences on
 * Accelerating Data Parallel Training" (arXiv 2006.15704).  The R training
 * processes of the paper are stood in for by R replica copies of every
 * gradient, all resident in one GPU's HBM; the AllReduce of a bucket
 * (Section 2.3: every participant provides an equally sized tensor and
 * collects the global sum) becomes an R-way sum kernel, followed by the
 * division by R that turns the sum into DDP's average (Section 3.2.1).
 *
 * Conventions
 *   - Every function returns an int32_t status: >= 0 success (DDP_OK unless
 *     stated otherwise), < 0 one of the DDP_ERR_* codes.  Nothing aborts,
 *     throws or blocks forever.  ddp_last_error() returns a text for the most
 *     recent failure on that context (or, with ctx == NULL, of the most recent
 *     failed ddp_create on this thread).
 *   - "device pointer" = address in the GPU's global memory; "host pointer" =
 *     ordinary process memory.  Host arrays passed in are copied before the
 *     call returns.  Gradient memory is owned by the caller and borrowed until
 *     ddp_destroy; bucket storage is owned by the library.
 *   - Streams are hipStream_t values passed as void* (NULL = the null stream).
 *     The library creates reduction streams of its own (one at ddp_create when
 *     the two streams differ, more if DDP_OPT_REDUCE_STREAMS asks for them), all
 *     at the default priority and non-blocking with respect to the null stream.
 *   - A context is not thread-safe (the paper's hooks fire from one autograd
 *     thread).  Different contexts may be used from different threads.
 *   - All compute calls are asynchronous with respect to the host unless
 *     stated otherwise.
 *   - Graph capture: the ready marks and ddp_finalize_backward of an iteration
 *     may be captured into a HIP graph on backward_stream (the capture forks
 *     to the reduction streams and joins again by itself) if every replica
 *     takes part in every parameter (no participation flags: their staging
 *     copies read host memory that later iterations rewrite), DDP_OPT_TIMING is
 *     0 and the staged pipeline is not used.  The host state (launch log,
 *     iteration count) advances at capture time only; a replay repeats the same
 *     launches on whatever the gradient tensors hold then.
 */
#ifndef DDP_GFX950_H
#define DDP_GFX950_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ddp_ctx ddp_ctx;

/* status codes */
#define DDP_OK                  0
#define DDP_ERR_ARG            -1  /* invalid argument (null, out of range, unknown code) */
#define DDP_ERR_STATE          -2  /* call out of order (e.g. mark before build, register twice) */
#define DDP_ERR_ALREADY_READY  -3  /* parameter already marked ready in this iteration */
#define DDP_ERR_HIP            -4  /* a HIP runtime call failed; text in ddp_last_error */
#define DDP_ERR_NO_DEVICE      -5  /* compute requested on a plan-only context */
#define DDP_ERR_UNSUPPORTED    -6  /* combination not supported (e.g. R above DDP_MAX_REPLICAS) */

/* element types of gradients */
#define DDP_FP32 0
#define DDP_FP16 1
#define DDP_BF16 2

#define DDP_MAX_REPLICAS 64

/* device == DDP_DEVICE_NONE makes a plan-only context: bucket assignment and
 * the ready/launch state machine run and can be inspected, no device memory is
 * touched, nothing is computed, and ddp_no_sync_accumulate / ddp_synchronize /
 * ddp_synth_backward return DDP_ERR_NO_DEVICE.  It exists so that the host
 * logic can be tested on machines without a GPU; it is not a CPU fallback. */
#define DDP_DEVICE_NONE (-1)

/* ddp_build_buckets cap meaning "one bucket per run of equal element type" */
#define DDP_CAP_WHOLE_MODEL UINT64_MAX

/* options for ddp_set_option (set before ddp_build_buckets unless noted) */
#define DDP_OPT_PIPELINE       1  /* DDP_PIPELINE_STAGED (default) or DDP_PIPELINE_FUSED */
#define DDP_OPT_WRITE_ALL      2  /* 0 (default): the average is written to replica 0's gradient
                                     tensors only (one rank's view); 1: to all R replicas' tensors */
#define DDP_OPT_TIMING         3  /* any time.  1: every pack / reduce / unpack / accumulate launch
                                     carries a pair of HIP events that the runtime stamps with the
                                     kernel's own start and end (no event packet between the
                                     kernels of a stream); 2: one pair per iteration, from just
                                     before its first bucket launch to just after its last (kind
                                     DDP_K_ITERATION); 0: off.  Read with ddp_get_kernel_times */
#define DDP_OPT_NONTEMPORAL    5  /* any time: 1 (default) = read-once inputs are loaded, and the
                                     averages stored, with the non-temporal hint; 0 = plain */
#define DDP_OPT_EMIT_BUSY_BLOCKS 8 /* any time: ddp_synth_backward's delay kernel.  0 (default): one
                                     thread block that sleeps between clock polls; n > 0: n blocks
                                     that do arithmetic between polls, so that the delay loads the
                                     GPU the way backward compute does */
#define DDP_OPT_COALESCE      10  /* any time: value > 0 = buckets that one API call makes launchable
                                     (ddp_mark_ready_many, ddp_finalize_backward, ddp_synth_backward
                                     between two of its kernels) and that are consecutive and of one
                                     element type share ONE launch per kernel as long as the launch
                                     stays within `value` bytes of bucket data (INT64_MAX: no
                                     limit); order and results are unchanged.  0 = one launch per
                                     bucket.  Default -1 = chosen from R so that a launch runs for
                                     roughly 150 to 300 us (400 MiB for R <= 2, 240 MiB up to 4,
                                     100 MiB up to 8, 70 MiB up to 16, else 50 MiB; measured: short
                                     launches pay a fixed start-up and drain cost each, much longer
                                     ones lose throughput again) */
#define DDP_OPT_FIND_UNUSED   11  /* any time between iterations: the paper's find_unused_parameters
                                     knob.  1 = gradients of parameters that no replica used in the
                                     iteration (the global bitmap of Section 4.2 says so) are left
                                     exactly as they are (a bucket made only of such parameters is
                                     then not launched at all in the fused pipeline: Section 6.2.2's
                                     skipping at the bucket level); 0 (default) = they are written as
                                     zeros */
#define DDP_OPT_REDUCE_STREAMS 12  /* between iterations: number of reduction streams, 1 to 8, or -1
                                     (default): two for launches that move less than DDP_OPT_REDUCE_CAP_MIN_BYTES
                                     (start-up and drain of a short launch then overlap with its
                                     neighbour: +2 to 3 points of HBM peak with one launch per 25 MiB
                                     bucket), one for larger launches (two long launches at a time share
                                     the memory system and lose).
                                     The launches of an iteration take the streams in turn: the
                                     caller's reduce_stream first, then streams the library creates
                                     (default priority).  This is the one-GPU form of Section 3.3's
                                     round-robin process groups (Section 5.4 measures rr1/rr3/rr5):
                                     launches are still enqueued in bucket order, but buckets on
                                     different streams may run at the same time.  Every stream waits
                                     for backward_stream like reduce_stream does, and at finalize
                                     backward_stream is made to wait for all of them (directly in the
                                     fused pipeline; through reduce_stream where the staged pipeline's
                                     write-back or the bitmap step runs there).  Results are
                                     unchanged */
#define DDP_OPT_REDUCE_BLOCKS_PER_CU 13 /* any time: cap on the thread blocks of the reduce kernels that
                                     are resident on one compute unit at a time (an LDS allocation
                                     the kernels do not touch enforces it).  A block keeps R x 2
                                     16-byte loads per thread in flight, so two or three blocks per
                                     unit fill the memory system; more only interleave more request
                                     streams at the DRAM channels and throughput drops.  0 = no cap
                                     (wave slots decide: 8).  Default -1 =
                                     chosen from R: no cap up to R = 4 (few loads per block), else 2 */
#define DDP_OPT_REDUCE_CAP_MIN_BYTES 14 /* any time: the cap applies to launches that move at least this
                                     many bytes, counted as (R + 1) x the launch's bucket bytes
                                     (measured at R = 8: it gains 1 to 2.5 points of HBM peak from
                                     50 MiB of bucket data up and loses 1.5 to 3 on launches of 25
                                     MiB and less; at R = 16 and 32 a 25 MiB bucket is already a long
                                     launch and gains 2.5 points).  Default 360 MiB (40 MiB of bucket
                                     data at R = 8) */
#define DDP_OPT_ACCUMULATE_BLOCKS_PER_CU 16 /* any time: likewise for the accumulate kernel (two loads
                                     and a store per vector; registers allow 8 blocks).  Default 5 */
#define DDP_OPT_TAIL_ON_BACKWARD 17 /* any time between iterations: 1 (default) = the buckets launched by
                                     the API call that completes an iteration (the call after which
                                     the last bucket is launchable: every gradient exists, nothing
                                     of the backward pass is left to overlap with) are enqueued on
                                     backward_stream instead of a reduction stream, fused pipeline
                                     only.  Stream order then replaces the cross-stream event, whose
                                     hand-over takes about 0.2 ms on this system when the waiting
                                     queue was armed long before the event fires.  0 = every bucket
                                     goes to a reduction stream */
#define DDP_OPT_LAUNCH_HOLD   21  /* between iterations: 0 (default) = a bucket is launched by the ready
                                     mark that completes it, as in Algorithm 1.  n > 0 = it is kept back
                                     until n further ready marks have arrived, the iteration's last
                                     bucket is launchable, the held buckets fill a launch
                                     (DDP_OPT_COALESCE) or ddp_finalize_backward / the end of a
                                     ddp_mark_ready_many call comes, whichever is first; every bucket
                                     that becomes launchable meanwhile joins it and restarts the count.
                                     Consecutive buckets then share launches although their marks
                                     arrive one call at a time: fewer launches, gates and announcements
                                     (what costs with many small buckets), at the price of starting
                                     each reduction up to n marks later.  Order, launch log and results
                                     are unchanged */
#define DDP_OPT_FLAG_ORDER    18  /* between iterations: how a bucket launch on a reduction stream is ordered
                                     after the work on backward_stream that produces its gradients
                                     (fused pipeline).  -1 (default): through device flags where the
                                     streams allow it -- ddp_mark_ready enqueues a one-block kernel on
                                     backward_stream that announces a sequence number, and a one-wave
                                     gate kernel in front of the bucket kernel waits for it; no event
                                     record stalls backward_stream and the bucket kernel starts as soon
                                     as the number is there.  The gate's wait is bounded
                                     (DDP_OPT_GATE_WAIT_US); a launch whose gate gave up does nothing and
                                     is redone by a repair launch that ddp_finalize_backward enqueues on
                                     backward_stream once every gradient exists, so results never depend
                                     on a wait succeeding.  The way back at ddp_finalize_backward is
                                     ordered likewise: each reduction stream stores the iteration's
                                     number behind its last launch and one kernel on backward_stream
                                     waits (bounded) for those numbers, followed by waits for events of
                                     the same streams, which have fired by then (a wait for an event
                                     that has yet to fire is handed over slowly on this system when it
                                     was enqueued long before).  Streams that share a hardware queue cannot
                                     run a gate and its announcement concurrently; ddp_create (and
                                     DDP_OPT_REDUCE_STREAMS) probe for that with a bounded test and such
                                     streams keep events.  0: events always */
#define DDP_OPT_CHAIN_LAUNCHES 22 /* any time: 1 (default) = with flag ordering, a bucket launch that
                                     follows another one of the same iteration on a different stream,
                                     one that moves at least 160 MiB ((R + 1) x its bucket bytes;
                                     unless both move DDP_OPT_REDUCE_CAP_MIN_BYTES or more),
                                     starts when that one has started its last thread block (its gate
                                     waits for that too, bounded like every wait; the iteration's
                                     last launches on backward_stream get a one-wave kernel of their
                                     own for it), so consecutive launches overlap where one drains
                                     and the next starts up instead of sharing the memory system
                                     from the start; and an API call that completes the iteration
                                     with several launches spreads them over backward_stream and
                                     reduce_stream in turn under the same rule instead of queueing
                                     them on backward_stream.  0 = launches on different streams
                                     start as soon as their gradients are there.  Scheduling only:
                                     results are unchanged */
#define DDP_OPT_GATE_WAIT_US  19  /* any time: upper bound, in microseconds, on a gate's wait (0 = look
                                     once).  Default 100000.  A backward pass that lags further behind
                                     the host only loses overlap for that iteration, never correctness */

/* DDP_PIPELINE_STAGED follows the paper's data flow literally: gradients are
 * copied into flat per-replica bucket buffers (Algorithm 1, autograd_hook),
 * the bucket is reduced, and the averaged bucket is copied back to the
 * gradient tensors by the finalizing step.  DDP_PIPELINE_FUSED computes the
 * same values in one pass per bucket: the kernel gathers each replica's
 * gradients through the bucket's segment table, sums and averages in
 * registers, and writes straight to the gradient tensors; the flat bucket is
 * virtual.  Bucket assignment, launch order and results are identical. */
#define DDP_PIPELINE_STAGED 0
#define DDP_PIPELINE_FUSED  1

/* kernel kinds for ddp_get_kernel_times */
#define DDP_K_PACK       0
#define DDP_K_REDUCE     1   /* staged reduce, or the fused gather-reduce-scatter */
#define DDP_K_UNPACK     2
#define DDP_K_ACCUMULATE 3
#define DDP_K_ITERATION  4   /* timing mode 2: all bucket launches of one iteration */

/* Create a context for R >= 1 replicas on HIP device `device` (or
 * DDP_DEVICE_NONE).  `reduce_stream` is the dedicated stream the bucket
 * kernels run on (Section 3.3: communication gets its own streams so that it
 * does not block computation); `backward_stream` is the stream on which the
 * caller produces gradients.  They may be equal.  *out receives the handle. */
int32_t ddp_create(ddp_ctx** out, int32_t R, int32_t device,
                   void* reduce_stream, void* backward_stream);

/* Waits for the context's outstanding work, frees library-owned memory and
 * events.  Gradient memory is untouched. */
int32_t ddp_destroy(ddp_ctx* ctx);

const char* ddp_last_error(const ddp_ctx* ctx);

int32_t ddp_set_option(ddp_ctx* ctx, int32_t option, int64_t value);

/* Reads back what is in effect for every DDP_OPT_ option as it was set (-1
 * where that means "the library chooses"), except: DDP_OPT_COALESCE gives the
 * byte limit in effect (also when it was chosen from R) and DDP_OPT_FLAG_ORDER
 * gives 1 if the launches of the next iteration would be ordered through device
 * flags (the option allows it, the pipeline is the fused one, the buckets are
 * built and every reduction stream in use passed the concurrency probe), else
 * 0.  Also reads DDP_STAT_REPAIRED_LAUNCHES below.  Unknown option ->
 * DDP_ERR_ARG. */
int32_t ddp_get_option(ddp_ctx* ctx, int32_t option, int64_t* value);

/* Read-only through ddp_get_option: the number of bucket launches whose gate
 * gave up and that a repair launch redid, since ddp_create (the call waits for
 * the context's outstanding work first).  A number that keeps growing says that
 * DDP_OPT_GATE_WAIT_US is too short for this backward pass. */
#define DDP_STAT_REPAIRED_LAUNCHES 100

/* Algorithm 1, constructor loop over net.parameters(): registers n parameters
 * in registration order (index = position in net.parameters()).
 *   numel[n]      host, element count of each gradient (0 allowed)
 *   dtype[n]      host, DDP_FP32 / DDP_FP16 / DDP_BF16
 *   grad_ptrs     host array of R*n device pointers, row-major [r][i]: replica
 *                 r's gradient of parameter i; contiguous, aligned at least to
 *                 its element size.  16-byte alignment is exploited, not
 *                 required: what matters is that the R tensors of a
 *                 parameter share one address modulo 16 (whatever it is);
 *                 then whole tiles take the unpredicated path (77 % of the HBM
 *                 peak measured on 25 MiB tensors, R = 8).  Replicas that are
 *                 shifted against each other are read with element-aligned
 *                 16-byte loads and cost extra cache lines (62 % measured on
 *                 the same list with the replicas 4 bytes apart modulo 16).
 *                 Ignored (may be NULL) on a plan-only context.
 * Errors: n <= 0, null arrays or pointers, unknown dtype -> DDP_ERR_ARG;
 * second call -> DDP_ERR_STATE. */
int32_t ddp_register_params(ddp_ctx* ctx, int32_t n, const int64_t* numel,
                            const int32_t* dtype, void* const* grad_ptrs);

/* Section 6.2.3 (gradient compression: gradients need not be communicated in
 * the parameter's type), in the form "16-bit on the wire, binary32 arithmetic and
 * result": every registered gradient is fp16 or bf16 -- what each of the R
 * processes would send -- and the average of parameter i, the binary32 sum over
 * the replicas in order r = 0 .. R-1 divided by R, is written UNROUNDED as
 * numel[i] binary32 values to out_ptrs[i] (device pointers, host array of n
 * entries, copied; memory owned by the caller and borrowed until ddp_destroy;
 * aligned to 4 bytes, 16-byte alignment is exploited).  No gradient tensor is
 * written; buckets are still filled and capped by the 16-bit gradient bytes (a
 * bucket is what is communicated).  A synchronization then moves (R/2 + 1) x
 * the binary32 model bytes instead of (R + 1) x.  Parameters that nobody used
 * receive binary32 zeros, or are left untouched with DDP_OPT_FIND_UNUSED.
 * Between ddp_register_params and ddp_build_buckets, fused pipeline, not with
 * DDP_OPT_WRITE_ALL (DDP_ERR_UNSUPPORTED from ddp_build_buckets otherwise).
 * Errors: a binary32 gradient among the registered ones, null or misaligned
 * pointer -> DDP_ERR_ARG; called out of order -> DDP_ERR_STATE. */
int32_t ddp_set_outputs(ddp_ctx* ctx, void* const* out_ptrs);

/* Algorithm 1, constructor: buckets are filled with the parameters taken in
 * reverse registration order, under the size cap `cap_bytes` (Section 4.2,
 * bucket_cap_mb; 0 = every gradient alone, Section 5.2; DDP_CAP_WHOLE_MODEL =
 * no cap).  Parameters are visited n-1 ... 0; a parameter that would push a
 * non-empty bucket past the cap, or whose element type differs from the
 * bucket's, closes it first, so a bucket exceeds the cap only if it holds a
 * single parameter.  Offsets inside a bucket are dense.  Allocates the flat
 * bucket storage (staged pipeline) and the device segment tables.
 * Returns the number of buckets (>= 1).  Errors: before register or called
 * twice -> DDP_ERR_STATE; allocation failure -> DDP_ERR_HIP. */
int32_t ddp_build_buckets(ddp_ctx* ctx, uint64_t cap_bytes);

/* Section 6.2.1 (gradient order prediction): rebuilds the parameter-to-bucket
 * mapping so that it follows the traced backward order.  The parameters are
 * visited in the order of the ready marks of the iteration closed by the latest
 * ddp_finalize_backward (ddp_get_ready_order(ctx, 1, ...)), followed by the
 * parameters that iteration never marked in reverse registration order; the
 * allocation rule is that of ddp_build_buckets (with an empty trace the result
 * is the default mapping).  Only between iterations: any ready mark since the
 * last finalize, or a ddp_no_sync_accumulate not yet followed by a
 * synchronization -> DDP_ERR_STATE.  The call waits for both streams, frees and
 * rebuilds the library's tables and flat buffers (the paper calls this
 * re-allocation costly and to be done rarely), and clears the closed launch log
 * and the kernel times; gradient memory is untouched.  Returns the new number
 * of buckets, or a negative error; after a DDP_ERR_HIP the context has no
 * buckets (as before ddp_build_buckets). */
int32_t ddp_rebuild_buckets(ddp_ctx* ctx, uint64_t cap_bytes);

/* The trace: ids[0..*n) = parameters in the order of their ready marks in the
 * running (which = 0) or the latest closed (which = 1) iteration.  At most cap
 * ids are written; *n is always the full count. */
int32_t ddp_get_ready_order(const ddp_ctx* ctx, int32_t which, int32_t* ids, int32_t cap, int32_t* n);

/* bucket_of[n], elem_offset[n] (host, caller-allocated): bucket index and
 * element offset inside the bucket for every parameter. */
int32_t ddp_get_assignment(const ddp_ctx* ctx, int32_t* bucket_of, int64_t* elem_offset);

/* Element count, number of parameters and element type of bucket b. */
int32_t ddp_get_bucket_info(const ddp_ctx* ctx, int32_t b, int64_t* elems,
                            int32_t* n_params, int32_t* dtype);

/* Staged pipeline only: device address of bucket b's flat buffer of replica r
 * (0 <= r < R), or of the averaged bucket (r == -1).  For tests. */
int32_t ddp_get_bucket_ptr(const ddp_ctx* ctx, int32_t b, int32_t r, void** ptr);

/* Algorithm 1, autograd_hook(param_index), with the pending counts of
 * Section 4.2: records that all R replica gradients of `param_id` have been
 * produced by work already enqueued on backward_stream, decrements the
 * bucket's pending count, and launches on reduce_stream (see also
 * DDP_OPT_REDUCE_STREAMS and DDP_OPT_TAIL_ON_BACKWARD), in bucket order,
 * every bucket that is complete and whose predecessors have all been launched
 * (Section 3.2.3: no bucket i+1 before bucket i).  A launch first makes
 * reduce_stream wait for backward_stream's work enqueued so far, then copies
 * the bucket's gradients into the flat buffers and reduces them (staged), or
 * runs the one-pass kernel (fused).  Returns after enqueueing.
 * Errors: buckets not built -> DDP_ERR_STATE; id out of range -> DDP_ERR_ARG;
 * marked twice in one iteration -> DDP_ERR_ALREADY_READY (no state change). */
int32_t ddp_mark_ready(ddp_ctx* ctx, int32_t param_id);

/* Ready mark with per-replica participation (Section 3.2.3, last paragraph;
 * Section 4.2 "Globally Unused Parameters"): used[r] != 0 (host array of R
 * bytes) says that replica r's backward pass produced a gradient for the
 * parameter.  A replica that did not contributes zeros to the sum (which is
 * still divided by R) and its tensor is not read.  Participation recorded by
 * ddp_no_sync_accumulate since the last finalize is OR-ed in (Section 3.2.4).
 * ddp_mark_ready(p) is the same call with every used[r] = 1.  At finalize the
 * per-replica flags are copied to the device and reduced with an OR over the
 * replicas (the extra AllReduce on the bitmap); parameters whose global bit is
 * 0 keep their gradients with DDP_OPT_FIND_UNUSED, else receive zeros.
 * Errors as for ddp_mark_ready; used == NULL -> DDP_ERR_ARG. */
int32_t ddp_mark_ready_local(ddp_ctx* ctx, int32_t param_id, const uint8_t* used);

/* used[n] (host): the global bitmap of the synchronization closed by the latest
 * ddp_finalize_backward, 1 = at least one replica used the parameter.  When any
 * flag of that iteration was 0 this is the device-computed result (the call
 * waits for the copy that finalize enqueued); otherwise it is all ones. */
int32_t ddp_get_global_used(ddp_ctx* ctx, uint8_t* used);

/* Same as calling ddp_mark_ready for ids[0..count) in order; stops at the
 * first error and returns it.  Buckets that complete during the call are
 * launched one after the other in index order; because the caller cannot
 * enqueue anything on backward_stream in the middle of the call, a single
 * stream-ordering point serves all of them. */
int32_t ddp_mark_ready_many(ddp_ctx* ctx, const int32_t* ids, int32_t count);

/* The finalizing step described after Algorithm 1 (wait for the reductions and
 * write the averages back to the gradients), plus Section 3.2.3's handling of
 * absent gradients: parameters not marked in this iteration are treated as
 * ready; replicas for which ddp_no_sync_accumulate recorded no gradient since
 * the last finalize contribute zeros (their memory is not read); a parameter
 * that nobody used receives zeros, or is left untouched with
 * DDP_OPT_FIND_UNUSED;
 * remaining buckets are launched in order; the averaged buckets are copied
 * into the gradient tensors; backward_stream is made to wait for all of it, so
 * work enqueued on backward_stream afterwards sees the averaged gradients;
 * pending counts are replenished for the next iteration (Section 4.2).
 * Host-asynchronous: use ddp_synchronize for host-visible completion. */
int32_t ddp_finalize_backward(ddp_ctx* ctx);

/* Blocks the host until everything enqueued by this context has finished. */
int32_t ddp_synchronize(ddp_ctx* ctx);

/* Launch log of the running iteration (which == 0: buckets launched since the
 * last ddp_finalize_backward) or of the iteration closed by the latest
 * ddp_finalize_backward (which == 1).  bucket_ids[i] is the i-th bucket
 * launched; after_call[i] is the 0-based index of the ready mark that
 * triggered the launch, or the total number of marks for buckets launched by
 * the finalizing step.  Arrays (host, may be NULL) hold `cap` entries; *n
 * receives the number of launches. */
int32_t ddp_get_launch_log(const ddp_ctx* ctx, int32_t which, int32_t* bucket_ids,
                           int32_t* after_call, int32_t cap, int32_t* n);

/* Section 3.2.4, no_sync: adds one micro-step's gradients into the registered
 * gradient tensors, grad[r][i] += micro[r][i] (sum in fp32, stored in the
 * gradient's type), on backward_stream.  No ready marks, no reduction.
 *   micro_grad_ptrs  host array of R*n device pointers, [r][i]; a NULL entry
 *                    means parameter i produced no gradient in this micro-step.
 * The micro buffers may be reused once work enqueued on backward_stream after
 * this call has started (stream order). */
int32_t ddp_no_sync_accumulate(ddp_ctx* ctx, void* const* micro_grad_ptrs);

/* used[n] (host): 1 if the parameter received a gradient through
 * ddp_no_sync_accumulate or a ready mark, else 0 -- since the last finalize
 * (which == 0) or in the synchronization closed by the latest finalize
 * (which == 1).  Section 3.2.4: participation information accumulates across
 * no_sync iterations and serves when the next synchronization takes place. */
int32_t ddp_get_used_map(const ddp_ctx* ctx, int32_t which, uint8_t* used);

/* Synthetic backward pass (stands in for the autograd engine, Section 3.2.3):
 * for k = 0..count-1, enqueue on backward_stream a kernel that busy-waits
 * delay_ns[k] nanoseconds (bounded) and then, if src_ptrs != NULL, copies
 * src_ptrs[r*n + order[k]] into the registered gradient of parameter order[k]
 * for every replica r ("the gradient is produced"); then call
 * ddp_mark_ready(order[k]).  delay_ns may be NULL (no delay).  With
 * mark == 0 the ready marks are left out (backward alone, for timing). */
int32_t ddp_synth_backward(ddp_ctx* ctx, const int32_t* order, int32_t count,
                           const int64_t* delay_ns, void* const* src_ptrs,
                           int32_t mark);

/* With DDP_OPT_TIMING on: durations in milliseconds of the launches of `kind`
 * since the option was last set, in launch order.  Call after
 * ddp_synchronize.  ms holds `cap` entries; *n receives the count available.
 * ids (may be NULL) receives, per launch: for pack and reduce the first bucket
 * of the launch plus 65536 times the number of further buckets coalesced into
 * it; -1 for unpack and accumulate (whole model); for DDP_K_ITERATION the
 * number of bucket launches inside the interval. */
int32_t ddp_get_kernel_times(ddp_ctx* ctx, int32_t kind, float* ms, int32_t* ids,
                             int32_t cap, int32_t* n);

/* For callers that cannot allocate device memory: code that runs under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  One
 * whole synchronization in one call, with no context: the same result as, on a
 * fresh DDP_PIPELINE_STAGED context, ddp_register_params + ddp_build_buckets
 * (cap_bytes) + ddp_mark_ready_many(n-1 ... 0) + ddp_finalize_backward -- every
 * replica takes part in every parameter, the average goes to replica 0's
 * gradient tensors, the other replicas' tensors are inputs only.  Arguments as
 * for ddp_create (R, device, one stream for everything) and ddp_register_params
 * (n, numel, dtype, grad_ptrs: host arrays, copied before the call returns;
 * gradient memory stays the caller's).  Returns the number of buckets.
 *
 * The device tables and the R + 1 flat bucket buffers live in a static device
 * array of DDP_STATIC_SCRATCH_BYTES that every GPU used through this call holds
 * until the process ends; host tables travel inside kernel arguments.  The call
 * makes no hipMalloc / hipFree / hipHostMalloc and no copy from host memory; all
 * its work is kernels enqueued on `stream`, in order, so it is asynchronous and
 * may be captured.  Limits: tables (32 bytes + 8 R bytes per parameter, 4 bytes
 * per 8 KiB of a gradient) plus (R + 1) x the padded gradient bytes must fit the
 * array, else DDP_ERR_UNSUPPORTED and nothing is enqueued (text in
 * ddp_last_error(NULL)).  All calls on one GPU share the array, which keeps the
 * previous call's contents (the call clears what it needs cleared): calls whose
 * work overlaps in time on one GPU -- different streams, different threads --
 * race; serialize them.  Other errors as for ddp_create / ddp_register_params. */
#define DDP_STATIC_SCRATCH_BYTES (32u << 20)
int32_t ddp_sync_static(int32_t R, int32_t device, void* stream, int32_t n,
                        const int64_t* numel, const int32_t* dtype,
                        void* const* grad_ptrs, uint64_t cap_bytes);

/* Library version string. */
const char* ddp_version(void);

#ifdef __cplusplus
}
#endif
#endif /* DDP_GFX950_H */
