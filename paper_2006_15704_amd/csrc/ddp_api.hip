// C ABI of the library: context, registration, bucket building, ready marks,
// finalize, no_sync accumulation and the synthetic backward emitter.  Host
// code only; the kernels are in ddp_kernels.hip.
#include "../../include/ddp_gfx950.h"

#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstring>
#include <string>
#include <utility>
#include <vector>

#include "bucket_plan.h"
#include "ddp_kernels.h"
#include "seg_layout.h"

namespace {

// Cross-stream ordering events: no timestamps, and a device-scope release --
// producer and consumer kernels run on the same GPU, so the default
// system-scope release (a cache write-back at every record) is not needed.
// Host-visible completion always goes through hipStreamSynchronize.
constexpr unsigned kOrderEvent = hipEventDisableTiming | hipEventReleaseToDevice;
// Timing events: device-scope release as well, so that the record itself does
// not add cache maintenance to the interval it measures.
constexpr unsigned kTimingEvent = hipEventReleaseToDevice;

thread_local std::string g_create_error;   // failures of calls that have no context

struct TimedLaunch {
    int32_t kind;
    int32_t bucket;
    hipEvent_t start, stop;
};

}  // namespace

struct ddp_ctx {
    int32_t R = 0;
    int32_t device = DDP_DEVICE_NONE;
    bool plan_only = true;
    hipStream_t reduce = nullptr, backward = nullptr;
    int64_t wall_clock_khz = 100000;

    // options
    int32_t pipeline = DDP_PIPELINE_STAGED;
    int32_t write_all = 0;
    int32_t timing = 0;
    int32_t nontemporal = 1;
    int64_t coalesce = -1;                        // > 0: consecutive buckets of one API call share a
                                                  // launch while it stays within this many bytes
    int32_t emit_busy_blocks = 0;                 // synthetic backward: 0 = sleeping delay kernel
    int32_t n_streams = -1;                       // reduction streams taken in turn by the launches; -1 = two
                                                  // for launches below cap_min_traffic, one for larger ones
    int32_t chain_launches = 1;                   // flag-ordered launches on alternating streams wait for their predecessor's last block
    unsigned long long launch_ord = 0;            // ordinal of the latest bucket launch that reports its dispatch (monotonic
                                                  // over the context's life)
    unsigned long long prev_launch_ord = 0;       // this iteration's latest such launch (0 = none yet), ...
    int prev_launch_lane = -1;                    // ... the reduction stream it went to (-1 = the backward stream) ...
    int64_t prev_launch_traffic = 0;              // ... and the bytes it moves, (R + 1) x its bucket bytes
    int32_t tail_on_backward = 1;                 // the call that completes an iteration launches on the backward stream
    int32_t blocks_per_cu = -1;                   // reduce kernels: resident blocks per compute unit (0 = no cap,
                                                  // -1 = chosen from R, see auto_blocks_per_cu)
    int64_t cap_min_traffic = int64_t(360) << 20; // ... applied to launches that move at least this many bytes
    int32_t acc_blocks_per_cu = 5;                // accumulate kernel: likewise
    int64_t lds_per_cu = 160 * 1024;              // read from the device at creation

    bool registered = false, built = false;
    ddp::BucketPlan plan;
    ddp::ReadyTracker tracker;
    std::vector<void*> grad_ptrs;            // [R][n], registration order
    std::vector<void*> out_ptrs;             // [n] binary32 output tensors (ddp_set_outputs), else empty

    // device memory owned by the library
    char* slabs = nullptr;                   // R input slabs followed by the output slab
    int64_t slab_stride = 0;
    std::vector<int64_t> bucket_slab_off;    // byte offset of each bucket inside a slab
    std::vector<int64_t> bucket_vecs;        // 16-byte vectors per bucket (padded)
    std::vector<int64_t> h_tile0;            // [G+1]
    void* d_tables = nullptr;                // one allocation holding all segment tables
    int32_t* d_tile_seg = nullptr;           // [tiles] segment index of every tile
    ddp::SegTables tables{};
    // participation flags: [segment][replica], 1 = the replica used the parameter
    int32_t find_unused = 0;                 // 1: parameters nobody used keep their gradients
    std::vector<uint8_t> local_cur;          // running iteration (rows of marked parameters are valid)
    std::vector<uint8_t> acc_used;           // recorded by ddp_no_sync_accumulate since the last finalize
    std::vector<uint8_t> bucket_zero;        // per bucket: some flag of the running iteration is 0
    bool iter_zero = false;                  // any flag of the running iteration is 0
    int64_t iteration = 0;
    int64_t pin_ready_iter = -1;             // iteration for which the pinned staging buffer was claimed
    std::vector<uint8_t> global_closed;      // [n] host view of the closed iteration's global bitmap
    bool global_on_device = false;           // closed iteration: the bitmap kernel ran, result in h_global
    uint8_t* d_local = nullptr;              // [G*R]
    uint8_t* d_global = nullptr;             // [G]
    uint8_t* h_local[2] = {nullptr, nullptr};   // pinned staging, one per iteration parity
    uint8_t* h_global = nullptr;             // pinned
    hipEvent_t ev_local[2] = {nullptr, nullptr};
    hipEvent_t ev_global = nullptr;
    bool local_in_flight[2] = {false, false};
    bool global_in_flight = false;
    void** d_micro = nullptr;
    void** h_micro = nullptr;                // pinned
    void** d_emit = nullptr;
    void** h_emit = nullptr;                 // pinned
    int64_t emit_cap = 0;                    // pointers
    std::vector<hipEvent_t> ev_ready;        // one per bucket
    hipEvent_t ev_done = nullptr, ev_micro = nullptr, ev_emit = nullptr;
    bool micro_in_flight = false, emit_in_flight = false;

    std::vector<std::pair<int32_t, int32_t>> log_running, log_closed;
    std::vector<int32_t> order_running, order_closed;   // ready marks in the order they came (the trace)
    std::vector<uint8_t> used_running, used_closed;
    std::vector<TimedLaunch> timed;
    size_t open_group = static_cast<size_t>(-1);   // timing mode 2: the running iteration's entry
    // Reduction streams: lane 0 is the caller's reduce stream, lanes 1.. are created by the library
    // (DDP_OPT_REDUCE_STREAMS).  The launches of an iteration take the lanes in turn.
    static constexpr int kMaxLanes = 8;
    hipStream_t lane[kMaxLanes] = {};
    hipEvent_t ev_join[kMaxLanes] = {};           // lane's work of the iteration is done (waited for by lane 0)
    hipEvent_t call_event = nullptr;              // backward-stream position of the running API call
    bool lane_used[kMaxLanes] = {};               // lane received work in the running iteration
    bool lane_ordered[kMaxLanes] = {};            // lane already waits for ev_call in the running API call
    int64_t launches_in_iter = 0;
    bool tail_used = false;                       // some launch of the running iteration went to the backward stream
    bool backward_idle_in_call = false;           // backward stream was found drained in this API call
    bool ordered_in_call = false;   // backward stream position of this API call already examined
    int32_t hold_marks = 0;         // DDP_OPT_LAUNCH_HOLD: a launchable bucket waits for up to this many
                                    // further ready marks for its successors to share its launch
    int32_t hold_until = 0;         // ready-mark count at which the held buckets go out at the latest
    std::vector<int32_t> deferred;  // buckets made launchable by the running API call, not yet enqueued

    // Stream ordering through device flags (DDP_OPT_FLAG_ORDER): the backward stream announces a
    // sequence number, a one-wave gate kernel in front of each bucket launch waits for it.
    int32_t flag_order = -1;                      // -1 = where the streams allow it, 0 = never (events)
    int64_t gate_wait_us = 100000;                // bound on one gate's wait
    int32_t num_cus = 256;                        // read from the device at creation
    char* d_order_mem = nullptr;                  // OrderState followed by the two probe words
    ddp::OrderState* d_order = nullptr;
    unsigned long long* d_probe = nullptr;
    // Gate records: kGateRows rows of one record per bucket plus one that summarizes the row
    // ("a gate of this iteration gave up"); iteration i uses row i % kGateRows.
    // Several iterations may be enqueued before the first one's repair launch has run, and a
    // gate of a later iteration that gives up early must not overwrite a record that an
    // earlier iteration's repair launch has yet to read.
    static constexpr int64_t kGateRows = 64;
    ddp::GateRecord* d_gate = nullptr;            // [kGateRows][buckets + 1], allocated with the buckets
    ddp::GateRecord* gate_row() const {
        return d_gate + (iteration % kGateRows) * (static_cast<int64_t>(plan.buckets.size()) + 1);
    }
    int64_t safe_iteration = 0;                   // everything enqueued before this iteration is known to be done
    uint64_t seq_issued = 0;                      // sequence numbers announced so far
    uint64_t probe_value = 0;
    uint64_t call_seq = 0;                        // the number announced for the running API call
    bool call_by_flag = false;                    // the running API call orders its launches by flag
    bool lane_concurrent[kMaxLanes] = {};         // probed: the lane runs concurrently with the backward stream
    int64_t gates_in_iter = 0;                    // gate kernels enqueued in the running iteration
    std::string err;
};

namespace {

int32_t fail(ddp_ctx* c, int32_t code, const std::string& msg) {
    if (c) c->err = msg;
    else g_create_error = msg;
    return code;
}

#define HIPCHK(c, expr)                                                                    \
    do {                                                                                   \
        hipError_t e_ = (expr);                                                            \
        if (e_ != hipSuccess)                                                              \
            return fail((c), DDP_ERR_HIP, std::string(#expr) + ": " + hipGetErrorString(e_)); \
    } while (0)

// Bytes of unused dynamic LDS per block that leave room for exactly
// blocks_per_cu blocks on a compute unit.
// Measured on BERT-large-shaped lists (fp32, launches of the size coalesce_limit
// gives): a block keeps min(R, 8) x 2 loads per thread in flight, so with few
// replicas many blocks are needed (R = 2: 77 % of the HBM peak without a cap,
// 67 % with two blocks; R = 3: 72 % with four, 60 % with two); from R = 5 on two
// blocks are best or close to it (R = 8: 75.6 % against 73.5 % without a cap and
// 71.6 % with one block; R = 12: 74.9 % against 71.9 % with one).  For R >= 16
// one block is 1 to 1.5 points better on lists of large tensors (a block runs
// several eight-replica phases) but 6 points worse on the ResNet-50 list in
// fp16, whose many small tensors put slow boundary tiles on a unit that then
// has nothing else to run -- so two it is, also with binary32 outputs next to 16-bit
// inputs (BERT-large shape in bf16, R = 8, launches of <= 100 MiB: 77.6 % with two or three
// blocks, 74.8 % with four or none, 74.3 % with five).
int32_t auto_blocks_per_cu(int32_t R) { return R <= 4 ? 0 : 2; }

// A launch should run for roughly 150 to 300 us: shorter ones pay their start-up
// and drain, much longer ones lose throughput again.  Bytes of bucket data per
// launch that gave the best rate: R = 2: 400 MiB (67 -> 77 % with no cap),
// R = 4: 240 MiB (76.5 -> 79 %), R = 8: 100 MiB, R = 16: 70 MiB, R = 32: 50 MiB.
int64_t auto_coalesce(int32_t R) {
    const int64_t mib = int64_t(1) << 20;
    return (R <= 2 ? 400 : R <= 4 ? 240 : R <= 8 ? 100 : R <= 16 ? 70 : 50) * mib;
}

int64_t coalesce_limit(const ddp_ctx* c) { return c->coalesce < 0 ? auto_coalesce(c->R) : c->coalesce; }

// A launch is chained to the one in front of it if that one moves at least this many bytes.
constexpr int64_t kChainMinTraffic = int64_t(160) << 20;

// Whether a launch over `launch_bytes` of bucket data is a long one: the cap on resident
// blocks pays, and a second reduction stream does not, from about 360 MiB of traffic on
// (R = 8: 40 MiB of bucket data; R = 32: every 25 MiB bucket, 72.0 against 69.4 % of peak with
// one mark per call; R = 16 likewise 71.7 against 69.4 %).
bool long_launch(const ddp_ctx* c, int64_t launch_bytes) {
    return launch_bytes * (c->R + 1) >= c->cap_min_traffic;
}

unsigned occupancy_lds(const ddp_ctx* c, int64_t launch_bytes) {
    const int32_t blocks = c->blocks_per_cu < 0 ? auto_blocks_per_cu(c->R) : c->blocks_per_cu;
    if (blocks <= 0 || !long_launch(c, launch_bytes)) return 0;
    return static_cast<unsigned>((c->lds_per_cu / blocks) & ~int64_t(1023));
}

unsigned lds_for_blocks(const ddp_ctx* c, int32_t blocks) {
    if (blocks <= 0) return 0;
    return static_cast<unsigned>((c->lds_per_cu / blocks) & ~int64_t(1023));
}

using ddp::make_scale;

// DDP_OPT_TIMING = 1: the launch between timed_begin and timed_end (exactly one kernel) carries a
// pair of events stamped with the kernel's own start and end.
int32_t timed_begin(ddp_ctx* c, int32_t kind, int32_t bucket, hipStream_t s, size_t* slot) {
    (void)s;
    *slot = static_cast<size_t>(-1);
    if (c->timing != 1) return DDP_OK;
    TimedLaunch t{kind, bucket, nullptr, nullptr};
    HIPCHK(c, hipEventCreateWithFlags(&t.start, kTimingEvent));
    HIPCHK(c, hipEventCreateWithFlags(&t.stop, kTimingEvent));
    ddp::time_next_launch(t.start, t.stop);
    c->timed.push_back(t);
    *slot = c->timed.size() - 1;
    return DDP_OK;
}

int32_t timed_end(ddp_ctx* c, size_t slot, hipStream_t s) {
    if (slot == static_cast<size_t>(-1)) return DDP_OK;
    if (ddp::timing_pair_unused()) {
        // nothing was launched (an empty range): an empty interval on the stream
        HIPCHK(c, hipEventRecord(c->timed[slot].start, s));
        HIPCHK(c, hipEventRecord(c->timed[slot].stop, s));
    }
    return DDP_OK;
}

void drop_timed(ddp_ctx* c) {
    for (TimedLaunch& t : c->timed) {
        if (t.start) (void)hipEventDestroy(t.start);
        if (t.stop) (void)hipEventDestroy(t.stop);
    }
    c->timed.clear();
    c->open_group = static_cast<size_t>(-1);
}

// A new API call begins: whatever the caller enqueued on the backward stream
// since the last call has to be ordered before the launches of this one.
void new_call(ddp_ctx* c) {
    c->call_by_flag = false;
    c->ordered_in_call = false;
    c->backward_idle_in_call = false;
    c->call_event = nullptr;
    for (bool& b : c->lane_ordered) b = false;
}

// Whether stream `waiter` makes progress while stream `other` is busy and vice versa.  HIP
// streams that share a hardware queue run one after the other.  The probe is a bounded wait on
// `waiter` for a value written from `other`.
int32_t probe_pair(ddp_ctx* c, hipStream_t waiter, hipStream_t other, bool* concurrent) {
    *concurrent = false;
    if (waiter == other) return DDP_OK;
    HIPCHK(c, hipStreamSynchronize(waiter));
    HIPCHK(c, hipStreamSynchronize(other));
    ++c->probe_value;
    HIPCHK(c, ddp::launch_probe(c->d_probe, c->probe_value, 300 * c->wall_clock_khz / 1000, waiter, other));
    HIPCHK(c, hipStreamSynchronize(waiter));
    HIPCHK(c, hipStreamSynchronize(other));
    unsigned long long seen = 0;
    HIPCHK(c, hipMemcpy(&seen, c->d_probe + 1, sizeof(seen), hipMemcpyDeviceToHost));
    *concurrent = seen == 1;
    return DDP_OK;
}

// Lane l against the backward stream: a gate kernel on a lane that shares the backward
// stream's hardware queue would keep the announcement it waits for from running, so such
// pairs keep events.
int32_t probe_lane(ddp_ctx* c, int l) {
    return probe_pair(c, c->lane[l], c->backward, &c->lane_concurrent[l]);
}

// Creates reduction stream l (default priority, no implicit ordering with the legacy
// default stream).  A new stream may land on the hardware queue of the backward stream, or
// on that of the caller's reduction stream, next to which it is meant to run; a few more are
// tried then (the misfits are destroyed once one fits, so that the next try does not get the
// same queue again).  A stream that runs side by side with both is taken at once; failing
// that, the first one that does so with the backward stream.
int32_t create_lane(ddp_ctx* c, int l) {
    if (c->lane[l]) return DDP_OK;
    hipStream_t tried[7];
    int n_tried = 0, second_best = -1, best = -1;
    while (n_tried < 7 && best < 0) {
        hipStream_t s = nullptr;
        HIPCHK(c, hipStreamCreateWithFlags(&s, hipStreamNonBlocking));
        tried[n_tried] = s;
        bool with_backward = false, with_first = true;
        int32_t rc = probe_pair(c, s, c->backward, &with_backward);
        if (rc == DDP_OK && with_backward && c->lane[0] != c->backward) rc = probe_pair(c, s, c->lane[0], &with_first);
        if (rc != DDP_OK) {
            for (int k = 0; k <= n_tried; ++k) (void)hipStreamDestroy(tried[k]);
            return rc;
        }
        if (with_backward && with_first) best = n_tried;
        else if (with_backward && second_best < 0) second_best = n_tried;
        ++n_tried;
    }
    const int pick = best >= 0 ? best : second_best >= 0 ? second_best : n_tried - 1;
    c->lane[l] = tried[pick];
    c->lane_concurrent[l] = best >= 0 || second_best >= 0;
    for (int k = 0; k < n_tried; ++k)
        if (k != pick) (void)hipStreamDestroy(tried[k]);
    HIPCHK(c, hipEventCreateWithFlags(&c->ev_join[l], kOrderEvent));
    return DDP_OK;
}

// Flags order the launches of the running API call if every reduction stream in use passed
// the probe (fused pipeline only: its kernels carry the gate check).
bool flags_usable(const ddp_ctx* c) {
    if (c->flag_order == 0 || c->pipeline != DDP_PIPELINE_FUSED || c->d_gate == nullptr) return false;
    // (by default the second stream is only used if it passed the probe, see launch_range)
    const int lanes = c->n_streams < 0 ? 1 : c->n_streams;
    for (int l = 0; l < lanes; ++l)
        if (!c->lane_concurrent[l]) return false;
    return true;
}

// Order the launches of the running API call after the gradient-producing work enqueued so
// far: one look at the backward stream, and at most one announcement or event on it, serves
// every bucket the call launches (the caller cannot enqueue anything in the middle of a call).
// If the backward stream has already drained there is nothing to wait for.
int32_t order_call(ddp_ctx* c, int32_t first) {
    if (c->ordered_in_call) return DDP_OK;
    // (a stream that is being captured into a graph cannot be queried: treat it as busy)
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    const bool capturing = hipStreamIsCapturing(c->backward, &cap) == hipSuccess &&
                           cap != hipStreamCaptureStatusNone;
    const bool by_flag = !capturing && flags_usable(c);
    // With flags the announcement is enqueued without first asking whether the backward
    // stream has drained: the question (a stream query takes as long on the host as
    // two launches) would only save the two small kernels when it has.
    const hipError_t q = (capturing || by_flag) ? hipErrorNotReady : hipStreamQuery(c->backward);
    if (q == hipErrorNotReady) {
        if (by_flag) {
            // a one-block kernel instead of an event record (which stalls the stream
            // for about 12 us here)
            c->call_seq = ++c->seq_issued;
            HIPCHK(c, ddp::launch_announce(c->d_order, c->call_seq, c->backward));
            c->call_by_flag = true;
        } else {
            HIPCHK(c, hipEventRecord(c->ev_ready[first], c->backward));
            c->call_event = c->ev_ready[first];
        }
    } else if (q == hipSuccess) {
        c->backward_idle_in_call = true;
        c->safe_iteration = c->iteration;     // every earlier iteration has finished
    } else {
        return fail(c, DDP_ERR_HIP, std::string("hipStreamQuery: ") + hipGetErrorString(q));
    }
    c->ordered_in_call = true;
    return DDP_OK;
}

// Where a launch goes: a reduction stream taken in turn, the backward stream (the API call that
// completes the iteration, see flush_deferred), or the caller's reduction stream as the
// partner of the backward stream when such a call makes several launches.
enum class Target { kLane, kBackward, kPartner };

// Enqueue everything buckets [first, last] need, as one launch per kernel.  The buckets are
// consecutive, hold one element type, and their tiles and slab ranges are contiguous.
int32_t launch_range(ddp_ctx* c, int32_t first, int32_t last, Target target) {
    const ddp::BucketInfo& bf = c->plan.buckets[first];
    const ddp::BucketInfo& bl = c->plan.buckets[last];
    const int seg_begin = bf.seg_begin;
    const int seg_end = bl.seg_begin + static_cast<int>(bl.params.size());
    const int64_t tile_base = c->h_tile0[seg_begin];
    const int64_t ntiles = c->h_tile0[seg_end] - tile_base;
    int64_t bytes = 0;
    for (int32_t b = first; b <= last; ++b) bytes += static_cast<int64_t>(c->plan.buckets[b].bytes());
    const int64_t traffic = bytes * (c->R + 1);
    const int32_t id = first + 65536 * (last - first);
    int lane = -1;                    // -1: the backward stream
    hipStream_t st = c->backward;
    if (target == Target::kLane) {
        // Short launches gain from a neighbour on a second stream (start-up and drain of one
        // overlap with the other); launches long enough for the cap on resident blocks lose
        // when two of them share the memory system, so by default those stay on one stream.
        const int lanes = c->n_streams < 0 ? (!long_launch(c, bytes) && c->lane[1] && c->lane_concurrent[1] ? 2 : 1) : c->n_streams;
        lane = static_cast<int>(c->launches_in_iter++ % lanes);
    } else if (target == Target::kPartner) {
        lane = 0;
    }
    if (lane >= 0 && c->lane[lane] != c->backward) {
        st = c->lane[lane];
        c->lane_used[lane] = true;
    } else {
        lane = -1;
        c->tail_used = true;
    }
    const ddp::GateRecord* gate = nullptr;
    ddp::DispatchSignal sig{nullptr, 0};
    if (lane >= 0 && (!c->lane_ordered[lane] || c->call_by_flag)) {
        const int32_t rc = order_call(c, first);
        if (rc != DDP_OK) return rc;
    }
    // Chained launches.  With flag ordering in use (so the streams are known to run side by
    // side and nothing is being captured), a launch that follows another launch of this
    // iteration on a DIFFERENT stream lets that one reach its last thread block first (a
    // bounded wait: in the gate of a launch on a reduction stream, in a one-wave kernel of its
    // own on the backward stream), so that the two overlap where one drains and the other
    // starts up rather than sharing the memory system all the way (on one stream, stream order
    // does more).  It pays from about 160 MiB moved by the launch in front (measured with one
    // mark per call, gain of chaining: 225 MiB +4.7 to +6.1 %, 170-180 MiB +3.2 to +5.4 %,
    // 125-135 MiB -1.2 to -3.0 %, 45-90 MiB -0.5 to -4.4 %: short launches are mostly start-up
    // and drain, and those overlap best when both run at once).  Two launches that are both
    // long enough for the cap on resident blocks are left alone: in turn on two streams,
    // chained, they lose 1.5 to 3 points against one stream (R = 16 and 32, binary32
    // outputs).  A launch on the backward stream is chained whenever it moves 160 MiB itself:
    // with back-to-back iterations it would otherwise run next to the iteration's first
    // launches for all of its time.
    const bool flags_in_use = c->call_by_flag || c->gates_in_iter > 0;
    const bool both_long = c->prev_launch_traffic >= c->cap_min_traffic && traffic >= c->cap_min_traffic;
    const bool chained = c->chain_launches != 0 && flags_in_use && c->prev_launch_ord != 0 && c->prev_launch_lane != lane &&
                         ntiles > 0 && c->pipeline == DDP_PIPELINE_FUSED &&
                         ((c->prev_launch_traffic >= kChainMinTraffic && !both_long) ||
                          (lane < 0 && traffic >= kChainMinTraffic));
    const long long wait_ticks = c->gate_wait_us * c->wall_clock_khz / 1000;
    if (lane < 0 && chained)
        HIPCHK(c, ddp::launch_chain_wait(c->d_order, c->prev_launch_ord, wait_ticks, st));
    if (lane >= 0 && (!c->lane_ordered[lane] || c->call_by_flag)) {
        if (c->call_by_flag) {
            // every launch gets a gate of its own: if the gate gives up, exactly this launch
            // is skipped and redone by the repair launch of the finalizing step
            if (c->gates_in_iter == 0 && c->iteration - c->safe_iteration >= ddp_ctx::kGateRows - 1) {
                // this iteration's row of gate records was last used kGateRows iterations ago:
                // that iteration's repair launch must have read it (a host that enqueues that
                // many iterations without ever synchronizing waits here once per cycle)
                HIPCHK(c, hipStreamSynchronize(c->backward));
                c->safe_iteration = c->iteration;
            }
            ddp::GateRecord* rec = c->gate_row() + first;
            HIPCHK(c, ddp::launch_gate(c->d_order, c->call_seq, wait_ticks, rec,
                                       c->gate_row() + c->plan.buckets.size(),
                                       static_cast<int32_t>(tile_base), static_cast<int32_t>(ntiles), bf.dtype,
                                       static_cast<uint32_t>(c->iteration + 1),
                                       chained ? c->prev_launch_ord : 0ull, chained ? wait_ticks : 0, st));
            gate = rec;
            ++c->gates_in_iter;
        } else if (!c->backward_idle_in_call) {
            HIPCHK(c, hipStreamWaitEvent(st, c->call_event, 0));
        }
        c->lane_ordered[lane] = true;
    }
    if (c->chain_launches != 0 && (c->call_by_flag || c->gates_in_iter > 0) && ntiles > 0 &&
        c->pipeline == DDP_PIPELINE_FUSED) {
        // the launch reports when its last block starts, for whatever is chained behind it
        sig.word = &c->d_order->dispatched;
        sig.ord = ++c->launch_ord;
        c->prev_launch_ord = sig.ord;
        c->prev_launch_lane = lane;
        c->prev_launch_traffic = traffic;
    }
    // Participation flags travel to the device only for launches that hold a
    // zero flag (a replica that did not use a parameter, or a parameter nobody
    // marked); everything else runs without a flag table.
    const uint8_t* d_flags = nullptr;
    bool need_flags = false;
    for (int32_t b = first; b <= last; ++b) need_flags = need_flags || c->bucket_zero[b] != 0;
    if (need_flags) {
        const int par = static_cast<int>(c->iteration & 1);
        if (c->pin_ready_iter != c->iteration) {      // first use in this iteration: the copies of
            if (c->local_in_flight[par])               // two iterations ago must have left the buffer
                HIPCHK(c, hipEventSynchronize(c->ev_local[par]));
            c->pin_ready_iter = c->iteration;
        }
        const size_t off = static_cast<size_t>(seg_begin) * c->R;
        const size_t len = static_cast<size_t>(seg_end - seg_begin) * c->R;
        std::memcpy(c->h_local[par] + off, c->local_cur.data() + off, len);
        // After the ordering above the stream is also behind the previous iteration's readers of
        // the table; finalize records ev_local[par] once every stream of the iteration is joined.
        HIPCHK(c, hipMemcpyAsync(c->d_local + off, c->h_local[par] + off, len, hipMemcpyHostToDevice, st));
        d_flags = c->d_local;
    }
    const ddp::Scale sc = make_scale(c->R);
    size_t slot;
    int32_t rc;
    if (c->timing == 2 && c->open_group == static_cast<size_t>(-1)) {
        // one event pair per iteration: opened by its first bucket launch
        TimedLaunch t{DDP_K_ITERATION, 0, nullptr, nullptr};
        HIPCHK(c, hipEventCreateWithFlags(&t.start, kTimingEvent));
        HIPCHK(c, hipEventCreateWithFlags(&t.stop, kTimingEvent));
        HIPCHK(c, hipEventRecord(t.start, st));
        c->timed.push_back(t);
        c->open_group = c->timed.size() - 1;
    }
    if (c->timing == 2) c->timed[c->open_group].bucket += 1;   // counts the launches
    if (c->pipeline == DDP_PIPELINE_STAGED) {
        char* in0 = c->slabs + c->bucket_slab_off[first];
        char* out = c->slabs + static_cast<int64_t>(c->R) * c->slab_stride + c->bucket_slab_off[first];
        // the range of the slab from the first bucket's base to the last one's padded end
        const int64_t nvec = (c->bucket_slab_off[last] - c->bucket_slab_off[first]) / 16 + c->bucket_vecs[last];
        if ((rc = timed_begin(c, DDP_K_PACK, id, st, &slot)) != DDP_OK) return rc;
        HIPCHK(c, ddp::launch_pack(c->tables, tile_base, ntiles, c->slabs, c->slab_stride, c->R,
                                   d_flags, st));
        if ((rc = timed_end(c, slot, st)) != DDP_OK) return rc;
        if ((rc = timed_begin(c, DDP_K_REDUCE, id, st, &slot)) != DDP_OK) return rc;
        HIPCHK(c, ddp::launch_flat_reduce(bf.dtype, in0, c->slab_stride, out, nvec, c->R, sc,
                                          c->nontemporal != 0,
                                          occupancy_lds(c, bytes), st));
        if ((rc = timed_end(c, slot, st)) != DDP_OK) return rc;
    } else {
        if ((rc = timed_begin(c, DDP_K_REDUCE, id, st, &slot)) != DDP_OK) return rc;
        HIPCHK(c, ddp::launch_fused_reduce(bf.dtype, c->tables, tile_base, ntiles, c->R,
                                           c->write_all ? c->R : 1, d_flags, c->find_unused != 0, sc,
                                           c->nontemporal != 0, occupancy_lds(c, bytes),
                                           gate, static_cast<uint32_t>(c->iteration + 1), sig, st));
        if ((rc = timed_end(c, slot, st)) != DDP_OK) return rc;
    }
    return DDP_OK;
}

// True if no replica used any parameter of bucket b in the running iteration.
bool bucket_all_unused(const ddp_ctx* c, int32_t b) {
    if (!c->bucket_zero[b]) return false;
    const ddp::BucketInfo& bk = c->plan.buckets[b];
    const size_t begin = static_cast<size_t>(bk.seg_begin) * c->R;
    const size_t end = begin + bk.params.size() * static_cast<size_t>(c->R);
    for (size_t k = begin; k < end; ++k)
        if (c->local_cur[k]) return false;
    return true;
}

// Enqueue the buckets the running API call has made launchable: one launch per
// bucket, or (DDP_OPT_COALESCE) one per run of consecutive buckets of equal
// element type.
int32_t flush_deferred(ddp_ctx* c) {
    if (c->deferred.empty()) return DDP_OK;
    std::vector<int32_t> todo;
    todo.swap(c->deferred);
    if (c->plan_only) return DDP_OK;
    HIPCHK(c, hipSetDevice(c->device));
    // Buckets are launched in index order, so if the last bucket is among the
    // ones this API call launches, every gradient of the iteration has been
    // produced and the backward stream has nothing left to overlap with.  The
    // call's launches then go to the backward stream: stream order replaces
    // the cross-stream event, whose hand-over costs about 0.2 ms here when the
    // waiting queue was armed long before the event fires.  (The staged
    // pipeline keeps its flat buffers and unpack on the reduction stream.)
    const bool closing = c->tail_on_backward != 0 && c->pipeline == DDP_PIPELINE_FUSED &&
                         todo.back() == static_cast<int32_t>(c->plan.buckets.size()) - 1;
    if (c->find_unused != 0 && c->pipeline == DDP_PIPELINE_FUSED && c->iter_zero) {
        // Skipping at the bucket level (Section 6.2.2): a bucket none of whose
        // parameters was used by any replica has nothing to reduce and, with
        // find_unused, nothing to write -- it needs no launch at all.
        size_t kept = 0;
        for (int32_t b : todo)
            if (!bucket_all_unused(c, b)) todo[kept++] = b;
        todo.resize(kept);
        if (todo.empty()) return DDP_OK;
    }
    std::vector<std::pair<int32_t, int32_t>> ranges;      // [first, last] bucket of every launch
    size_t i = 0;
    while (i < todo.size()) {
        size_t j = i;
        const int64_t limit = coalesce_limit(c);
        if (limit > 0) {
            uint64_t bytes = c->plan.buckets[todo[i]].bytes();
            while (j + 1 < todo.size() && todo[j + 1] == todo[j] + 1 &&
                   c->plan.buckets[todo[j + 1]].dtype == c->plan.buckets[todo[i]].dtype &&
                   bytes + c->plan.buckets[todo[j + 1]].bytes() <= static_cast<uint64_t>(limit)) {
                bytes += c->plan.buckets[todo[j + 1]].bytes();
                ++j;
            }
        }
        ranges.emplace_back(todo[i], todo[j]);
        i = j + 1;
    }
    // A closing call that makes several launches: on one stream each launch would start when
    // the one before has drained.  With chained launches they take the backward stream and the
    // caller's reduction stream in turn instead, every launch starting as its predecessor
    // reaches its last thread block.  The announcement that orders the reduction stream's
    // share goes out first, ahead of the backward stream's own launches.
    bool partner = false;
    if (closing && ranges.size() > 1 && c->chain_launches != 0 && c->reduce != c->backward && flags_usable(c)) {
        const int32_t rc = order_call(c, ranges[0].first);
        if (rc != DDP_OK) return rc;
        partner = c->call_by_flag;
    }
    bool prev_on_backward = false, prev_long = false;
    for (size_t k = 0; k < ranges.size(); ++k) {
        int64_t bytes = 0;
        for (int32_t b = ranges[k].first; b <= ranges[k].second; ++b) bytes += static_cast<int64_t>(c->plan.buckets[b].bytes());
        const bool is_long = long_launch(c, bytes);
        // (two long launches do best one after the other on one stream)
        const bool to_partner = partner && k > 0 && prev_on_backward && !(prev_long && is_long);
        const Target target = !closing ? Target::kLane : to_partner ? Target::kPartner : Target::kBackward;
        const int32_t st = launch_range(c, ranges[k].first, ranges[k].second, target);
        if (st != DDP_OK) return st;
        prev_on_backward = target == Target::kBackward;
        prev_long = is_long;
    }
    return DDP_OK;
}

// Bucket b has become launchable: log it and queue it for flush_deferred.
void note_launch(ddp_ctx* c, int32_t b, int32_t call_index) {
    c->log_running.emplace_back(b, call_index);
    c->deferred.push_back(b);
}

// Frees what ddp_build_buckets allocates (also after a build that failed half
// way, so that a retry does not leak).
void release_build(ddp_ctx* c) {
    for (hipEvent_t e : c->ev_ready)
        if (e) (void)hipEventDestroy(e);
    c->ev_ready.clear();
    if (c->slabs) (void)hipFree(c->slabs);
    if (c->d_tables) (void)hipFree(c->d_tables);
    if (c->d_tile_seg) (void)hipFree(c->d_tile_seg);
    if (c->d_local) (void)hipFree(c->d_local);
    if (c->d_global) (void)hipFree(c->d_global);
    if (c->d_micro) (void)hipFree(c->d_micro);
    if (c->d_gate) (void)hipFree(c->d_gate);
    c->d_gate = nullptr;
    for (int k = 0; k < 2; ++k) {
        if (c->h_local[k]) (void)hipHostFree(c->h_local[k]);
        c->h_local[k] = nullptr;
    }
    if (c->h_global) (void)hipHostFree(c->h_global);
    if (c->h_micro) (void)hipHostFree(c->h_micro);
    c->slabs = nullptr; c->d_tables = nullptr; c->d_tile_seg = nullptr; c->d_local = nullptr;
    c->d_global = nullptr; c->d_micro = nullptr; c->h_global = nullptr; c->h_micro = nullptr;
}

void release_device(ddp_ctx* c) {
    if (c->plan_only) return;
    (void)hipSetDevice(c->device);
    if (c->reduce) (void)hipStreamSynchronize(c->reduce);
    if (c->backward) (void)hipStreamSynchronize(c->backward);
    if (!c->reduce || !c->backward) (void)hipStreamSynchronize(nullptr);
    for (int l = 1; l < ddp_ctx::kMaxLanes; ++l) {
        if (c->lane[l]) {
            (void)hipStreamSynchronize(c->lane[l]);
            (void)hipStreamDestroy(c->lane[l]);
            c->lane[l] = nullptr;
        }
        if (c->ev_join[l]) { (void)hipEventDestroy(c->ev_join[l]); c->ev_join[l] = nullptr; }
    }
    drop_timed(c);
    release_build(c);
    for (hipEvent_t* e : {&c->ev_done, &c->ev_micro, &c->ev_emit, &c->ev_local[0], &c->ev_local[1], &c->ev_global})
        if (*e) { (void)hipEventDestroy(*e); *e = nullptr; }
    if (c->d_order_mem) (void)hipFree(c->d_order_mem);
    c->d_order_mem = nullptr; c->d_order = nullptr; c->d_probe = nullptr;
    if (c->d_emit) (void)hipFree(c->d_emit);
    if (c->h_emit) (void)hipHostFree(c->h_emit);
    c->d_emit = nullptr; c->h_emit = nullptr;
}

inline int64_t round_up(int64_t x, int64_t a) { return ddp::round_up_to(x, a); }

}  // namespace

namespace ddp {
int32_t fail_without_context(int32_t code, const std::string& msg) { return fail(nullptr, code, msg); }
}  // namespace ddp

extern "C" {

#ifndef DDP_SOURCE_HASH
#define DDP_SOURCE_HASH "0000000000000000"
#endif
// The build passes a digest of the sources; the Python binding compares it with
// the sources on disk so that a stale library is never tested or measured.
const char* ddp_version(void) { return "ddp_gfx950 0.2 ddp-src-hash:" DDP_SOURCE_HASH; }

const char* ddp_last_error(const ddp_ctx* ctx) {
    return ctx ? ctx->err.c_str() : g_create_error.c_str();
}

int32_t ddp_create(ddp_ctx** out, int32_t R, int32_t device, void* reduce_stream,
                   void* backward_stream) {
    if (!out) return fail(nullptr, DDP_ERR_ARG, "ddp_create: out is null");
    *out = nullptr;
    if (R < 1) return fail(nullptr, DDP_ERR_ARG, "ddp_create: R must be at least 1");
    if (R > DDP_MAX_REPLICAS) return fail(nullptr, DDP_ERR_UNSUPPORTED, "ddp_create: R above DDP_MAX_REPLICAS");
    if (device < DDP_DEVICE_NONE) return fail(nullptr, DDP_ERR_ARG, "ddp_create: bad device");
    ddp_ctx* c = new ddp_ctx();
    c->R = R;
    c->device = device;
    c->plan_only = device == DDP_DEVICE_NONE;
    c->reduce = static_cast<hipStream_t>(reduce_stream);
    c->backward = static_cast<hipStream_t>(backward_stream);
    c->lane[0] = c->reduce;
    if (!c->plan_only) {
        int count = 0;
        hipError_t e = hipGetDeviceCount(&count);
        if (e != hipSuccess || device >= count) {
            delete c;
            return fail(nullptr, DDP_ERR_HIP, "ddp_create: no such HIP device (the library needs a GPU; "
                                              "use DDP_DEVICE_NONE only for plan inspection)");
        }
        e = hipSetDevice(device);
        int khz = 0;
        if (e == hipSuccess) e = hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, device);
        if (e == hipSuccess && khz > 0) c->wall_clock_khz = khz;
        int lds = 0;
        if (e == hipSuccess) e = hipDeviceGetAttribute(&lds, hipDeviceAttributeMaxSharedMemoryPerMultiprocessor, device);
        if (e == hipSuccess && lds >= 64 * 1024) c->lds_per_cu = lds;
        if (e == hipSuccess) e = hipEventCreateWithFlags(&c->ev_done, kOrderEvent);
        if (e == hipSuccess) e = hipEventCreateWithFlags(&c->ev_local[0], hipEventDisableTiming);
        if (e == hipSuccess) e = hipEventCreateWithFlags(&c->ev_local[1], hipEventDisableTiming);
        if (e == hipSuccess) e = hipEventCreateWithFlags(&c->ev_global, hipEventDisableTiming);
        if (e == hipSuccess) e = hipEventCreateWithFlags(&c->ev_micro, hipEventDisableTiming);
        if (e == hipSuccess) e = hipEventCreateWithFlags(&c->ev_emit, hipEventDisableTiming);
        int cus = 0;
        if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device);
        if (e == hipSuccess && cus > 0) c->num_cus = cus;
        const size_t order_bytes = sizeof(ddp::OrderState) + 2 * sizeof(unsigned long long);
        if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&c->d_order_mem), order_bytes);
        if (e == hipSuccess) e = hipMemset(c->d_order_mem, 0, order_bytes);
        if (e == hipSuccess) e = hipDeviceSynchronize();
        if (e != hipSuccess) {
            std::string msg = std::string("ddp_create: ") + hipGetErrorString(e);
            release_device(c);
            delete c;
            return fail(nullptr, DDP_ERR_HIP, msg);
        }
        c->d_order = reinterpret_cast<ddp::OrderState*>(c->d_order_mem);
        c->d_probe = reinterpret_cast<unsigned long long*>(c->d_order_mem + sizeof(ddp::OrderState));
        // the second reduction stream of the default configuration (not when both roles share
        // one stream: then nothing can overlap anyway)
        if (probe_lane(c, 0) != DDP_OK || (c->reduce != c->backward && create_lane(c, 1) != DDP_OK)) {
            std::string msg = "ddp_create: stream probe: " + c->err;
            release_device(c);
            delete c;
            return fail(nullptr, DDP_ERR_HIP, msg);
        }
    }
    *out = c;
    return DDP_OK;
}

int32_t ddp_destroy(ddp_ctx* ctx) {
    if (!ctx) return DDP_ERR_ARG;
    release_device(ctx);
    delete ctx;
    return DDP_OK;
}

int32_t ddp_set_option(ddp_ctx* c, int32_t option, int64_t value) {
    if (!c) return DDP_ERR_ARG;
    switch (option) {
        case DDP_OPT_PIPELINE:
            if (c->built) return fail(c, DDP_ERR_STATE, "pipeline must be chosen before ddp_build_buckets");
            if (value != DDP_PIPELINE_STAGED && value != DDP_PIPELINE_FUSED)
                return fail(c, DDP_ERR_ARG, "unknown pipeline");
            c->pipeline = static_cast<int32_t>(value);
            return DDP_OK;
        case DDP_OPT_WRITE_ALL:
            if (c->built) return fail(c, DDP_ERR_STATE, "write-all must be chosen before ddp_build_buckets");
            c->write_all = value != 0;
            return DDP_OK;
        case DDP_OPT_TIMING:
            if (!c->plan_only) {
                (void)hipSetDevice(c->device);
                drop_timed(c);
            }
            if (value < 0 || value > 2) return fail(c, DDP_ERR_ARG, "timing mode must be 0, 1 or 2");
            c->timing = c->plan_only ? 0 : static_cast<int32_t>(value);
            return DDP_OK;
        case DDP_OPT_EMIT_BUSY_BLOCKS:
            if (value < 0 || value > 4096) return fail(c, DDP_ERR_ARG, "busy blocks outside [0, 4096]");
            c->emit_busy_blocks = static_cast<int32_t>(value);
            return DDP_OK;
        case DDP_OPT_FIND_UNUSED:
            c->find_unused = value != 0;
            return DDP_OK;
        case DDP_OPT_REDUCE_BLOCKS_PER_CU:
            if (value < -1 || value > 16) return fail(c, DDP_ERR_ARG, "blocks per compute unit outside [-1, 16]");
            c->blocks_per_cu = static_cast<int32_t>(value);
            return DDP_OK;
        case DDP_OPT_ACCUMULATE_BLOCKS_PER_CU:
            if (value < 0 || value > 16) return fail(c, DDP_ERR_ARG, "blocks per compute unit outside [0, 16]");
            c->acc_blocks_per_cu = static_cast<int32_t>(value);
            return DDP_OK;
        case DDP_OPT_REDUCE_CAP_MIN_BYTES:
            if (value < 0) return fail(c, DDP_ERR_ARG, "bad size");
            c->cap_min_traffic = value;
            return DDP_OK;
        case DDP_OPT_TAIL_ON_BACKWARD:
            c->tail_on_backward = value != 0;
            return DDP_OK;
        case DDP_OPT_REDUCE_STREAMS:
            if (value != -1 && (value < 1 || value > ddp_ctx::kMaxLanes))
                return fail(c, DDP_ERR_ARG, "number of reduction streams outside [1, 8] and not -1");
            if (c->tracker.marks() != 0 || !c->log_running.empty())
                return fail(c, DDP_ERR_STATE, "reduction streams can only change between iterations");
            if (!c->plan_only) {
                HIPCHK(c, hipSetDevice(c->device));
                for (int l = 1; l < value; ++l) {
                    const int32_t rc = create_lane(c, l);
                    if (rc != DDP_OK) return rc;
                }
            }
            c->n_streams = static_cast<int32_t>(value);
            return DDP_OK;
        case DDP_OPT_LAUNCH_HOLD:
            if (value < 0 || value > 1000000) return fail(c, DDP_ERR_ARG, "launch hold outside [0, 1000000] marks");
            if (c->tracker.marks() != 0 || !c->log_running.empty())
                return fail(c, DDP_ERR_STATE, "the launch hold can only change between iterations");
            c->hold_marks = static_cast<int32_t>(value);
            return DDP_OK;
        case DDP_OPT_FLAG_ORDER:
            if (value != -1 && value != 0) return fail(c, DDP_ERR_ARG, "flag ordering must be -1 (where possible) or 0 (never)");
            if (c->tracker.marks() != 0 || !c->log_running.empty())
                return fail(c, DDP_ERR_STATE, "the ordering mode can only change between iterations");
            c->flag_order = static_cast<int32_t>(value);
            return DDP_OK;
        case DDP_OPT_CHAIN_LAUNCHES:
            c->chain_launches = value != 0;
            return DDP_OK;
        case DDP_OPT_GATE_WAIT_US:
            if (value < 0 || value > 10000000) return fail(c, DDP_ERR_ARG, "gate wait outside [0, 10 s]");
            c->gate_wait_us = value;
            return DDP_OK;
        case DDP_OPT_COALESCE:
            if (value < -1) return fail(c, DDP_ERR_ARG, "bad size");
            c->coalesce = value;
            return DDP_OK;
        case DDP_OPT_NONTEMPORAL:
            c->nontemporal = value != 0;
            return DDP_OK;
        default:
            return fail(c, DDP_ERR_ARG, "unknown option");
    }
}

int32_t ddp_get_option(ddp_ctx* c, int32_t option, int64_t* value) {
    if (!c || !value) return DDP_ERR_ARG;
    switch (option) {
        case DDP_STAT_REPAIRED_LAUNCHES: {
            *value = 0;
            if (c->plan_only) return DDP_OK;
            HIPCHK(c, hipSetDevice(c->device));
            const int32_t rc = ddp_synchronize(c);
            if (rc != DDP_OK) return rc;
            uint32_t n = 0;
            HIPCHK(c, hipMemcpy(&n, &c->d_order->repaired, sizeof(n), hipMemcpyDeviceToHost));
            *value = n;
            return DDP_OK;
        }
        case DDP_OPT_PIPELINE: *value = c->pipeline; return DDP_OK;
        case DDP_OPT_WRITE_ALL: *value = c->write_all; return DDP_OK;
        case DDP_OPT_TIMING: *value = c->timing; return DDP_OK;
        case DDP_OPT_FIND_UNUSED: *value = c->find_unused; return DDP_OK;
        case DDP_OPT_REDUCE_STREAMS: *value = c->n_streams; return DDP_OK;
        case DDP_OPT_COALESCE: *value = coalesce_limit(c); return DDP_OK;
        case DDP_OPT_TAIL_ON_BACKWARD: *value = c->tail_on_backward; return DDP_OK;
        case DDP_OPT_GATE_WAIT_US: *value = c->gate_wait_us; return DDP_OK;
        case DDP_OPT_LAUNCH_HOLD: *value = c->hold_marks; return DDP_OK;
        case DDP_OPT_FLAG_ORDER: *value = flags_usable(c) ? 1 : 0; return DDP_OK;
        case DDP_OPT_CHAIN_LAUNCHES: *value = c->chain_launches; return DDP_OK;
        case DDP_OPT_NONTEMPORAL: *value = c->nontemporal; return DDP_OK;
        case DDP_OPT_EMIT_BUSY_BLOCKS: *value = c->emit_busy_blocks; return DDP_OK;
        case DDP_OPT_REDUCE_BLOCKS_PER_CU: *value = c->blocks_per_cu; return DDP_OK;
        case DDP_OPT_REDUCE_CAP_MIN_BYTES: *value = c->cap_min_traffic; return DDP_OK;
        case DDP_OPT_ACCUMULATE_BLOCKS_PER_CU: *value = c->acc_blocks_per_cu; return DDP_OK;
        default: return fail(c, DDP_ERR_ARG, "unknown option");
    }
}

int32_t ddp_register_params(ddp_ctx* c, int32_t n, const int64_t* numel, const int32_t* dtype,
                            void* const* grad_ptrs) {
    if (!c) return DDP_ERR_ARG;
    if (c->registered) return fail(c, DDP_ERR_STATE, "ddp_register_params called twice");
    if (n <= 0 || !numel || !dtype) return fail(c, DDP_ERR_ARG, "ddp_register_params: n <= 0 or null array");
    if (!c->plan_only && !grad_ptrs) return fail(c, DDP_ERR_ARG, "ddp_register_params: grad_ptrs is null");
    for (int32_t i = 0; i < n; ++i) {
        if (numel[i] < 0) return fail(c, DDP_ERR_ARG, "ddp_register_params: negative numel");
        if (dtype[i] != DDP_FP32 && dtype[i] != DDP_FP16 && dtype[i] != DDP_BF16)
            return fail(c, DDP_ERR_ARG, "ddp_register_params: unknown dtype");
    }
    if (!c->plan_only) {
        for (int32_t r = 0; r < c->R; ++r)
            for (int32_t i = 0; i < n; ++i) {
                const void* p = grad_ptrs[static_cast<int64_t>(r) * n + i];
                if (numel[i] > 0 && !p) return fail(c, DDP_ERR_ARG, "ddp_register_params: null gradient pointer");
                if (reinterpret_cast<uintptr_t>(p) % static_cast<uintptr_t>(ddp::elem_size(dtype[i])) != 0)
                    return fail(c, DDP_ERR_ARG, "ddp_register_params: gradient pointer not aligned to its element size");
            }
        c->grad_ptrs.assign(grad_ptrs, grad_ptrs + static_cast<int64_t>(c->R) * n);
    }
    c->plan.params.resize(n);
    for (int32_t i = 0; i < n; ++i) {
        c->plan.params[i].numel = numel[i];
        c->plan.params[i].dtype = dtype[i];
    }
    c->registered = true;
    return DDP_OK;
}

int32_t ddp_set_outputs(ddp_ctx* c, void* const* out_ptrs) {
    if (!c) return DDP_ERR_ARG;
    if (!c->registered) return fail(c, DDP_ERR_STATE, "ddp_set_outputs before ddp_register_params");
    if (c->built) return fail(c, DDP_ERR_STATE, "ddp_set_outputs after ddp_build_buckets");
    const int32_t n = static_cast<int32_t>(c->plan.params.size());
    for (int32_t i = 0; i < n; ++i)
        if (c->plan.params[i].dtype != DDP_FP16 && c->plan.params[i].dtype != DDP_BF16)
            return fail(c, DDP_ERR_ARG, "ddp_set_outputs: binary32 outputs are for gradients held in fp16 or bf16");
    if (c->plan_only) {            // the plan does not depend on where the averages go
        c->out_ptrs.assign(n, nullptr);
        return DDP_OK;
    }
    if (!out_ptrs) return fail(c, DDP_ERR_ARG, "ddp_set_outputs: out_ptrs is null");
    for (int32_t i = 0; i < n; ++i) {
        if (c->plan.params[i].numel > 0 && !out_ptrs[i]) return fail(c, DDP_ERR_ARG, "ddp_set_outputs: null output pointer");
        if (reinterpret_cast<uintptr_t>(out_ptrs[i]) % 4 != 0)
            return fail(c, DDP_ERR_ARG, "ddp_set_outputs: output pointer not aligned to 4 bytes");
    }
    c->out_ptrs.assign(out_ptrs, out_ptrs + n);
    return DDP_OK;
}

// Assigns the buckets (visiting the parameters in `order`, or in reverse
// registration order without one) and builds everything that depends on the
// assignment: tracker, flag tables, slabs, segment tables, events.
static int32_t build_internal(ddp_ctx* c, uint64_t cap_bytes, const std::vector<int32_t>* order) {
    if (!c->plan.assign(cap_bytes, order)) return fail(c, DDP_ERR_ARG, "visit order is not a permutation");
    c->tracker.reset(c->plan);
    const int32_t n = static_cast<int32_t>(c->plan.params.size());
    const int32_t nb = static_cast<int32_t>(c->plan.buckets.size());
    c->used_running.assign(n, 0);
    c->used_closed.assign(n, 0);
    c->local_cur.assign(static_cast<size_t>(n) * c->R, 0);
    c->acc_used.assign(static_cast<size_t>(n) * c->R, 0);
    c->bucket_zero.assign(nb, 0);
    c->global_closed.assign(n, 0);

    if (!c->plan_only) {
        // slab layout (bucket bases aligned to 256 bytes, lengths padded to 16) and segment
        // tables in bucket-major fill order
        ddp::HostTables ht;
        if (!c->out_ptrs.empty()) {
            if (c->pipeline != DDP_PIPELINE_FUSED)
                return fail(c, DDP_ERR_UNSUPPORTED, "binary32 outputs (ddp_set_outputs) need the fused pipeline");
            if (c->write_all)
                return fail(c, DDP_ERR_UNSUPPORTED, "binary32 outputs (ddp_set_outputs) cannot be combined with DDP_OPT_WRITE_ALL");
        }
        ddp::build_host_tables(c->plan, c->grad_ptrs.data(), c->R, ht, c->out_ptrs.empty() ? nullptr : c->out_ptrs.data());
        c->bucket_slab_off = ht.bucket_slab_off;
        c->bucket_vecs = ht.bucket_vecs;
        c->slab_stride = ht.slab_stride;
        c->h_tile0 = ht.tile0;
        if (c->h_tile0[n] >= (int64_t(1) << 31)) {
            c->built = false;
            return fail(c, DDP_ERR_UNSUPPORTED, "model too large for one launch grid");
        }
        HIPCHK(c, hipSetDevice(c->device));
        release_build(c);   // leftovers of an earlier attempt that failed
        // one allocation for the segment records and the pointer rows
        const int64_t R = c->R;
        const size_t seg_bytes = sizeof(ddp::SegInfo) * n;
        const size_t grad_bytes = sizeof(void*) * ht.grad.size();
        const size_t bytes = seg_bytes + grad_bytes + sizeof(void*) * ht.out.size();
        std::vector<char> host(bytes);
        std::memcpy(host.data(), ht.seg.data(), seg_bytes);
        std::memcpy(host.data() + seg_bytes, ht.grad.data(), grad_bytes);
        if (!ht.out.empty()) std::memcpy(host.data() + seg_bytes + grad_bytes, ht.out.data(), sizeof(void*) * ht.out.size());
        HIPCHK(c, hipMalloc(&c->d_tables, bytes));
        HIPCHK(c, hipMemcpy(c->d_tables, host.data(), bytes, hipMemcpyHostToDevice));
        char* d = static_cast<char*>(c->d_tables);
        c->tables.seg = reinterpret_cast<const ddp::SegInfo*>(d);
        c->tables.grad = reinterpret_cast<void* const*>(d + seg_bytes);
        c->tables.out = ht.out.empty() ? nullptr : reinterpret_cast<void* const*>(d + seg_bytes + grad_bytes);
        c->tables.G = n;
        c->tables.R = c->R;
        {
            const std::vector<int32_t>& tile_seg = ht.tile_seg;
            const size_t tb = sizeof(int32_t) * (tile_seg.empty() ? 1 : tile_seg.size());
            HIPCHK(c, hipMalloc(reinterpret_cast<void**>(&c->d_tile_seg), tb));
            if (!tile_seg.empty())
                HIPCHK(c, hipMemcpy(c->d_tile_seg, tile_seg.data(), sizeof(int32_t) * tile_seg.size(), hipMemcpyHostToDevice));
            c->tables.tile_seg = c->d_tile_seg;
        }

        const size_t flag_bytes = static_cast<size_t>(n) * R;
        HIPCHK(c, hipMalloc(reinterpret_cast<void**>(&c->d_local), flag_bytes + 16));
        HIPCHK(c, hipMalloc(reinterpret_cast<void**>(&c->d_global), static_cast<size_t>(n) + 16));
        for (int k = 0; k < 2; ++k)
            HIPCHK(c, hipHostMalloc(reinterpret_cast<void**>(&c->h_local[k]), flag_bytes, hipHostMallocDefault));
        HIPCHK(c, hipHostMalloc(reinterpret_cast<void**>(&c->h_global), static_cast<size_t>(n), hipHostMallocDefault));
        HIPCHK(c, hipMalloc(reinterpret_cast<void**>(&c->d_micro), sizeof(void*) * R * n));
        HIPCHK(c, hipHostMalloc(reinterpret_cast<void**>(&c->h_micro), sizeof(void*) * R * n, hipHostMallocDefault));
        HIPCHK(c, hipMalloc(reinterpret_cast<void**>(&c->d_gate), sizeof(ddp::GateRecord) * (nb + 1) * ddp_ctx::kGateRows));
        HIPCHK(c, hipMemset(c->d_gate, 0, sizeof(ddp::GateRecord) * (nb + 1) * ddp_ctx::kGateRows));
        c->gates_in_iter = 0;
        c->safe_iteration = c->iteration;
        c->ev_ready.resize(nb, nullptr);
        for (int32_t b = 0; b < nb; ++b)
            HIPCHK(c, hipEventCreateWithFlags(&c->ev_ready[b], kOrderEvent));
        if (c->pipeline == DDP_PIPELINE_STAGED) {
            const size_t total = static_cast<size_t>(c->slab_stride) * static_cast<size_t>(R + 1);
            HIPCHK(c, hipMalloc(reinterpret_cast<void**>(&c->slabs), total));
            HIPCHK(c, hipMemset(c->slabs, 0, total));
        }
        HIPCHK(c, hipDeviceSynchronize());
    }
    c->built = true;
    return nb;
}

int32_t ddp_build_buckets(ddp_ctx* c, uint64_t cap_bytes) {
    if (!c) return DDP_ERR_ARG;
    if (!c->registered) return fail(c, DDP_ERR_STATE, "ddp_build_buckets before ddp_register_params");
    if (c->built) return fail(c, DDP_ERR_STATE, "ddp_build_buckets called twice");
    return build_internal(c, cap_bytes, nullptr);
}

int32_t ddp_rebuild_buckets(ddp_ctx* c, uint64_t cap_bytes) {
    if (!c) return DDP_ERR_ARG;
    if (!c->built) return fail(c, DDP_ERR_STATE, "ddp_rebuild_buckets before ddp_build_buckets");
    if (c->tracker.marks() != 0 || !c->deferred.empty())
        return fail(c, DDP_ERR_STATE, "ddp_rebuild_buckets in the middle of an iteration");
    for (uint8_t u : c->acc_used)
        if (u) return fail(c, DDP_ERR_STATE, "ddp_rebuild_buckets between a no_sync accumulation and its synchronization");
    const int32_t n = static_cast<int32_t>(c->plan.params.size());
    // visit order: the trace of the closed iteration, then what it never saw in
    // reverse registration order
    std::vector<int32_t> order = c->order_closed;
    {
        std::vector<uint8_t> seen(n, 0);
        for (int32_t p : order) seen[p] = 1;
        for (int32_t i = n - 1; i >= 0; --i)
            if (!seen[i]) order.push_back(i);
    }
    if (!c->plan_only) {
        // nothing may still use the tables, slabs and staging buffers that are about to be freed
        HIPCHK(c, hipSetDevice(c->device));
        HIPCHK(c, hipStreamSynchronize(c->backward));
        for (int l = 1; l < ddp_ctx::kMaxLanes; ++l)
            if (c->lane[l]) HIPCHK(c, hipStreamSynchronize(c->lane[l]));
        HIPCHK(c, hipStreamSynchronize(c->reduce));
        if (c->global_on_device) {      // keep the closed iteration's bitmap readable
            for (int32_t i = 0; i < n; ++i) c->global_closed[i] = c->h_global[c->plan.params[i].segment];
            c->global_on_device = false;
        }
        drop_timed(c);
        c->local_in_flight[0] = c->local_in_flight[1] = false;
        c->global_in_flight = false;
        c->micro_in_flight = false;
        c->pin_ready_iter = -1;
    }
    const std::vector<uint8_t> keep_global = c->global_closed, keep_used = c->used_closed;
    c->built = false;
    const int32_t nb = build_internal(c, cap_bytes, &order);
    if (nb < 0) return nb;
    c->global_closed = keep_global;     // indexed by parameter: unaffected by the new mapping
    c->used_closed = keep_used;
    c->log_closed.clear();              // its bucket numbers belong to the old mapping
    return nb;
}

int32_t ddp_get_ready_order(const ddp_ctx* c, int32_t which, int32_t* ids, int32_t cap, int32_t* n) {
    if (!c || !n || cap < 0 || (which != 0 && which != 1)) return DDP_ERR_ARG;
    if (!c->built) return DDP_ERR_STATE;
    const std::vector<int32_t>& o = which == 0 ? c->order_running : c->order_closed;
    *n = static_cast<int32_t>(o.size());
    for (int32_t i = 0; i < *n && i < cap; ++i)
        if (ids) ids[i] = o[i];
    return DDP_OK;
}

int32_t ddp_get_assignment(const ddp_ctx* c, int32_t* bucket_of, int64_t* elem_offset) {
    if (!c || !bucket_of || !elem_offset) return DDP_ERR_ARG;
    if (!c->built) return DDP_ERR_STATE;
    for (size_t i = 0; i < c->plan.params.size(); ++i) {
        bucket_of[i] = c->plan.params[i].bucket;
        elem_offset[i] = c->plan.params[i].offset;
    }
    return DDP_OK;
}

int32_t ddp_get_bucket_info(const ddp_ctx* c, int32_t b, int64_t* elems, int32_t* n_params,
                            int32_t* dtype) {
    if (!c) return DDP_ERR_ARG;
    if (!c->built) return DDP_ERR_STATE;
    if (b < 0 || b >= static_cast<int32_t>(c->plan.buckets.size())) return DDP_ERR_ARG;
    const ddp::BucketInfo& bk = c->plan.buckets[b];
    if (elems) *elems = bk.elems;
    if (n_params) *n_params = static_cast<int32_t>(bk.params.size());
    if (dtype) *dtype = bk.dtype;
    return DDP_OK;
}

int32_t ddp_get_bucket_ptr(const ddp_ctx* c, int32_t b, int32_t r, void** ptr) {
    if (!c || !ptr) return DDP_ERR_ARG;
    if (!c->built) return DDP_ERR_STATE;
    if (c->plan_only) return DDP_ERR_NO_DEVICE;
    if (c->pipeline != DDP_PIPELINE_STAGED || !c->slabs) return DDP_ERR_STATE;
    if (b < 0 || b >= static_cast<int32_t>(c->plan.buckets.size()) || r < -1 || r >= c->R) return DDP_ERR_ARG;
    const int64_t slab = r < 0 ? c->R : r;
    *ptr = c->slabs + slab * c->slab_stride + c->bucket_slab_off[b];
    return DDP_OK;
}

// Writes the participation row of a parameter: used[r] (null = every replica),
// OR what no_sync iterations recorded.  Returns whether any replica used it.
static bool set_participation(ddp_ctx* c, int32_t param_id, const uint8_t* used) {
    const ddp::ParamInfo& p = c->plan.params[param_id];
    const size_t row = static_cast<size_t>(p.segment) * c->R;
    bool any = false, zero = false;
    for (int32_t r = 0; r < c->R; ++r) {
        const uint8_t eff = ((used == nullptr || used[r] != 0) || c->acc_used[row + r] != 0) ? 1 : 0;
        c->local_cur[row + r] = eff;
        any = any || eff != 0;
        zero = zero || eff == 0;
    }
    if (zero) {
        c->bucket_zero[p.bucket] = 1;
        c->iter_zero = true;
    }
    return any;
}

// What a single ready-mark call does with the buckets that are launchable: enqueue them now
// (the default: Algorithm 1 launches a bucket as soon as it is ready), or, with
// DDP_OPT_LAUNCH_HOLD, keep them back for a bounded number of further marks so that buckets
// that become ready shortly afterwards share their launch.
static int32_t flush_or_hold(ddp_ctx* c) {
    if (c->deferred.empty() || c->hold_marks <= 0) return flush_deferred(c);
    const int32_t last = static_cast<int32_t>(c->plan.buckets.size()) - 1;
    bool now = c->deferred.back() == last || c->tracker.marks() >= c->hold_until;
    if (!now) {
        uint64_t bytes = 0;
        for (int32_t b : c->deferred) bytes += c->plan.buckets[b].bytes();
        const int64_t limit = coalesce_limit(c);
        now = limit <= 0 || bytes >= static_cast<uint64_t>(limit);     // nothing more fits into the launch
    }
    return now ? flush_deferred(c) : DDP_OK;
}

static int32_t mark_one(ddp_ctx* c, int32_t param_id, const uint8_t* used) {
    std::vector<int32_t> launch;
    const int rc = c->tracker.mark(param_id, launch);
    if (rc == -1) return fail(c, DDP_ERR_ARG, "ddp_mark_ready: parameter id out of range");
    if (rc == -2) return fail(c, DDP_ERR_ALREADY_READY, "ddp_mark_ready: parameter already marked in this iteration");
    c->order_running.push_back(param_id);
    if (set_participation(c, param_id, used)) c->used_running[param_id] = 1;
    for (int32_t b : launch) note_launch(c, b, c->tracker.marks() - 1);
    if (!launch.empty()) c->hold_until = c->tracker.marks() + c->hold_marks;
    if (coalesce_limit(c) <= 0) return flush_deferred(c);
    return DDP_OK;
}

int32_t ddp_mark_ready(ddp_ctx* c, int32_t param_id) {
    if (!c) return DDP_ERR_ARG;
    if (!c->built) return fail(c, DDP_ERR_STATE, "ddp_mark_ready before ddp_build_buckets");
    new_call(c);
    const int32_t st = mark_one(c, param_id, nullptr);
    if (st != DDP_OK) return st;
    return flush_or_hold(c);
}

int32_t ddp_mark_ready_local(ddp_ctx* c, int32_t param_id, const uint8_t* used) {
    if (!c) return DDP_ERR_ARG;
    if (!c->built) return fail(c, DDP_ERR_STATE, "ddp_mark_ready_local before ddp_build_buckets");
    if (!used) return fail(c, DDP_ERR_ARG, "ddp_mark_ready_local: used is null");
    new_call(c);
    const int32_t st = mark_one(c, param_id, used);
    if (st != DDP_OK) return st;
    return flush_or_hold(c);
}

int32_t ddp_mark_ready_many(ddp_ctx* c, const int32_t* ids, int32_t count) {
    if (!c || (count > 0 && !ids) || count < 0) return DDP_ERR_ARG;
    if (!c->built) return fail(c, DDP_ERR_STATE, "ddp_mark_ready_many before ddp_build_buckets");
    new_call(c);
    for (int32_t k = 0; k < count; ++k) {
        const int32_t st = mark_one(c, ids[k], nullptr);
        if (st != DDP_OK) {
            (void)flush_deferred(c);   // what the earlier marks completed is still launched
            return st;
        }
    }
    return flush_deferred(c);
}

int32_t ddp_finalize_backward(ddp_ctx* c) {
    if (!c) return DDP_ERR_ARG;
    if (!c->built) return fail(c, DDP_ERR_STATE, "ddp_finalize_backward before ddp_build_buckets");
    const int32_t n = static_cast<int32_t>(c->plan.params.size());
    const int32_t marks = c->tracker.marks();
    new_call(c);
    std::vector<int32_t> launch;
    c->tracker.drain(launch);
    if (!c->plan_only) HIPCHK(c, hipSetDevice(c->device));
    if (marks < n) {
        // Parameters never marked in this iteration: what earlier no_sync
        // iterations recorded still counts (Section 3.2.4); replicas without any
        // record contribute zeros and are not read.  Every bucket launched
        // before this point was complete, so only the buckets in `launch` can
        // contain such parameters.
        for (int32_t i = 0; i < n; ++i)
            if (!c->tracker.marked(i)) {
                static const uint8_t nobody[DDP_MAX_REPLICAS] = {0};
                if (set_participation(c, i, nobody)) c->used_running[i] = 1;
            }
    }
    for (int32_t b : launch) note_launch(c, b, marks);
    {
        const int32_t st = flush_deferred(c);
        if (st != DDP_OK) return st;
    }
    if (!c->plan_only) {
        // Fused pipeline, no bitmap step: nothing else runs on the reduction side at finalize, and
        // every reduction stream that received work joins the backward stream directly.  If the
        // iteration's launches were ordered by device flags, so is the way back: each stream
        // stores the iteration's tag behind its last launch and one kernel on the backward
        // stream waits for the tags; the events behind it have fired by then.
        const bool direct_join = c->pipeline == DDP_PIPELINE_FUSED && !c->iter_zero;
        bool reduce_side_used = c->lane_used[0];
        if (direct_join) {
            const bool by_flag = c->gates_in_iter > 0;
            const unsigned long long tag = static_cast<unsigned long long>(c->iteration + 1);
            uint32_t mask = 0;
            for (int l = 0; l < ddp_ctx::kMaxLanes; ++l)
                if (c->lane_used[l] && c->lane[l] != c->backward) {
                    HIPCHK(c, hipEventRecord(l == 0 ? c->ev_done : c->ev_join[l], c->lane[l]));
                    if (by_flag) HIPCHK(c, ddp::launch_done(c->d_order, l, tag, c->lane[l]));
                    mask |= 1u << l;
                }
            if (by_flag && mask)
                HIPCHK(c, ddp::launch_join(c->d_order, mask, tag, c->gate_wait_us * c->wall_clock_khz / 1000, c->backward));
            for (int l = 0; l < ddp_ctx::kMaxLanes; ++l)
                if ((mask >> l) & 1u) HIPCHK(c, hipStreamWaitEvent(c->backward, l == 0 ? c->ev_done : c->ev_join[l], 0));
            if (mask) c->tail_used = true;       // the iteration's launches end on the backward stream
            reduce_side_used = false;            // (joined already)
        } else {
            // every reduction stream that received work in this iteration joins the caller's
            for (int l = 1; l < ddp_ctx::kMaxLanes; ++l)
                if (c->lane_used[l]) {
                    HIPCHK(c, hipEventRecord(c->ev_join[l], c->lane[l]));
                    HIPCHK(c, hipStreamWaitEvent(c->reduce, c->ev_join[l], 0));
                    reduce_side_used = true;
                }
        }
        // the interval of this iteration's bucket launches ends here if all of them ran on the
        // reduction side, else on the backward stream below
        // an iteration that used gates ends with the repair launch on the backward stream
        if (c->gates_in_iter > 0) c->tail_used = true;
        if (c->open_group != static_cast<size_t>(-1) && !c->tail_used) {
            HIPCHK(c, hipEventRecord(c->timed[c->open_group].stop, c->reduce));
            c->open_group = static_cast<size_t>(-1);
        }
        const int par = static_cast<int>(c->iteration & 1);
        if (c->iter_zero) {
            // The bitmap step of Section 4.2: the host bitmap goes to the device
            // with a non-blocking copy and one extra reduction (an OR over the
            // replicas) yields the parameters that somebody used.
            if (c->pin_ready_iter != c->iteration) {
                if (c->local_in_flight[par]) HIPCHK(c, hipEventSynchronize(c->ev_local[par]));
                c->pin_ready_iter = c->iteration;
            }
            const size_t flag_bytes = static_cast<size_t>(n) * c->R;
            std::memcpy(c->h_local[par], c->local_cur.data(), flag_bytes);
            HIPCHK(c, hipMemcpyAsync(c->d_local, c->h_local[par], flag_bytes, hipMemcpyHostToDevice, c->reduce));
            HIPCHK(c, ddp::launch_bitmap_or(c->d_local, c->d_global, n, c->R, c->reduce));
            if (c->global_in_flight) HIPCHK(c, hipEventSynchronize(c->ev_global));
            HIPCHK(c, hipMemcpyAsync(c->h_global, c->d_global, static_cast<size_t>(n), hipMemcpyDeviceToHost, c->reduce));
            HIPCHK(c, hipEventRecord(c->ev_global, c->reduce));
            c->global_in_flight = true;
            reduce_side_used = true;
        }
        if (c->pipeline == DDP_PIPELINE_STAGED) {
            size_t slot;
            int32_t rc;
            if ((rc = timed_begin(c, DDP_K_UNPACK, -1, c->reduce, &slot)) != DDP_OK) return rc;
            HIPCHK(c, ddp::launch_unpack(c->tables, 0, c->h_tile0[n],
                                         c->slabs + static_cast<int64_t>(c->R) * c->slab_stride,
                                         c->write_all ? c->R : 1, c->iter_zero ? c->d_global : nullptr,
                                         c->find_unused != 0, c->reduce));
            if ((rc = timed_end(c, slot, c->reduce)) != DDP_OK) return rc;
            reduce_side_used = true;
        }
        // the backward stream waits for whatever ran on the reduction side
        if (c->backward != c->reduce && reduce_side_used) {
            HIPCHK(c, hipEventRecord(c->ev_done, c->reduce));
            HIPCHK(c, hipStreamWaitEvent(c->backward, c->ev_done, 0));
        }
        if (c->gates_in_iter > 0) {
            // Gates wait a bounded time.  Launches whose gate gave up did nothing; they are
            // redone now that every gradient exists (normally there is none and the launch
            // ends at once).  With a zero participation flag in the iteration the whole
            // bitmap is on the device by now (copied above on the reduction stream).
            uint32_t dtypes_seen = 0;
            for (const ddp::BucketInfo& bk : c->plan.buckets) dtypes_seen |= 1u << bk.dtype;
            for (int dt = 0; dt < 3; ++dt)
                if (dtypes_seen & (1u << dt))
                    HIPCHK(c, ddp::launch_repair(dt, c->tables, c->d_order,
                                                 c->gate_row(),
                                                 static_cast<int>(c->plan.buckets.size()),
                                                 static_cast<uint32_t>(c->iteration + 1), c->R,
                                                 c->write_all ? c->R : 1, c->iter_zero ? c->d_local : nullptr,
                                                 c->find_unused != 0, make_scale(c->R), 2 * c->num_cus,
                                                 c->nontemporal != 0, c->backward));
        }
        // from here on the backward stream is behind everything of this iteration
        if (c->pin_ready_iter == c->iteration) {      // the flag staging buffer was used: free for reuse after this
            HIPCHK(c, hipEventRecord(c->ev_local[par], c->backward));
            c->local_in_flight[par] = true;
        }
        if (c->open_group != static_cast<size_t>(-1)) {      // closes this iteration's bucket launches
            HIPCHK(c, hipEventRecord(c->timed[c->open_group].stop, c->backward));
            c->open_group = static_cast<size_t>(-1);
        }
    }
    c->log_closed.swap(c->log_running);
    c->log_running.clear();
    c->order_closed.swap(c->order_running);
    c->order_running.clear();
    c->used_closed = c->used_running;
    std::fill(c->used_running.begin(), c->used_running.end(), 0);
    // host view of the global bitmap (all ones unless a flag was zero)
    for (int32_t i = 0; i < n; ++i) {
        const size_t row = static_cast<size_t>(c->plan.params[i].segment) * c->R;
        uint8_t any = 0;
        for (int32_t r = 0; r < c->R; ++r) any |= c->local_cur[row + r];
        c->global_closed[i] = any;
    }
    c->global_on_device = c->iter_zero && !c->plan_only;
    std::fill(c->acc_used.begin(), c->acc_used.end(), 0);
    std::fill(c->bucket_zero.begin(), c->bucket_zero.end(), 0);
    c->iter_zero = false;
    for (bool& b : c->lane_used) b = false;
    c->launches_in_iter = 0;
    c->tail_used = false;
    c->gates_in_iter = 0;
    c->prev_launch_ord = 0;
    ++c->iteration;
    c->tracker.new_iteration();
    return DDP_OK;
}

int32_t ddp_get_global_used(ddp_ctx* c, uint8_t* used) {
    if (!c || !used) return DDP_ERR_ARG;
    if (!c->built) return DDP_ERR_STATE;
    const int32_t n = static_cast<int32_t>(c->plan.params.size());
    if (c->global_on_device) {
        // what the bitmap kernel computed, brought back by the copy enqueued at finalize
        HIPCHK(c, hipSetDevice(c->device));
        HIPCHK(c, hipEventSynchronize(c->ev_global));
        for (int32_t i = 0; i < n; ++i) used[i] = c->h_global[c->plan.params[i].segment];
    } else {
        std::memcpy(used, c->global_closed.data(), static_cast<size_t>(n));
    }
    return DDP_OK;
}

int32_t ddp_synchronize(ddp_ctx* c) {
    if (!c) return DDP_ERR_ARG;
    if (c->plan_only) return fail(c, DDP_ERR_NO_DEVICE, "plan-only context has nothing to wait for");
    HIPCHK(c, hipSetDevice(c->device));
    HIPCHK(c, hipStreamSynchronize(c->backward));
    for (int l = 1; l < ddp_ctx::kMaxLanes; ++l)
        if (c->lane[l]) HIPCHK(c, hipStreamSynchronize(c->lane[l]));
    HIPCHK(c, hipStreamSynchronize(c->reduce));
    c->safe_iteration = c->iteration;
    return DDP_OK;
}

int32_t ddp_get_launch_log(const ddp_ctx* c, int32_t which, int32_t* bucket_ids,
                           int32_t* after_call, int32_t cap, int32_t* n) {
    if (!c || !n || cap < 0 || (which != 0 && which != 1)) return DDP_ERR_ARG;
    const auto& log = which == 0 ? c->log_running : c->log_closed;
    *n = static_cast<int32_t>(log.size());
    for (int32_t i = 0; i < *n && i < cap; ++i) {
        if (bucket_ids) bucket_ids[i] = log[i].first;
        if (after_call) after_call[i] = log[i].second;
    }
    return DDP_OK;
}

int32_t ddp_no_sync_accumulate(ddp_ctx* c, void* const* micro) {
    if (!c) return DDP_ERR_ARG;
    if (!c->built) return fail(c, DDP_ERR_STATE, "ddp_no_sync_accumulate before ddp_build_buckets");
    // Section 3.2.4's no_sync covers whole iterations: once a ready mark has been taken, buckets
    // may already be reducing these very tensors in place on another stream.
    if (c->tracker.marks() != 0 || !c->deferred.empty())
        return fail(c, DDP_ERR_STATE, "ddp_no_sync_accumulate in the middle of a synchronizing iteration");
    if (c->plan_only) return fail(c, DDP_ERR_NO_DEVICE, "plan-only context cannot accumulate");
    if (!micro) return fail(c, DDP_ERR_ARG, "ddp_no_sync_accumulate: null pointer array");
    const int32_t n = static_cast<int32_t>(c->plan.params.size());
    const int64_t R = c->R;
    for (int64_t r = 0; r < R; ++r)
        for (int32_t i = 0; i < n; ++i) {
            const void* p = micro[r * n + i];
            if (p && reinterpret_cast<uintptr_t>(p) % static_cast<uintptr_t>(ddp::elem_size(c->plan.params[i].dtype)) != 0)
                return fail(c, DDP_ERR_ARG, "ddp_no_sync_accumulate: pointer not aligned to its element size");
        }
    HIPCHK(c, hipSetDevice(c->device));
    if (c->micro_in_flight) HIPCHK(c, hipEventSynchronize(c->ev_micro));
    std::memcpy(c->h_micro, micro, sizeof(void*) * R * n);
    HIPCHK(c, hipMemcpyAsync(c->d_micro, c->h_micro, sizeof(void*) * R * n, hipMemcpyHostToDevice, c->backward));
    HIPCHK(c, hipEventRecord(c->ev_micro, c->backward));
    c->micro_in_flight = true;
    size_t slot;
    int32_t rc;
    if ((rc = timed_begin(c, DDP_K_ACCUMULATE, -1, c->backward, &slot)) != DDP_OK) return rc;
    HIPCHK(c, ddp::launch_accumulate(c->tables, c->h_tile0[n], c->R, n, c->d_micro,
                                     lds_for_blocks(c, c->acc_blocks_per_cu), c->backward));
    if ((rc = timed_end(c, slot, c->backward)) != DDP_OK) return rc;
    for (int32_t i = 0; i < n; ++i) {
        const size_t row = static_cast<size_t>(c->plan.params[i].segment) * R;
        for (int64_t r = 0; r < R; ++r)
            if (micro[r * n + i]) {
                c->acc_used[row + r] = 1;
                c->used_running[i] = 1;
            }
    }
    return DDP_OK;
}

int32_t ddp_get_used_map(const ddp_ctx* c, int32_t which, uint8_t* used) {
    if (!c || !used || (which != 0 && which != 1)) return DDP_ERR_ARG;
    if (!c->built) return DDP_ERR_STATE;
    const auto& m = which == 0 ? c->used_running : c->used_closed;
    std::memcpy(used, m.data(), m.size());
    return DDP_OK;
}

int32_t ddp_synth_backward(ddp_ctx* c, const int32_t* order, int32_t count, const int64_t* delay_ns,
                           void* const* src_ptrs, int32_t mark) {
    if (!c) return DDP_ERR_ARG;
    if (!c->built) return fail(c, DDP_ERR_STATE, "ddp_synth_backward before ddp_build_buckets");
    if (c->plan_only) return fail(c, DDP_ERR_NO_DEVICE, "plan-only context cannot run a backward pass");
    if (count < 0 || (count > 0 && !order)) return fail(c, DDP_ERR_ARG, "ddp_synth_backward: bad order");
    const int32_t n = static_cast<int32_t>(c->plan.params.size());
    const int64_t R = c->R;
    for (int32_t k = 0; k < count; ++k) {
        if (order[k] < 0 || order[k] >= n) return fail(c, DDP_ERR_ARG, "ddp_synth_backward: id out of range");
        if (delay_ns && (delay_ns[k] < 0 || delay_ns[k] > 100000000))
            return fail(c, DDP_ERR_ARG, "ddp_synth_backward: delay outside [0, 100 ms]");
    }
    HIPCHK(c, hipSetDevice(c->device));
    new_call(c);
    void** d_rows = nullptr;
    if (src_ptrs && count > 0) {
        const int64_t need = 2 * R * count;
        if (c->emit_in_flight) HIPCHK(c, hipEventSynchronize(c->ev_emit));
        if (need > c->emit_cap) {
            HIPCHK(c, hipStreamSynchronize(c->backward));
            if (c->d_emit) HIPCHK(c, hipFree(c->d_emit));
            if (c->h_emit) HIPCHK(c, hipHostFree(c->h_emit));
            c->d_emit = nullptr; c->h_emit = nullptr; c->emit_cap = 0;
            HIPCHK(c, hipMalloc(reinterpret_cast<void**>(&c->d_emit), sizeof(void*) * need));
            HIPCHK(c, hipHostMalloc(reinterpret_cast<void**>(&c->h_emit), sizeof(void*) * need, hipHostMallocDefault));
            c->emit_cap = need;
        }
        for (int32_t k = 0; k < count; ++k)
            for (int64_t r = 0; r < R; ++r) {
                void* src = src_ptrs[r * n + order[k]];
                if (!src && c->plan.params[order[k]].numel > 0)
                    return fail(c, DDP_ERR_ARG, "ddp_synth_backward: null source pointer");
                c->h_emit[2 * R * k + r] = c->grad_ptrs[r * n + order[k]];
                c->h_emit[2 * R * k + R + r] = src;
            }
        HIPCHK(c, hipMemcpyAsync(c->d_emit, c->h_emit, sizeof(void*) * need, hipMemcpyHostToDevice, c->backward));
        HIPCHK(c, hipEventRecord(c->ev_emit, c->backward));
        c->emit_in_flight = true;
        d_rows = c->d_emit;
    }
    for (int32_t k = 0; k < count; ++k) {
        const int32_t p = order[k];
        const int64_t ticks = delay_ns ? delay_ns[k] * c->wall_clock_khz / 1000000 : 0;
        if (ticks > 0 || d_rows) {
            // buckets completed so far go out before more backward work is enqueued
            // (unless a launch hold keeps them back for a few more marks)
            const int32_t stf = flush_or_hold(c);
            if (stf != DDP_OK) return stf;
            new_call(c);
            HIPCHK(c, ddp::launch_emit(ticks, d_rows ? d_rows + 2 * R * k : nullptr, c->R,
                                       c->plan.params[p].numel, ddp::elem_size(c->plan.params[p].dtype),
                                       c->emit_busy_blocks,
                                       reinterpret_cast<float*>(c->d_global + round_up(n, 4)),   // spare tail
                                       c->backward));
        }
        if (mark) {
            const int32_t st = mark_one(c, p, nullptr);
            if (st != DDP_OK) {
                (void)flush_deferred(c);
                return st;
            }
        }
    }
    // with marks this is a call that delivers many of them: what they completed goes out now
    return mark ? flush_deferred(c) : flush_or_hold(c);
}

int32_t ddp_get_kernel_times(ddp_ctx* c, int32_t kind, float* ms, int32_t* ids, int32_t cap,
                             int32_t* n) {
    if (!c || !n || cap < 0) return DDP_ERR_ARG;
    if (c->plan_only) return fail(c, DDP_ERR_NO_DEVICE, "plan-only context has no kernel times");
    HIPCHK(c, hipSetDevice(c->device));
    int32_t k = 0;
    for (const TimedLaunch& t : c->timed) {
        if (t.kind != kind) continue;
        if (k < cap) {
            float v = 0.f;
            HIPCHK(c, hipEventElapsedTime(&v, t.start, t.stop));
            if (ms) ms[k] = v;
            if (ids) ids[k] = t.bucket;
        }
        ++k;
    }
    *n = k;
    return DDP_OK;
}

}  // extern "C"
