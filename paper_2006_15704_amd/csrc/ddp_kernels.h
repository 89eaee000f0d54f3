// Launch wrappers of the HIP kernels (gfx950).  Internal to the library.
#pragma once
#include <hip/hip_runtime.h>
#include <cstdint>

namespace ddp {

// Work is cut into tiles of TILE_BYTES of gradient data: one thread block of
// BLOCK threads moves TILE_VECS 16-byte vectors per replica.  8 KiB tiles (two
// vectors per thread and replica) measured best: 16 KiB tiles with two or four
// vectors per thread were 1 to 4 points of HBM peak slower on the ResNet-50-
// and BERT-large-shaped lists under every cap on resident blocks.
constexpr int BLOCK = 256;
#ifndef DDP_TILE_VECS
#define DDP_TILE_VECS 512
#endif
constexpr int TILE_VECS = DDP_TILE_VECS;
constexpr int TILE_BYTES = TILE_VECS * 16;

// Tiles of a segment.  Vectors are cut at 16-byte boundaries of the
// destination, so a destination that starts `lead_bytes` (< 16) past such a
// boundary shifts the grid by that much; the caller passes the largest lead-in
// over all destinations the segment can have.
inline int64_t tiles_for(int64_t numel, int es, int lead_bytes) {
    if (numel <= 0) return 0;
    return (numel * es + lead_bytes + TILE_BYTES - 1) / TILE_BYTES;
}

// Device-resident tables over the G segments (parameters in bucket-major fill
// order) of the model.
struct SegInfo {               // 32 bytes, read with one scalar load
    int64_t numel;             // elements
    int64_t tile0;             // first tile of the segment in the global tile numbering
    int64_t flat_byte;         // byte offset of the segment inside a replica slab
    int32_t param;             // registration index
    int32_t flags;             // bits 0-7: element type; bit 8: all R gradient tensors share
                               // replica 0's address modulo 16; bits 16-19: that address
                               // modulo 16 (replica 0)
    __host__ __device__ int dtype() const { return flags & 0xFF; }
    __host__ __device__ bool congruent() const { return (flags & 0x100) != 0; }
    // bit 9 (binary32 outputs only): the output tensor's address modulo 16 equals twice
    // replica 0's address modulo 16, so whole input vectors map to whole output vectors
    __host__ __device__ bool out_congruent() const { return (flags & 0x200) != 0; }
    __host__ __device__ int lead_bytes() const { return (flags >> 16) & 0xF; }
};

struct SegTables {
    const SegInfo* seg;        // [G]
    const int32_t* tile_seg;   // [tiles] segment that each tile belongs to
    void* const* grad;         // [G*R + 8] replica r's gradient of segment g at [g*R+r]; eight
                               // null entries of padding so that any row can be read 8 wide
    void* const* out;          // [G] binary32 output tensor of segment g (lower-precision
                               // transport, Section 6.2.3), or null: averages go to the gradients
    int32_t G;
    int32_t R;
};

struct Scale {       // y = use_mul ? s * mul : s / div
    float div;
    float mul;
    int32_t use_mul;
};

// The division by R that turns the sum into DDP's average (Section 3.2.1).
inline Scale make_scale(int R) {
    Scale sc;
    sc.div = static_cast<float>(R);
    sc.mul = 1.0f / static_cast<float>(R);
    sc.use_mul = (R & (R - 1)) == 0;   // power of two: the reciprocal is exact, same bits as dividing
    return sc;
}

// All segment launches cover the tiles [tile_base, tile_base + ntiles) of the
// global tile numbering (tile0 / tile_seg).  `lds` in K2 and K4: bytes of
// dynamic LDS per block that the kernels do not use; they cap the number of
// blocks resident on a compute unit (0 = no cap).  The copy kernels K1 and K3
// keep one or two loads per thread in flight and want every block they can get.

// Timing: the next kernel launched on this thread through one of the pack / reduce / unpack /
// accumulate wrappers below carries `start` and `stop`; the runtime stamps them with the
// kernel's own start and end.  timing_pair_unused() clears the request and tells whether it
// was still pending (the wrapper had nothing to launch).
void time_next_launch(hipEvent_t start, hipEvent_t stop);
bool timing_pair_unused();

// K1: gradients -> flat replica slabs for all `nrep` replicas.  local (may be
// null = every replica used every parameter): participation flags
// [segment][replica]; 0 = write zeros into that replica's slot and do not read
// its tensor.
hipError_t launch_pack(const SegTables& t, int64_t tile_base, int64_t ntiles, char* slab0,
                       int64_t slab_stride, int nrep, const uint8_t* local, hipStream_t s);

// K3: averaged slab -> gradient tensors of replicas [0, nrep).  global_used (may
// be null): per segment, 0 = no replica used the parameter; with keep_unused
// such parameters are not written.
hipError_t launch_unpack(const SegTables& t, int64_t tile_base, int64_t ntiles,
                         const char* out_slab, int nrep, const uint8_t* global_used, bool keep_unused,
                         hipStream_t s);

// K2 (staged): out[v] = scale(sum_r in_r[v]) over nvec 16-byte vectors;
// in_r = in0 + r*stride.
hipError_t launch_flat_reduce(int dtype, const char* in0, int64_t stride, char* out, int64_t nvec,
                              int R, Scale sc, bool nontemporal, unsigned lds, hipStream_t s);

// K2 (fused): gather R replicas through the segment table, reduce, scatter to
// the gradient tensors of replicas [0, nwrite).  local / keep_unused as above
// (a replica with flag 0 contributes +0 and is not read; a parameter nobody
// used is skipped with keep_unused, else written as zeros).  pair = blocks
// take two tiles each (for large launches).
struct GateRecord;   // below, with the flag-ordering kernels

// gate (may be null): the record of the gate kernel enqueued in front of this
// launch; if gate->failed_tag == tag the launch does nothing.
// sig: where (null = nowhere) and with which ordinal the launch's last thread block reports that it
// has started (OrderState::dispatched)
struct DispatchSignal {
    unsigned long long* word;
    unsigned long long ord;
};
hipError_t launch_fused_reduce(int dtype, const SegTables& t, int64_t tile_base, int64_t ntiles,
                               int R, int nwrite, const uint8_t* local, bool keep_unused, Scale sc,
                               bool nontemporal, unsigned lds,
                               const GateRecord* gate, uint32_t tag, DispatchSignal sig, hipStream_t s);
// (with t.out set -- 16-bit gradients, binary32 averages written to t.out -- nwrite must be 1)

// ---- stream ordering through device flags -------------------------------------
// A bucket launch on a reduction stream must come after the backward-stream work
// that produces its gradients (Section 3.2.3).  Instead of an event pair per
// launch, the backward stream announces its position with a one-block kernel
// that stores a sequence number, and the reduction stream runs a one-wave gate
// kernel in front of the bucket kernel that polls for it.  The gate's wait is
// bounded; a gate that gives up marks its launch as failed, the bucket kernel
// that follows sees the mark and does nothing, and the repair launch enqueued by
// the finalizing step (when every gradient exists) redoes exactly those launches.
struct OrderState {
    unsigned long long ready_seq;   // latest announced sequence number (monotonic)
    unsigned long long pad0[15];    // the polled word has a cache line of its own
    uint32_t abort_tag;             // == iteration tag: a gate of this iteration has given up,
                                    //    later gates of the iteration give up at once
    uint32_t repaired;              // launches redone by repair launches since the context was created
    uint32_t pad1[30];
    unsigned long long lane_done[16];   // per reduction stream: the latest iteration tag whose launches
                                        //    on that stream have all ended (monotonic)
    unsigned long long dispatched;      // ordinal of the latest gated bucket launch whose last thread block
    unsigned long long pad2[15];        //    has started (monotonic): the launch is draining or done
};
constexpr int kOrderLanes = 16;

struct GateRecord {                 // one per bucket, used by the launch whose first bucket it is
    int32_t tile_base;              // tile range of the launch
    int32_t ntiles;
    uint32_t failed_tag;            // == iteration tag: the gate gave up, the launch did nothing
    int32_t dtype;
};

// backward stream: ready_seq = seq.  (Everything enqueued before it on that stream has
// ended, and is visible device-wide, by the time the kernel that stores the number runs.)
hipError_t launch_announce(OrderState* st, unsigned long long seq, hipStream_t s);

// The way back at the end of an iteration.  Reduction stream `lane`, behind its last bucket
// launch: lane_done[lane] = tag.  Backward stream: wait (at most wait_ticks) until lane_done[l]
// >= tag for every l in lane_mask.  The join only spares the backward stream a wait for an
// event that has not fired yet (slow on this system when the wait was enqueued long before):
// the events of the same streams are recorded before the done kernels and waited for after
// the join kernel, so a join that gives up changes nothing but the time.
// backward stream, in front of a bucket launch that needs no gate there: the scheduling wait alone
hipError_t launch_chain_wait(OrderState* st, unsigned long long chain_ord, long long chain_ticks, hipStream_t s);
hipError_t launch_done(OrderState* st, int lane, unsigned long long tag, hipStream_t s);
hipError_t launch_join(OrderState* st, uint32_t lane_mask, unsigned long long tag, long long wait_ticks,
                       hipStream_t s);

// reduction stream: wait (at most wait_ticks of the device wall clock) until
// ready_seq >= need; on failure fill *rec, tag *row_summary (the record behind the last bucket's
// in the iteration's row: "a gate of this row gave up") and raise abort_tag.
// chain_ord / chain_ticks: once the number is there, the gate also waits (at most chain_ticks; 0 =
// not at all) until the bucket launch with ordinal chain_ord on ANOTHER reduction stream has
// started its last thread block, so that this launch fills the compute units as that one drains
// instead of sharing the memory system with it from its start.  A pure scheduling hint: the
// gate goes on when the bound is reached.
hipError_t launch_gate(OrderState* st, unsigned long long need, long long wait_ticks, GateRecord* rec,
                       GateRecord* row_summary, int32_t tile_base, int32_t ntiles, int32_t dtype, uint32_t tag,
                       unsigned long long chain_ord, long long chain_ticks, hipStream_t s);

// Redo the launches of element type `dtype` whose gate gave up in iteration `tag`
// (rec[0..nb)).  `blocks` persistent blocks; normally there is nothing to do.
hipError_t launch_repair(int dtype, const SegTables& t, OrderState* st, const GateRecord* rec, int nb, uint32_t tag,
                         int R, int nwrite, const uint8_t* local, bool keep_unused, Scale sc,
                         int blocks, bool nontemporal, hipStream_t s);

// Bounded probe: one wave on stream `waiter` polls word[0] for `value` (at most
// wait_ticks), then a one-thread kernel on stream `writer` stores it.
// word[1] = 1 if the waiter saw the value, i.e. if the two streams make progress
// independently (streams that share a hardware queue run one after the other).
hipError_t launch_probe(unsigned long long* word, unsigned long long value, long long wait_ticks,
                        hipStream_t waiter, hipStream_t writer);

// global[g] = OR_r local[g*R + r]  (the bitmap AllReduce of Section 4.2).
hipError_t launch_bitmap_or(const uint8_t* local, uint8_t* global, int G, int R, hipStream_t s);

// K4: grad[r][g] += micro[r*n + param[g]] for all segments and replicas
// (null micro pointers are skipped).  ntiles = tile0[G].
hipError_t launch_accumulate(const SegTables& t, int64_t ntiles, int R, int n, void* const* micro,
                             unsigned lds, hipStream_t s);

// K6: a kernel that waits `ticks` of the device wall clock (bounded; skipped for
// ticks <= 0), followed by a kernel that copies src_r -> dst_r (nelem elements
// of es bytes) for r < R, where ptrs = [dst_0..dst_{R-1}, src_0..src_{R-1}] is a
// device array (null = delay only).  busy_blocks = 0: the delay is one block that
// sleeps between polls; > 0: that many blocks doing arithmetic between polls.
hipError_t launch_emit(int64_t ticks, void* const* ptrs, int R, int64_t nelem, int es,
                       int busy_blocks, float* sink, hipStream_t s);

}  // namespace ddp
