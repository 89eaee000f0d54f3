// Host-side bucket plan and ready/launch state machine.  No GPU types here.
//
// Paper: Algorithm 1 (constructor: parameters are allocated to buckets in the
// reverse order of net.parameters() under a size cap; autograd_hook: a bucket
// whose gradients are all ready is marked ready and ready buckets are launched
// in order), Section 4.2 (per-bucket pending counts, replenished every
// iteration) and Section 3.2.3 (bucket i+1 never before bucket i; absent
// gradients must not stall a bucket).
#pragma once
#include <algorithm>
#include <cstdint>
#include <vector>

namespace ddp {

inline int elem_size(int dtype) { return dtype == 0 ? 4 : 2; }

struct ParamInfo {
    int64_t numel = 0;
    int32_t dtype = 0;
    int32_t bucket = -1;
    int64_t offset = 0;     // elements from the start of the bucket
    int32_t segment = -1;   // index into the bucket-ordered segment list
};

struct BucketInfo {
    std::vector<int32_t> params;   // fill order (default: descending registration index)
    int64_t elems = 0;
    int32_t dtype = 0;
    int32_t seg_begin = 0;         // first global segment index
    uint64_t bytes() const { return (uint64_t)elems * (uint64_t)elem_size(dtype); }
};

struct BucketPlan {
    std::vector<ParamInfo> params;
    std::vector<BucketInfo> buckets;
    // Fills bucket / offset / segment of every parameter and the bucket list.
    // Parameters are visited in `order` (a permutation of the indices; Section
    // 6.2.1: a traced backward order) or, without one, in reverse registration
    // order (Algorithm 1).  Returns false if `order` is not a permutation.
    bool assign(uint64_t cap_bytes, const std::vector<int32_t>* order = nullptr);
};

// Pending counts and in-order launch.  launch decisions are returned to the
// caller, which owns the actual kernel launches.
class ReadyTracker {
public:
    void reset(const BucketPlan& plan);
    // 0 ok, -1 id out of range, -2 already marked.  Appends to `launch` the
    // buckets that become launchable, in order.
    int mark(int32_t param, std::vector<int32_t>& launch);
    // Buckets still to be launched, in order; marks them launched.
    void drain(std::vector<int32_t>& launch);
    bool marked(int32_t param) const { return marked_[param] != 0; }
    int32_t marks() const { return marks_; }
    int32_t unmarked_in(int32_t bucket) const { return pending_[bucket]; }
    void new_iteration();
private:
    const BucketPlan* plan_ = nullptr;
    std::vector<int32_t> pending_;
    std::vector<uint8_t> marked_;
    int32_t next_ = 0;
    int32_t marks_ = 0;
};

}  // namespace ddp
