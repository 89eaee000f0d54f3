#include "bucket_plan.h"

namespace ddp {

bool BucketPlan::assign(uint64_t cap_bytes, const std::vector<int32_t>* order) {
    const int n = (int)params.size();
    if (order) {
        if ((int)order->size() != n) return false;
        std::vector<uint8_t> seen(n, 0);
        for (int32_t i : *order) {
            if (i < 0 || i >= n || seen[i]) return false;
            seen[i] = 1;
        }
    }
    buckets.clear();
    bool open = false;
    for (int k = 0; k < n; ++k) {
        const int i = order ? (*order)[k] : n - 1 - k;
        ParamInfo& p = params[i];
        const uint64_t size = (uint64_t)p.numel * (uint64_t)elem_size(p.dtype);
        if (open) {
            const BucketInfo& cur = buckets.back();
            // cur.bytes() + size > cap, written so that it cannot wrap around
            const bool over = cur.bytes() > cap_bytes || size > cap_bytes - cur.bytes();
            if (over || cur.dtype != p.dtype) open = false;
        }
        if (!open) {
            buckets.emplace_back();
            buckets.back().dtype = p.dtype;
            open = true;
        }
        BucketInfo& cur = buckets.back();
        p.bucket = (int32_t)buckets.size() - 1;
        p.offset = cur.elems;
        cur.params.push_back(i);
        cur.elems += p.numel;
    }
    int32_t seg = 0;
    for (BucketInfo& b : buckets) {
        b.seg_begin = seg;
        for (int32_t i : b.params) params[i].segment = seg++;
    }
    return true;
}

void ReadyTracker::reset(const BucketPlan& plan) {
    plan_ = &plan;
    marked_.assign(plan.params.size(), 0);
    pending_.resize(plan.buckets.size());
    new_iteration();
}

void ReadyTracker::new_iteration() {
    for (size_t b = 0; b < pending_.size(); ++b)
        pending_[b] = (int32_t)plan_->buckets[b].params.size();
    std::fill(marked_.begin(), marked_.end(), 0);
    next_ = 0;
    marks_ = 0;
}

int ReadyTracker::mark(int32_t param, std::vector<int32_t>& launch) {
    if (param < 0 || param >= (int32_t)marked_.size()) return -1;
    if (marked_[param]) return -2;
    marked_[param] = 1;
    ++marks_;
    --pending_[plan_->params[param].bucket];
    while (next_ < (int32_t)pending_.size() && pending_[next_] == 0) launch.push_back(next_++);
    return 0;
}

void ReadyTracker::drain(std::vector<int32_t>& launch) {
    while (next_ < (int32_t)pending_.size()) launch.push_back(next_++);
}

}  // namespace ddp
