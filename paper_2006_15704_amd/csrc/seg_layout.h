// Host-side construction of the device tables that the kernels walk: the slab
// layout of the flat buckets (Algorithm 1's bucket views) and the segment
// tables (parameters in bucket-major fill order).  Shared by the context path
// and the allocation-free entry point; no HIP calls here.
#pragma once
#include <cstdint>
#include <vector>

#include "bucket_plan.h"
#include "ddp_kernels.h"

namespace ddp {

struct HostTables {
    std::vector<int64_t> bucket_slab_off;   // byte offset of every bucket inside a slab (256-byte aligned)
    std::vector<int64_t> bucket_vecs;       // 16-byte vectors per bucket (length padded to 16 bytes)
    int64_t slab_stride = 0;                // bytes of one replica's slab (all buckets), multiple of 4096
    std::vector<int64_t> tile0;             // [G + 1] first tile of every segment
    std::vector<SegInfo> seg;               // [G]
    std::vector<void*> grad;                // [G * R + 8], see SegTables::grad
    std::vector<int32_t> tile_seg;          // [tile0[G]]
    std::vector<void*> out;                 // [G] binary32 output tensors (empty without outputs)
};

inline int64_t round_up_to(int64_t x, int64_t a) { return (x + a - 1) / a * a; }

// grad_ptrs: [R][n] in registration order (the layout of ddp_register_params).
// out_ptrs: [n] binary32 output tensors in registration order, or null.
inline void build_host_tables(const BucketPlan& plan, void* const* grad_ptrs, int R, HostTables& h,
                              void* const* out_ptrs = nullptr) {
    const int32_t n = static_cast<int32_t>(plan.params.size());
    const int32_t nb = static_cast<int32_t>(plan.buckets.size());
    h.bucket_slab_off.resize(nb);
    h.bucket_vecs.resize(nb);
    int64_t off = 0;
    for (int32_t b = 0; b < nb; ++b) {
        h.bucket_slab_off[b] = off;
        const int64_t bytes = static_cast<int64_t>(plan.buckets[b].bytes());
        h.bucket_vecs[b] = (bytes + 15) / 16;
        off = round_up_to(off + h.bucket_vecs[b] * 16, 256);
    }
    h.slab_stride = round_up_to(off > 0 ? off : 256, 4096);

    h.tile0.assign(n + 1, 0);
    h.seg.assign(n, SegInfo{});
    h.grad.assign(static_cast<size_t>(R) * n + 8, nullptr);
    h.out.assign(out_ptrs ? n : 0, nullptr);
    for (int32_t b = 0; b < nb; ++b) {
        const BucketInfo& bk = plan.buckets[b];
        for (size_t k = 0; k < bk.params.size(); ++k) {
            const int32_t i = bk.params[k];
            const int32_t g = bk.seg_begin + static_cast<int32_t>(k);
            const ParamInfo& p = plan.params[i];
            const int es = elem_size(p.dtype);
            const int64_t flat_byte = h.bucket_slab_off[b] + p.offset * es;
            // largest lead-in over every destination this segment can have: its slot in the
            // flat slab and each replica's gradient tensor
            int lead = static_cast<int>(flat_byte & 15);
            const uintptr_t a0 = reinterpret_cast<uintptr_t>(grad_ptrs[i]);
            bool cong = true;
            for (int64_t r = 0; r < R; ++r) {
                void* ptr = grad_ptrs[r * n + i];
                const uintptr_t a = reinterpret_cast<uintptr_t>(ptr);
                h.grad[static_cast<size_t>(g) * R + r] = ptr;
                if (static_cast<int>(a & 15u) > lead) lead = static_cast<int>(a & 15u);
                cong = cong && ((a ^ a0) & 15u) == 0;
            }
            h.tile0[g + 1] = h.tile0[g] + tiles_for(p.numel, es, lead);
            h.seg[g].numel = p.numel;
            h.seg[g].tile0 = h.tile0[g];
            h.seg[g].flat_byte = flat_byte;
            h.seg[g].param = i;
            h.seg[g].flags = p.dtype | (cong ? 0x100 : 0) | (static_cast<int>(a0 & 15u) << 16);
            if (out_ptrs) {
                h.out[g] = out_ptrs[i];
                const uintptr_t o = reinterpret_cast<uintptr_t>(out_ptrs[i]);
                if ((o & 15u) == ((2 * (a0 & 15u)) & 15u)) h.seg[g].flags |= 0x200;
            }
        }
    }
    h.tile_seg.resize(static_cast<size_t>(h.tile0[n]));
    for (int32_t g = 0; g < n; ++g)
        for (int64_t tl = h.tile0[g]; tl < h.tile0[g + 1]; ++tl) h.tile_seg[tl] = g;
}

}  // namespace ddp
