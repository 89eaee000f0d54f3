// The allocation-free entry point: one whole synchronization (staged
// pipeline: pack, reduce and average, write back) whose device tables and
// flat bucket buffers live in a file-scope device array instead of memory
// obtained from hipMalloc.  For callers that cannot allocate: code under HIP
// graph capture, tight serving loops, harnesses that forbid allocation.
#include "../../include/ddp_gfx950.h"

#include <hip/hip_runtime.h>

#include <cstring>
#include <mutex>
#include <string>
#include <vector>

#include "bucket_plan.h"
#include "ddp_kernels.h"
#include "seg_layout.h"

namespace ddp {
int32_t fail_without_context(int32_t code, const std::string& msg);   // ddp_api.hip
}

namespace {

// Every GPU the library runs on holds its own copy of this array, at its own
// address, until the process ends.  In host code the name below is only a
// handle for hipGetSymbolAddress; the device address is looked up once per
// device (scratch_on) and that pointer is what kernels and fills receive.
static __device__ __align__(256) unsigned char scratch[DDP_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
std::mutex g_mu;
unsigned char* g_scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on the current device (which must be `device`).
hipError_t scratch_on(int device, unsigned char** out) {
    std::lock_guard<std::mutex> lock(g_mu);
    if (g_scratch_ptr[device] == nullptr) {
        void* p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (p == nullptr) return hipErrorInvalidSymbol;
        g_scratch_ptr[device] = static_cast<unsigned char*>(p);
    }
    *out = g_scratch_ptr[device];
    return hipSuccess;
}

// Host data reaches the device inside kernel arguments: no copy engine, no
// staging buffer, nothing that reads host memory after the call has returned
// (so the call can also be captured into a graph).
constexpr int kPayloadWords = 768;              // 3 KiB per launch
struct Payload { uint32_t w[kPayloadWords]; };

__global__ __launch_bounds__(256) void table_write_kernel(uint32_t* __restrict__ dst, Payload p, int nwords) {
    for (int i = threadIdx.x; i < nwords; i += 256) dst[i] = p.w[i];
}

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
__global__ __launch_bounds__(256) void clear_kernel(u32x4* __restrict__ dst, int64_t nvec) {
    const u32x4 z = {0u, 0u, 0u, 0u};
    const int64_t stride = static_cast<int64_t>(gridDim.x) * 256;
    for (int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x; i < nvec; i += stride) dst[i] = z;
}

hipError_t upload(unsigned char* dst, const void* src, size_t bytes, hipStream_t s) {
    // dst and bytes are multiples of 4 by construction of the layout
    const uint32_t* w = static_cast<const uint32_t*>(src);
    size_t words = bytes / 4;
    uint32_t* d = reinterpret_cast<uint32_t*>(dst);
    while (words > 0) {
        Payload p;
        const int nw = static_cast<int>(words < static_cast<size_t>(kPayloadWords) ? words : kPayloadWords);
        std::memcpy(p.w, w, static_cast<size_t>(nw) * 4);
        hipLaunchKernelGGL(table_write_kernel, dim3(1), dim3(256), 0, s, d, p, nw);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        w += nw; d += nw; words -= static_cast<size_t>(nw);
    }
    return hipSuccess;
}

#define HIPCHK0(expr)                                                                        \
    do {                                                                                     \
        hipError_t e_ = (expr);                                                              \
        if (e_ != hipSuccess)                                                                \
            return ddp::fail_without_context(DDP_ERR_HIP, std::string("ddp_sync_static: ") + #expr + ": " + hipGetErrorString(e_)); \
    } while (0)

}  // namespace

extern "C" int32_t ddp_sync_static(int32_t R, int32_t device, void* stream, int32_t n,
                                   const int64_t* numel, const int32_t* dtype,
                                   void* const* grad_ptrs, uint64_t cap_bytes) {
    using ddp::fail_without_context;
    if (R < 1) return fail_without_context(DDP_ERR_ARG, "ddp_sync_static: R must be at least 1");
    if (R > DDP_MAX_REPLICAS) return fail_without_context(DDP_ERR_UNSUPPORTED, "ddp_sync_static: R above DDP_MAX_REPLICAS");
    if (device < 0 || device >= kMaxDevices) return fail_without_context(DDP_ERR_ARG, "ddp_sync_static: bad device");
    if (n <= 0 || !numel || !dtype || !grad_ptrs)
        return fail_without_context(DDP_ERR_ARG, "ddp_sync_static: n <= 0 or null array");
    ddp::BucketPlan plan;
    plan.params.resize(n);
    for (int32_t i = 0; i < n; ++i) {
        if (numel[i] < 0) return fail_without_context(DDP_ERR_ARG, "ddp_sync_static: negative numel");
        if (dtype[i] != DDP_FP32 && dtype[i] != DDP_FP16 && dtype[i] != DDP_BF16)
            return fail_without_context(DDP_ERR_ARG, "ddp_sync_static: unknown dtype");
        plan.params[i].numel = numel[i];
        plan.params[i].dtype = dtype[i];
    }
    // Sizes first (before any pointer is looked at): a model that cannot fit is refused.
    {
        uint64_t total = 0;
        for (int32_t i = 0; i < n; ++i) {
            const uint64_t b = static_cast<uint64_t>(numel[i]) * static_cast<uint64_t>(ddp::elem_size(dtype[i]));
            if (static_cast<uint64_t>(numel[i]) > (uint64_t(1) << 40) || total + b > (uint64_t(1) << 40)) {
                total = uint64_t(1) << 40;
                break;
            }
            total += b;
        }
        if (total * static_cast<uint64_t>(R + 1) > DDP_STATIC_SCRATCH_BYTES)
            return fail_without_context(DDP_ERR_UNSUPPORTED,
                        "ddp_sync_static: (R + 1) x gradient bytes exceed the static scratch buffer of " +
                        std::to_string(DDP_STATIC_SCRATCH_BYTES) + " bytes");
    }
    for (int64_t r = 0; r < R; ++r)
        for (int32_t i = 0; i < n; ++i) {
            const void* p = grad_ptrs[r * n + i];
            if (numel[i] > 0 && !p) return fail_without_context(DDP_ERR_ARG, "ddp_sync_static: null gradient pointer");
            if (reinterpret_cast<uintptr_t>(p) % static_cast<uintptr_t>(ddp::elem_size(dtype[i])) != 0)
                return fail_without_context(DDP_ERR_ARG, "ddp_sync_static: gradient pointer not aligned to its element size");
        }
    plan.assign(cap_bytes, nullptr);
    ddp::HostTables ht;
    ddp::build_host_tables(plan, grad_ptrs, R, ht);
    const int32_t nb = static_cast<int32_t>(plan.buckets.size());

    // layout of the scratch array: [segment records | pointer rows | tile map | pad to 256 | R + 1 slabs]
    const size_t seg_bytes = sizeof(ddp::SegInfo) * static_cast<size_t>(n);
    const size_t ptr_bytes = sizeof(void*) * ht.grad.size();
    const size_t map_bytes = sizeof(int32_t) * ht.tile_seg.size();
    const size_t table_bytes = static_cast<size_t>(ddp::round_up_to(static_cast<int64_t>(seg_bytes + ptr_bytes + map_bytes), 256));
    const size_t slab_bytes = static_cast<size_t>(ht.slab_stride) * static_cast<size_t>(R + 1);
    if (table_bytes + slab_bytes > DDP_STATIC_SCRATCH_BYTES)
        return fail_without_context(DDP_ERR_UNSUPPORTED,
                    "ddp_sync_static: tables and flat buckets need " + std::to_string(table_bytes + slab_bytes) +
                    " bytes, the static scratch buffer holds " + std::to_string(DDP_STATIC_SCRATCH_BYTES));

    hipStream_t s = static_cast<hipStream_t>(stream);
    HIPCHK0(hipSetDevice(device));
    unsigned char* base = nullptr;
    HIPCHK0(scratch_on(device, &base));

    std::vector<unsigned char> host(seg_bytes + ptr_bytes + map_bytes);
    std::memcpy(host.data(), ht.seg.data(), seg_bytes);
    std::memcpy(host.data() + seg_bytes, ht.grad.data(), ptr_bytes);
    if (map_bytes) std::memcpy(host.data() + seg_bytes + ptr_bytes, ht.tile_seg.data(), map_bytes);
    HIPCHK0(upload(base, host.data(), host.size(), s));

    ddp::SegTables t{};
    t.seg = reinterpret_cast<const ddp::SegInfo*>(base);
    t.grad = reinterpret_cast<void* const*>(base + seg_bytes);
    t.tile_seg = reinterpret_cast<const int32_t*>(base + seg_bytes + ptr_bytes);
    t.G = n;
    t.R = R;
    char* slabs = reinterpret_cast<char*>(base + table_bytes);

    // The array keeps what the previous call left in it.  The flat buckets are
    // rewritten by the pack kernel except for the padding between them, which the
    // reduce kernel reads (whole 16-byte vectors): clear the slabs.
    {
        const int64_t nvec = static_cast<int64_t>(slab_bytes / 16);
        int64_t blocks = (nvec + 255) / 256;
        if (blocks > 2048) blocks = 2048;
        if (blocks > 0) {
            hipLaunchKernelGGL(clear_kernel, dim3(static_cast<unsigned>(blocks)), dim3(256), 0, s,
                               reinterpret_cast<u32x4*>(slabs), nvec);
            HIPCHK0(hipGetLastError());
        }
    }
    const int64_t ntiles = ht.tile0[n];
    HIPCHK0(ddp::launch_pack(t, 0, ntiles, slabs, ht.slab_stride, R, nullptr, s));
    const ddp::Scale sc = ddp::make_scale(R);
    char* out = slabs + static_cast<int64_t>(R) * ht.slab_stride;
    for (int32_t b = 0; b < nb; ++b)      // in bucket order (Section 3.2.3)
        HIPCHK0(ddp::launch_flat_reduce(plan.buckets[b].dtype, slabs + ht.bucket_slab_off[b], ht.slab_stride,
                                        out + ht.bucket_slab_off[b], ht.bucket_vecs[b], R, sc, true, 0, s));
    HIPCHK0(ddp::launch_unpack(t, 0, ntiles, out, 1, nullptr, false, s));
    return nb;
}
