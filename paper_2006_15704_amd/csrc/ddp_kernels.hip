// HIP kernels of the bucketed gradient synchronization path, written for
// gfx950 (MI355X): 64-wide wavefronts, 16-byte vector loads, fp32
// accumulation in registers.  The path is a streaming reduction (about one
// add per four bytes read), so every kernel here is bound by HBM bandwidth
// and none uses the matrix cores.
//
// Paper anchors: pack = the copy of a gradient into its bucket view
// (Algorithm 1, autograd_hook); reduce = the bucket AllReduce (Section 2.3:
// sum over participants) followed by DDP's averaging (Section 3.2.1); unpack
// = the finalizing write-back described after Algorithm 1; accumulate = the
// local gradient accumulation of no_sync (Section 3.2.4).
#include "ddp_kernels.h"

#include <hip/hip_ext.h>

#include <mutex>
#include <set>
#include <utility>

namespace ddp {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Every gradient, slab and table lives in global memory.  Pointers that are
// read from tables carry no address space, and the compiler would fall back to
// generic (flat) accesses for them; the casts below keep all traffic on the
// global path.
#define DDP_GLOBAL __attribute__((address_space(1)))
typedef DDP_GLOBAL const u32x4* gc_u32x4;
typedef DDP_GLOBAL u32x4* g_u32x4;

template <typename T>
__device__ __forceinline__ T gload(const char* p) {
    return *(DDP_GLOBAL const T*)(p);
}
template <typename T>
__device__ __forceinline__ void gstore(char* p, T v) {
    *(DDP_GLOBAL T*)(p) = v;
}

template <bool NT>
__device__ __forceinline__ u32x4 load16(const char* p) {
    gc_u32x4 q = (gc_u32x4)(p);
    if (NT) return __builtin_nontemporal_load(q);
    return *q;
}
__device__ __forceinline__ void store16(char* p, u32x4 v) {
    *(g_u32x4)(p) = v;
}
// Results that are not read again soon are stored with the non-temporal hint.
template <bool NT>
__device__ __forceinline__ void store16s(char* p, u32x4 v) {
    if (NT) __builtin_nontemporal_store(v, (g_u32x4)(p));
    else *(g_u32x4)(p) = v;
}
__device__ __forceinline__ u32x4 zero16() {
    u32x4 z = {0u, 0u, 0u, 0u};
    return z;
}
// 16 bytes at an address that is only element-aligned (2 or 4 bytes): gfx950
// serves such an access with one vector instruction too, so a tensor that sits
// off the 16-byte grid of its peers costs extra cache lines, not a scalar loop.
typedef u32x4 u32x4_a2 __attribute__((aligned(2)));
template <bool NT>
__device__ __forceinline__ u32x4 load16u(const char* p) {
    DDP_GLOBAL const u32x4_a2* q = (DDP_GLOBAL const u32x4_a2*)(p);
    if (NT) return __builtin_nontemporal_load(q);
    return *q;
}
template <bool NT>
__device__ __forceinline__ void store16u(char* p, u32x4 v) {
    DDP_GLOBAL u32x4_a2* q = (DDP_GLOBAL u32x4_a2*)(p);
    if (NT) __builtin_nontemporal_store(v, q);
    else *q = v;
}

// ---- element formats ------------------------------------------------------
template <int DT> struct Fmt;

template <> struct Fmt<0> {   // binary32
    static constexpr int ES = 4, VEC = 4;
    static __device__ __forceinline__ void widen(u32x4 v, float (&f)[4]) {
#pragma unroll
        for (int i = 0; i < 4; ++i) f[i] = __uint_as_float(v[i]);
    }
    static __device__ __forceinline__ u32x4 narrow(const float (&f)[4]) {
        u32x4 v;
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] = __float_as_uint(f[i]);
        return v;
    }
    static __device__ __forceinline__ float load1(const char* p) {
        return gload<float>(p);
    }
    static __device__ __forceinline__ void store1(char* p, float y) {
        gstore<float>(p, y);
    }
};

template <> struct Fmt<1> {   // binary16: exact widening, round-to-nearest-even narrowing
    static constexpr int ES = 2, VEC = 8;
    static __device__ __forceinline__ float up(uint32_t bits16) {
        return static_cast<float>(__builtin_bit_cast(_Float16, static_cast<uint16_t>(bits16)));
    }
    static __device__ __forceinline__ uint32_t down(float y) {
        return __builtin_bit_cast(uint16_t, static_cast<_Float16>(y));
    }
    static __device__ __forceinline__ void widen(u32x4 v, float (&f)[8]) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            f[2 * i] = up(v[i] & 0xFFFFu);
            f[2 * i + 1] = up(v[i] >> 16);
        }
    }
    static __device__ __forceinline__ u32x4 narrow(const float (&f)[8]) {
        u32x4 v;
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] = down(f[2 * i]) | (down(f[2 * i + 1]) << 16);
        return v;
    }
    static __device__ __forceinline__ float load1(const char* p) {
        return up(gload<uint16_t>(p));
    }
    static __device__ __forceinline__ void store1(char* p, float y) {
        gstore<uint16_t>(p, static_cast<uint16_t>(down(y)));
    }
};

template <> struct Fmt<2> {   // bfloat16 = upper half of binary32
    static constexpr int ES = 2, VEC = 8;
    static __device__ __forceinline__ uint32_t down(float y) {
        uint32_t u = __float_as_uint(y);
        if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (u >> 16) | 0x0040u;   // NaN stays NaN
        u += 0x7FFFu + ((u >> 16) & 1u);                                     // nearest, ties to even
        return u >> 16;
    }
    static __device__ __forceinline__ void widen(u32x4 v, float (&f)[8]) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            f[2 * i] = __uint_as_float(v[i] << 16);
            f[2 * i + 1] = __uint_as_float(v[i] & 0xFFFF0000u);
        }
    }
    static __device__ __forceinline__ u32x4 narrow(const float (&f)[8]) {
        u32x4 v;
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] = down(f[2 * i]) | (down(f[2 * i + 1]) << 16);
        return v;
    }
    static __device__ __forceinline__ float load1(const char* p) {
        return __uint_as_float(static_cast<uint32_t>(gload<uint16_t>(p)) << 16);
    }
    static __device__ __forceinline__ void store1(char* p, float y) {
        gstore<uint16_t>(p, static_cast<uint16_t>(down(y)));
    }
};

__device__ __forceinline__ float apply_scale(const Scale& sc, float s) {
    return sc.use_mul ? s * sc.mul : s / sc.div;
}

// Vectors are cut at 16-byte boundaries of the destination.  `sh` elements
// precede the segment start inside the first vector, so element index
// e = tile_elem - sh may be negative for the first vector of a segment.
__device__ __forceinline__ int lead_in(const void* dst, int es) {
    return static_cast<int>(reinterpret_cast<uintptr_t>(dst) & 15u) / es;
}
__device__ __forceinline__ bool congruent16(const void* a, const void* b) {
    return ((reinterpret_cast<uintptr_t>(a) ^ reinterpret_cast<uintptr_t>(b)) & 15u) == 0;
}

enum { V_NONE = 0, V_FULL = 1, V_EDGE = 2 };
__device__ __forceinline__ int classify(int64_t e, int vec, int64_t numel) {
    if (e >= numel) return V_NONE;
    return (e >= 0 && e + vec <= numel) ? V_FULL : V_EDGE;
}

// ---- K1 / K3: segment copies ---------------------------------------------
template <int ES>
__device__ __forceinline__ void copy_tile(const char* __restrict__ src, char* __restrict__ dst,
                                          int64_t numel, int64_t ltile, bool zero) {
    constexpr int VEC = 16 / ES;
    constexpr int U = TILE_VECS / BLOCK;
    const int sh = lead_in(dst, ES);
    const bool cong = congruent16(src, dst);
    const int64_t e_tile = ltile * (TILE_BYTES / ES) - sh;
    int64_t e[U];
    int kind[U];
    u32x4 v[U];
#pragma unroll
    for (int k = 0; k < U; ++k) {
        e[k] = e_tile + static_cast<int64_t>(k * BLOCK + threadIdx.x) * VEC;
        kind[k] = classify(e[k], VEC, numel);
        v[k] = zero16();
        if (kind[k] == V_FULL && !zero)
            v[k] = cong ? load16<true>(src + e[k] * ES) : load16u<true>(src + e[k] * ES);
    }
#pragma unroll
    for (int k = 0; k < U; ++k) {
        if (kind[k] == V_FULL) {
            store16(dst + e[k] * ES, v[k]);
        } else if (kind[k] == V_EDGE) {
            for (int i = 0; i < VEC; ++i) {
                const int64_t idx = e[k] + i;
                if (idx < 0 || idx >= numel) continue;
                if (ES == 4) {
                    gstore<uint32_t>(dst + idx * 4, zero ? 0u : gload<uint32_t>(src + idx * 4));
                } else {
                    gstore<uint16_t>(dst + idx * 2, zero ? uint16_t(0) : gload<uint16_t>(src + idx * 2));
                }
            }
        }
    }
}

// PACK: grad[r][g] -> slab_r + flat_byte[g];  UNPACK: out slab -> grad[r][g].
template <bool PACK>
__global__ __launch_bounds__(BLOCK) void seg_copy_kernel(SegTables t, int64_t tile_base,
                                                         char* slab0, int64_t slab_stride,
                                                         const uint8_t* __restrict__ flags,
                                                         int keep_unused) {
    const int64_t tile = tile_base + blockIdx.x;
    const int r = blockIdx.y;
    const int g = t.tile_seg[tile];
    const SegInfo si = t.seg[g];
    const int64_t numel = si.numel;
    const int64_t ltile = tile - si.tile0;
    char* grad = static_cast<char*>(t.grad[static_cast<int64_t>(g) * t.R + r]);
    // PACK: flags = per (segment, replica) participation, 0 = the replica did
    // not use the parameter: its slot gets zeros and its tensor is not read.
    // UNPACK: flags = global bitmap per segment, 0 = no replica used the
    // parameter: with keep_unused its gradients are left as they are.
    const bool zero = PACK && flags != nullptr && flags[static_cast<int64_t>(g) * t.R + r] == 0;
    if (!PACK && keep_unused && flags != nullptr && flags[g] == 0) return;
    const char* src;
    char* dst;
    if (PACK) {
        src = grad;
        dst = slab0 + r * slab_stride + si.flat_byte;
    } else {
        src = slab0 + si.flat_byte;
        dst = grad;
    }
    if (si.dtype() == 0) copy_tile<4>(src, dst, numel, ltile, zero);
    else copy_tile<2>(src, dst, numel, ltile, zero);
}

// ---- K2: reduce and average ------------------------------------------------
// acc += widen(x), elementwise, in the order the calls are made.
template <int DT>
__device__ __forceinline__ void add_into(float (&acc)[Fmt<DT>::VEC], u32x4 x) {
    float f[Fmt<DT>::VEC];
    Fmt<DT>::widen(x, f);
#pragma unroll
    for (int i = 0; i < Fmt<DT>::VEC; ++i) acc[i] += f[i];
}

// Interior work (every vector of the block lies inside the data): no lane is
// predicated.  base_of(r) returns replica r's block-uniform base address; the
// per-thread part of the address is a 32-bit byte offset, so the loads take the
// scalar-base + vector-offset form.  All C*U loads are issued before the adds,
// which run in ascending r.
template <int DT, bool NT, int C, int U, typename BaseFn>
__device__ __forceinline__ void chunk_interior(BaseFn base_of, int r, const uint32_t (&lane_off)[U],
                                               float (&acc)[U][Fmt<DT>::VEC]) {
    const char* base[C];
#pragma unroll
    for (int i = 0; i < C; ++i) base[i] = base_of(r + i);
    u32x4 x[C][U];
#pragma unroll
    for (int i = 0; i < C; ++i)
#pragma unroll
        for (int u = 0; u < U; ++u) x[i][u] = load16<NT>(base[i] + lane_off[u]);
#pragma unroll
    for (int i = 0; i < C; ++i)
#pragma unroll
        for (int u = 0; u < U; ++u) add_into<DT>(acc[u], x[i][u]);
}

// The last `left` (0..7) replicas as ONE chunk, so that all of their loads are
// in flight together (a 4 + 2 + 1 split would run three dependent phases).
template <int DT, bool NT, int U, typename BaseFn>
__device__ __forceinline__ void tail_interior(BaseFn base_of, int r, int left,
                                              const uint32_t (&lane_off)[U],
                                              float (&acc)[U][Fmt<DT>::VEC]) {
    switch (left) {
        case 7: chunk_interior<DT, NT, 7, U>(base_of, r, lane_off, acc); break;
        case 6: chunk_interior<DT, NT, 6, U>(base_of, r, lane_off, acc); break;
        case 5: chunk_interior<DT, NT, 5, U>(base_of, r, lane_off, acc); break;
        case 4: chunk_interior<DT, NT, 4, U>(base_of, r, lane_off, acc); break;
        case 3: chunk_interior<DT, NT, 3, U>(base_of, r, lane_off, acc); break;
        case 2: chunk_interior<DT, NT, 2, U>(base_of, r, lane_off, acc); break;
        case 1: chunk_interior<DT, NT, 1, U>(base_of, r, lane_off, acc); break;
        default: break;
    }
}

template <int DT, bool NT, int U, typename BaseFn>
__device__ __forceinline__ void sum_interior(BaseFn base_of, int R, const uint32_t (&lane_off)[U],
                                             float (&acc)[U][Fmt<DT>::VEC]) {
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
        for (int i = 0; i < Fmt<DT>::VEC; ++i) acc[u][i] = -0.0f;   // -0 + x == x for every x
    int r = 0;
    for (; r + 8 <= R; r += 8) chunk_interior<DT, NT, 8, U>(base_of, r, lane_off, acc);
    tail_interior<DT, NT, U>(base_of, r, R - r, lane_off, acc);
}

// The same with the first eight replica pointers already in registers (they are
// fetched together with the segment record, one dependent memory access
// earlier than a fetch inside the loop would be).
template <int DT, bool NT, int U, typename BaseFn>
__device__ __forceinline__ void sum_interior_pre(const char* const (&pre)[8], int64_t byte0,
                                                 BaseFn base_of, int R,
                                                 const uint32_t (&lane_off)[U],
                                                 float (&acc)[U][Fmt<DT>::VEC]) {
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
        for (int i = 0; i < Fmt<DT>::VEC; ++i) acc[u][i] = -0.0f;
    int r = 0;
    if (R >= 8) {
        chunk_interior<DT, NT, 8, U>([&](int k) { return pre[k] + byte0; }, 0, lane_off, acc);
        r = 8;
    }
    for (; r + 8 <= R; r += 8) chunk_interior<DT, NT, 8, U>(base_of, r, lane_off, acc);
    if (r == 0) {
        // fewer than eight replicas: their pointers are the preloaded ones
        tail_interior<DT, NT, U>([&](int k) { return pre[k] + byte0; }, 0, R, lane_off, acc);
    } else {
        tail_interior<DT, NT, U>(base_of, r, R - r, lane_off, acc);
    }
}

template <int DT>
__device__ __forceinline__ u32x4 scaled(const Scale& sc, const float (&acc)[Fmt<DT>::VEC]) {
    float y[Fmt<DT>::VEC];
#pragma unroll
    for (int i = 0; i < Fmt<DT>::VEC; ++i) y[i] = apply_scale(sc, acc[i]);
    return Fmt<DT>::narrow(y);
}

// C replicas starting at r, U vectors per thread: issue all C*U loads, then
// add them in ascending r.
template <int DT, bool NT, int C, int U>
__device__ __forceinline__ void chunk_flat(const char* __restrict__ in0, int64_t stride, int r,
                                           const int64_t (&off)[U], const bool (&ok)[U],
                                           float (&acc)[U][Fmt<DT>::VEC]) {
    u32x4 x[C][U];
#pragma unroll
    for (int i = 0; i < C; ++i) {
        const char* p = in0 + static_cast<int64_t>(r + i) * stride;
#pragma unroll
        for (int u = 0; u < U; ++u) x[i][u] = ok[u] ? load16<NT>(p + off[u]) : zero16();
    }
#pragma unroll
    for (int i = 0; i < C; ++i)
#pragma unroll
        for (int u = 0; u < U; ++u) add_into<DT>(acc[u], x[i][u]);
}

// Every block handles one row of BLOCK*U consecutive vectors, so blocks stream
// through memory in launch order (a bounded grid whose blocks loop over distant
// rows measured slower).
template <int DT, bool NT, int U>
__global__ __launch_bounds__(BLOCK) void flat_reduce_kernel(const char* __restrict__ in0,
                                                            int64_t stride, char* __restrict__ out,
                                                            int64_t nvec, int R, Scale sc) {
    constexpr int VEC = Fmt<DT>::VEC;
    const int64_t row = blockIdx.x;
    float acc[U][VEC];
    if ((row + 1) * (BLOCK * U) <= nvec) {
        const int64_t row_byte = row * (BLOCK * U * 16);
        uint32_t lane_off[U];
#pragma unroll
        for (int u = 0; u < U; ++u) lane_off[u] = (u * BLOCK + threadIdx.x) * 16u;
        sum_interior<DT, NT, U>(
            [&](int r) { return in0 + static_cast<int64_t>(r) * stride + row_byte; }, R, lane_off, acc);
#pragma unroll
        for (int u = 0; u < U; ++u)
            store16s<NT>(out + row_byte + lane_off[u], scaled<DT>(sc, acc[u]));
        return;
    }
    int64_t off[U];
    bool ok[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int64_t v = row * (BLOCK * U) + u * BLOCK + threadIdx.x;
        ok[u] = v < nvec;
        off[u] = v * 16;
#pragma unroll
        for (int i = 0; i < VEC; ++i) acc[u][i] = -0.0f;   // -0 + x == x for every x
    }
    int r = 0;
    for (; r + 8 <= R; r += 8) chunk_flat<DT, NT, 8, U>(in0, stride, r, off, ok, acc);
    if (r + 4 <= R) { chunk_flat<DT, NT, 4, U>(in0, stride, r, off, ok, acc); r += 4; }
    if (r + 2 <= R) { chunk_flat<DT, NT, 2, U>(in0, stride, r, off, ok, acc); r += 2; }
    if (r < R) { chunk_flat<DT, NT, 1, U>(in0, stride, r, off, ok, acc); }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        if (!ok[u]) continue;
        float y[VEC];
#pragma unroll
        for (int i = 0; i < VEC; ++i) y[i] = apply_scale(sc, acc[u][i]);
        store16s<NT>(out + off[u], Fmt<DT>::narrow(y));
    }
}

// Fused variant, boundary tiles: replica pointers come from the segment table
// and lanes are predicated.  The C pointers are fetched first (one scalar
// load), then all C*U vector loads are issued, then the adds run in order.
template <int DT, bool NT, int C, int U>
__device__ __forceinline__ void chunk_seg(void* const* __restrict__ row, int r, uint64_t used, bool aligned,
                                          const int64_t (&off)[U], const bool (&ok)[U],
                                          float (&acc)[U][Fmt<DT>::VEC]) {
    const char* base[C];
#pragma unroll
    for (int i = 0; i < C; ++i) base[i] = static_cast<const char*>(row[r + i]);
    u32x4 x[C][U];
    // a replica that did not use the parameter contributes +0 in its place in
    // the sum, and its tensor is not read
#pragma unroll
    for (int i = 0; i < C; ++i)
#pragma unroll
        for (int u = 0; u < U; ++u)
            x[i][u] = (ok[u] && ((used >> (r + i)) & 1u))
                          ? (aligned ? load16<NT>(base[i] + off[u]) : load16u<NT>(base[i] + off[u]))
                          : zero16();
#pragma unroll
    for (int i = 0; i < C; ++i)
#pragma unroll
        for (int u = 0; u < U; ++u) add_into<DT>(acc[u], x[i][u]);
}

// Where the averages go.  Normally into the gradient tensors themselves, in
// their own format (replica 0's, or all of them).  With OUT32 the gradients are a
// 16-bit transport format (Section 6.2.3) and the averages are written as
// binary32, unrounded, to a separate tensor per parameter (SegTables::out): two
// 16-byte stores per 16-byte input vector, at twice the byte offset.
template <int DT, bool NT>
__device__ __forceinline__ void store_out32(char* out, int64_t in_byte_off, const float (&y)[Fmt<DT>::VEC],
                                            bool aligned = true) {
    static_assert(Fmt<DT>::VEC == 8, "binary32 outputs are for the 16-bit formats");
    u32x4 lo, hi;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        lo[i] = __float_as_uint(y[i]);
        hi[i] = __float_as_uint(y[4 + i]);
    }
    if (aligned) {
        store16s<NT>(out + 2 * in_byte_off, lo);
        store16s<NT>(out + 2 * in_byte_off + 16, hi);
    } else {
        store16u<NT>(out + 2 * in_byte_off, lo);
        store16u<NT>(out + 2 * in_byte_off + 16, hi);
    }
}

// The same for a whole wave whose 64 lanes hold 64 consecutive input vectors (interior tiles):
// lane i's eight values belong at bytes [32 i, 32 i + 32) of the wave's 2 KiB of output, which
// two stores per lane at a stride of 32 bytes would write as half cache lines (counters: 10 %
// more bytes written than the averages hold).  The values are exchanged between the lanes
// instead, so that each of the two store instructions writes 1 KiB without gaps: lane i stores
// floats 4 i .. 4 i + 3 of the first KiB, then of the second.
template <int DT, bool NT>
__device__ __forceinline__ void store_out32_wave(char* out, int64_t in_byte_off, const float (&y)[Fmt<DT>::VEC]) {
    static_assert(Fmt<DT>::VEC == 8, "binary32 outputs are for the 16-bit formats");
    const int lane = threadIdx.x & 63;
    char* wave_base = out + 2 * in_byte_off - 32 * lane;
    const int src = lane >> 1;                // the lane whose vector holds floats 4 i .. 4 i + 3
    const bool upper = (lane & 1) != 0;       // ... in its upper half
    u32x4 a, b;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int lo = __float_as_int(y[k]), hi = __float_as_int(y[4 + k]);
        const int a_lo = __shfl(lo, src), a_hi = __shfl(hi, src);
        const int b_lo = __shfl(lo, 32 + src), b_hi = __shfl(hi, 32 + src);
        a[k] = static_cast<uint32_t>(upper ? a_hi : a_lo);
        b[k] = static_cast<uint32_t>(upper ? b_hi : b_lo);
    }
    store16s<NT>(wave_base + 16 * lane, a);
    store16s<NT>(wave_base + 1024 + 16 * lane, b);
}

template <int DT, bool OUT32 = false>
__device__ __forceinline__ void reduce_element(const SegTables& t, int g, int R, int nwrite,
                                               int64_t idx, bool zero, uint64_t used, const Scale& sc) {
    constexpr int ES = Fmt<DT>::ES;
    float y = 0.0f;
    if (!zero) {
        float s = -0.0f;
        for (int r = 0; r < R; ++r) {
            float x = 0.0f;
            if ((used >> r) & 1u)
                x = Fmt<DT>::load1(static_cast<const char*>(t.grad[static_cast<int64_t>(g) * t.R + r]) + idx * ES);
            s += x;
        }
        y = apply_scale(sc, s);
    }
    if (OUT32) {
        gstore<float>(static_cast<char*>(t.out[g]) + idx * 4, y);
        return;
    }
    for (int w = 0; w < nwrite; ++w)
        Fmt<DT>::store1(static_cast<char*>(t.grad[static_cast<int64_t>(g) * t.R + w]) + idx * ES, y);
}

// Block-uniform: the R participation bytes of a segment as a bit mask.
__device__ __forceinline__ uint64_t used_mask(const uint8_t* __restrict__ flags, int R) {
    uint64_t m = 0;
    for (int r = 0; r < R; ++r)
        if (flags[r] != 0) m |= uint64_t(1) << r;
    return m;
}

// One tile of the fused gather-reduce-scatter.
// gate / tag: see GateRecord (null = no gate).  A launch whose gate gave up must
// not touch gradients that may still be incomplete; the repair launch redoes it.
// The gate word is fetched together with the tile's tables (one round of scalar
// loads, not one more in front of them) and looked at before any gradient is.
template <int DT, bool NT, int U, bool OUT32 = false>
__device__ __forceinline__ void fused_tile(const SegTables& t, int64_t tile, int R, int nwrite,
                                           const uint8_t* __restrict__ local, int keep_unused,
                                           const Scale& sc, const GateRecord* __restrict__ gate = nullptr,
                                           uint32_t tag = 0) {
    constexpr int ES = Fmt<DT>::ES;
    constexpr int VEC = Fmt<DT>::VEC;
    const uint32_t gate_word = gate != nullptr ? gate->failed_tag : ~tag;
    const int g = t.tile_seg[tile];
    // Everything that depends on g alone is fetched together: the segment
    // record and the first eight replica pointers (the pointer table is padded
    // so that eight entries can always be read).
    void* const* __restrict__ row = t.grad + static_cast<int64_t>(g) * t.R;   // this segment's R pointers
    const SegInfo si = t.seg[g];
    const char* pre[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) pre[i] = static_cast<const char*>(row[i]);
    if (gate_word == tag) return;          // the gate in front of this launch gave up
    const int64_t numel = si.numel;
    const int64_t ltile = tile - si.tile0;
    // participation of the R replicas in this parameter (bit r = replica r used
    // it); without a flag table every replica did
    const uint64_t everyone = R >= 64 ? ~uint64_t(0) : ((uint64_t(1) << R) - 1);
    const uint64_t used = local != nullptr ? used_mask(local + static_cast<int64_t>(g) * t.R, R) : everyone;
    if (used == 0 && keep_unused) return;   // globally unused: the gradients stay as they are
    const bool zero = used == 0;            // ... or become zeros
    const bool all_used = used == everyone;
    const int sh = si.lead_bytes() / ES;    // replica 0's tensor starts this many elements past a 16-byte boundary
    // every replica's tensor sits at the same offset modulo 16 (and, with binary32 outputs, the
    // output tensor sits where whole input vectors map to whole output vectors)
    const bool src_aligned = si.congruent();
    const bool fast = src_aligned && (!OUT32 || si.out_congruent());
    char* const outp = OUT32 ? static_cast<char*>(t.out[g]) : nullptr;
    const int64_t e_tile = ltile * (TILE_BYTES / ES) - sh;

    if (fast && all_used && e_tile >= 0 && e_tile + TILE_BYTES / ES <= numel) {
        // the whole tile is inside the segment, every replica took part and all are aligned alike
        const int64_t tile_byte = e_tile * ES;
#pragma unroll 1
        for (int step = 0; step < TILE_VECS / (BLOCK * U); ++step) {
            uint32_t lane_off[U];
            float acc[U][VEC];
#pragma unroll
            for (int u = 0; u < U; ++u) lane_off[u] = ((step * U + u) * BLOCK + threadIdx.x) * 16u;
            sum_interior_pre<DT, NT, U>(
                pre, tile_byte, [&](int r) { return static_cast<const char*>(row[r]) + tile_byte; }, R,
                lane_off, acc);
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (OUT32) {
                    float y[VEC];
#pragma unroll
                    for (int i = 0; i < VEC; ++i) y[i] = apply_scale(sc, acc[u][i]);
                    if constexpr (OUT32) store_out32_wave<DT, NT>(outp, tile_byte + lane_off[u], y);
                    continue;
                }
                const u32x4 out = scaled<DT>(sc, acc[u]);
                store16s<NT>(const_cast<char*>(pre[0]) + tile_byte + lane_off[u], out);
                for (int w = 1; w < nwrite; ++w)
                    store16s<NT>(static_cast<char*>(row[w]) + tile_byte + lane_off[u], out);
            }
        }
        return;
    }

#pragma unroll 1
    for (int step = 0; step < TILE_VECS / (BLOCK * U); ++step) {
        int64_t e[U], off[U];
        int kind[U];
        bool ok[U];
        float acc[U][VEC];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            e[u] = e_tile + static_cast<int64_t>((step * U + u) * BLOCK + threadIdx.x) * VEC;
            kind[u] = classify(e[u], VEC, numel);
            ok[u] = kind[u] == V_FULL && !zero;
            off[u] = e[u] * ES;
#pragma unroll
            for (int i = 0; i < VEC; ++i) acc[u][i] = -0.0f;
        }
        if (!zero) {
            // vectors sit on replica 0's 16-byte grid; replicas that are shifted against it
            // are read with element-aligned 16-byte loads
            int r = 0;
            for (; r + 8 <= R; r += 8) chunk_seg<DT, NT, 8, U>(row, r, used, src_aligned, off, ok, acc);
            if (r + 4 <= R) { chunk_seg<DT, NT, 4, U>(row, r, used, src_aligned, off, ok, acc); r += 4; }
            if (r + 2 <= R) { chunk_seg<DT, NT, 2, U>(row, r, used, src_aligned, off, ok, acc); r += 2; }
            if (r < R) { chunk_seg<DT, NT, 1, U>(row, r, used, src_aligned, off, ok, acc); }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (kind[u] == V_NONE) continue;
            if (kind[u] == V_FULL) {
                float y[VEC];
#pragma unroll
                for (int i = 0; i < VEC; ++i) y[i] = zero ? 0.0f : apply_scale(sc, acc[u][i]);
                if (OUT32) {
                    if constexpr (OUT32) store_out32<DT, NT>(outp, off[u], y, si.out_congruent());
                    continue;
                }
                const u32x4 out = zero ? zero16() : Fmt<DT>::narrow(y);
                store16s<NT>(static_cast<char*>(row[0]) + off[u], out);
                for (int w = 1; w < nwrite; ++w) {
                    char* d = static_cast<char*>(t.grad[static_cast<int64_t>(g) * t.R + w]);
                    if (src_aligned) store16s<NT>(d + off[u], out);
                    else store16u<NT>(d + off[u], out);
                }
            } else {
                for (int i = 0; i < VEC; ++i) {
                    const int64_t idx = e[u] + i;
                    if (idx >= 0 && idx < numel) reduce_element<DT, OUT32>(t, g, R, nwrite, idx, zero, used, sc);
                }
            }
        }
    }
}

template <int DT, bool NT, int U, bool OUT32 = false>
__global__ __launch_bounds__(BLOCK) void fused_reduce_kernel(SegTables t, int64_t tile_base, int R,
                                                             int nwrite,
                                                             const uint8_t* __restrict__ local,
                                                             int keep_unused, Scale sc,
                                                             const GateRecord* __restrict__ gate,
                                                             uint32_t tag, DispatchSignal sig) {
    // the last block of the grid tells that the launch has been dispatched in full (blocks start
    // in index order): a launch chained behind this one may begin to fill the compute units
    // (reporting a few hundred blocks earlier, to make up for the start-up of the next launch,
    // measured no better; 1024 and more blocks earlier lose the gain)
    if (sig.word != nullptr && blockIdx.x == gridDim.x - 1 && threadIdx.x == 0)
        __hip_atomic_fetch_max(sig.word, sig.ord, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    fused_tile<DT, NT, U, OUT32>(t, tile_base + blockIdx.x, R, nwrite, local, keep_unused, sc, gate, tag);
}

// ---- stream ordering through device flags ------------------------------------
constexpr uint32_t MAX_GATE_POLLS = 1u << 22;

// Memory ordering of the handshake.  What the bucket kernel must see is written
// by kernels that precede the announcement on the backward stream, and the bucket
// kernel is a launch of its own behind the gate.  Both hops are kernel boundaries
// of a stream: the writers have ended (their results are released to the device)
// before the announcing kernel starts, and the bucket kernel acquires at its
// start, after the gate has ended.  The sequence number itself therefore needs no
// release or acquire of its own -- a release here would only write back this
// XCD's L2, which holds none of the gradients in question but a good deal of the
// concurrently running reduce kernel's lines (measured: 11 us per announcement
// next to a BERT-sized reduction) -- just device-wide atomicity and visibility,
// which relaxed agent-scope atomics give.
__global__ __launch_bounds__(64) void announce_kernel(OrderState* st, unsigned long long seq) {
    if (threadIdx.x == 0)
        __hip_atomic_store(&st->ready_seq, seq, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// One wave; lane 0 polls.  Both bounds (wall-clock ticks and the poll count) end
// the loop whatever the other stream does.
__global__ __launch_bounds__(64) void gate_kernel(OrderState* st, unsigned long long need,
                                                  long long wait_ticks, GateRecord* rec, GateRecord* row_summary,
                                                  int32_t tile_base, int32_t ntiles, int32_t dtype,
                                                  uint32_t tag, unsigned long long chain_ord, long long chain_ticks) {
    if (threadIdx.x != 0) return;
    bool ok = false;
    if (__hip_atomic_load(&st->abort_tag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != tag) {
        const uint64_t t0 = wall_clock64();
        for (uint32_t poll = 0; poll < MAX_GATE_POLLS; ++poll) {
            if (__hip_atomic_load(&st->ready_seq, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= need) {
                ok = true;
                break;
            }
            if (static_cast<long long>(wall_clock64() - t0) >= wait_ticks) break;
            __builtin_amdgcn_s_sleep(2);
        }
    }
    if (ok && chain_ticks > 0) {
        // scheduling only: let the launch this one is chained to reach its last block first
        const uint64_t t1 = wall_clock64();
        for (uint32_t poll = 0; poll < MAX_GATE_POLLS; ++poll) {
            if (__hip_atomic_load(&st->dispatched, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= chain_ord) break;
            if (static_cast<long long>(wall_clock64() - t1) >= chain_ticks) break;
            __builtin_amdgcn_s_sleep(2);
        }
    }
    if (!ok) {
        rec->tile_base = tile_base;
        rec->ntiles = ntiles;
        rec->dtype = dtype;
        rec->failed_tag = tag;
        row_summary->failed_tag = tag;
        __hip_atomic_store(&st->abort_tag, tag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// The same handshake in the other direction, once per iteration and reduction stream: the
// stream's bucket kernels have ended when done_kernel runs, and what follows join_kernel on the
// backward stream starts after it has ended.
__global__ __launch_bounds__(64) void done_kernel(OrderState* st, int lane, unsigned long long tag) {
    if (threadIdx.x == 0)
        __hip_atomic_store(&st->lane_done[lane], tag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__global__ __launch_bounds__(64) void join_kernel(OrderState* st, uint32_t lane_mask, unsigned long long tag,
                                                  long long wait_ticks) {
    if (threadIdx.x != 0) return;
    const uint64_t t0 = wall_clock64();
    for (uint32_t poll = 0; poll < MAX_GATE_POLLS; ++poll) {
        uint32_t missing = 0;
        for (int l = 0; l < kOrderLanes; ++l)
            if ((lane_mask >> l) & 1u)
                missing |= __hip_atomic_load(&st->lane_done[l], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < tag ? 1u : 0u;
        if (!missing) break;
        if (static_cast<long long>(wall_clock64() - t0) >= wait_ticks) break;
        __builtin_amdgcn_s_sleep(2);
    }
}

__global__ __launch_bounds__(64) void chain_wait_kernel(OrderState* st, unsigned long long chain_ord, long long chain_ticks) {
    if (threadIdx.x != 0) return;
    const uint64_t t0 = wall_clock64();
    for (uint32_t poll = 0; poll < MAX_GATE_POLLS; ++poll) {
        if (__hip_atomic_load(&st->dispatched, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= chain_ord) break;
        if (static_cast<long long>(wall_clock64() - t0) >= chain_ticks) break;
        __builtin_amdgcn_s_sleep(2);
    }
}

// Launches whose gate gave up, redone once every gradient exists.  Block j takes
// the tiles j, j + G, ... of each failed launch.
template <int DT, bool NT, int U, bool OUT32 = false>
__global__ __launch_bounds__(BLOCK) void repair_kernel(SegTables t, OrderState* st,
                                                       const GateRecord* __restrict__ rec,
                                                       int nb, uint32_t tag, int R, int nwrite,
                                                       const uint8_t* __restrict__ local,
                                                       int keep_unused, Scale sc) {
    // rec[nb] is the row's summary: no gate of the iteration gave up (the normal case), nothing to look for
    if (rec[nb].failed_tag != tag) return;
    for (int b = 0; b < nb; ++b) {
        const GateRecord r = rec[b];
        if (r.failed_tag != tag || r.dtype != DT) continue;
        if (blockIdx.x == 0 && threadIdx.x == 0) st->repaired += 1;   // (repair launches run one after the other)
        for (int64_t i = blockIdx.x; i < r.ntiles; i += gridDim.x)
            fused_tile<DT, NT, U, OUT32>(t, r.tile_base + i, R, nwrite, local, keep_unused, sc);
    }
}

__global__ __launch_bounds__(64) void probe_wait_kernel(unsigned long long* word, unsigned long long value,
                                                        long long wait_ticks) {
    if (threadIdx.x != 0) return;
    const uint64_t t0 = wall_clock64();
    unsigned long long seen = 0;
    for (uint32_t poll = 0; poll < MAX_GATE_POLLS; ++poll) {
        if (__hip_atomic_load(&word[0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == value) {
            seen = 1;
            break;
        }
        if (static_cast<long long>(wall_clock64() - t0) >= wait_ticks) break;
        __builtin_amdgcn_s_sleep(16);
    }
    word[1] = seen;
}

__global__ __launch_bounds__(64) void probe_write_kernel(unsigned long long* word, unsigned long long value) {
    if (threadIdx.x == 0)
        __hip_atomic_store(&word[0], value, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// ---- K4: no_sync accumulation ---------------------------------------------
template <int DT>
__device__ __forceinline__ void accumulate_tile(const char* __restrict__ src, char* dst,
                                                int64_t numel, int64_t ltile) {
    constexpr int ES = Fmt<DT>::ES;
    constexpr int VEC = Fmt<DT>::VEC;
    constexpr int U = 2;
    const int sh = lead_in(dst, ES);
    const bool cong = congruent16(src, dst);
    const int64_t e_tile = ltile * (TILE_BYTES / ES) - sh;
#pragma unroll 1
    for (int step = 0; step < TILE_VECS / (BLOCK * U); ++step) {
        int64_t e[U];
        int kind[U];
        u32x4 a[U], b[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            e[u] = e_tile + static_cast<int64_t>((step * U + u) * BLOCK + threadIdx.x) * VEC;
            kind[u] = classify(e[u], VEC, numel);
            a[u] = zero16();
            b[u] = zero16();
            if (kind[u] == V_FULL) {
                a[u] = load16<false>(dst + e[u] * ES);
                b[u] = cong ? load16<true>(src + e[u] * ES) : load16u<true>(src + e[u] * ES);
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (kind[u] == V_FULL) {
                float fa[VEC], fb[VEC];
                Fmt<DT>::widen(a[u], fa);
                Fmt<DT>::widen(b[u], fb);
#pragma unroll
                for (int i = 0; i < VEC; ++i) fa[i] = fa[i] + fb[i];
                store16(dst + e[u] * ES, Fmt<DT>::narrow(fa));
            } else if (kind[u] == V_EDGE) {
                for (int i = 0; i < VEC; ++i) {
                    const int64_t idx = e[u] + i;
                    if (idx < 0 || idx >= numel) continue;
                    const float s = Fmt<DT>::load1(dst + idx * ES) + Fmt<DT>::load1(src + idx * ES);
                    Fmt<DT>::store1(dst + idx * ES, s);
                }
            }
        }
    }
}

__global__ __launch_bounds__(BLOCK) void accumulate_kernel(SegTables t, int n,
                                                           void* const* __restrict__ micro) {
    const int64_t tile = blockIdx.x;
    const int r = blockIdx.y;
    const int g = t.tile_seg[tile];
    const SegInfo si = t.seg[g];
    const char* src = static_cast<const char*>(micro[static_cast<int64_t>(r) * n + si.param]);
    if (src == nullptr) return;
    char* dst = static_cast<char*>(t.grad[static_cast<int64_t>(g) * t.R + r]);
    const int64_t numel = si.numel;
    const int64_t ltile = tile - si.tile0;
    switch (si.dtype()) {
        case 0: accumulate_tile<0>(src, dst, numel, ltile); break;
        case 1: accumulate_tile<1>(src, dst, numel, ltile); break;
        default: accumulate_tile<2>(src, dst, numel, ltile); break;
    }
}

// ---- global participation bitmap ---------------------------------------------
// The one-GPU form of the extra AllReduce on the unused-parameter bitmap
// (Section 4.2): global[g] = OR over the R replicas of local[g][r].
__global__ __launch_bounds__(BLOCK) void bitmap_or_kernel(const uint8_t* __restrict__ local,
                                                          uint8_t* __restrict__ global, int G, int R) {
    const int g = blockIdx.x * BLOCK + threadIdx.x;
    if (g >= G) return;
    uint8_t any = 0;
    for (int r = 0; r < R; ++r) any |= local[static_cast<int64_t>(g) * R + r] != 0 ? 1 : 0;
    global[g] = any;
}

// ---- K6: synthetic backward emitter -----------------------------------------
// With ticks > 0 every wave waits until `ticks` of the constant-rate wall clock
// have passed (at most MAX_SPINS polls, so the kernel always ends); with a
// pointer row replica blockIdx.y's gradient is copied from its source.  The
// host launches the two roles separately (launch_emit).
constexpr uint32_t MAX_SPINS = 1u << 20;

__global__ __launch_bounds__(BLOCK) void emit_kernel(int64_t ticks, void* const* __restrict__ ptrs,
                                                     int R, int64_t nelem, int es, int busy,
                                                     float* __restrict__ sink) {
    if (ticks > 0) {
        const uint64_t t0 = wall_clock64();
        float a = static_cast<float>(threadIdx.x);
        for (uint32_t spin = 0; spin < MAX_SPINS; ++spin) {
            if (static_cast<int64_t>(wall_clock64() - t0) >= ticks) break;
            if (busy) {
                // arithmetic between polls: the delay looks like compute to the GPU's
                // power management instead of like an idle wait
#pragma unroll
                for (int i = 0; i < 64; ++i) a = a * 1.0000001f + 0.5f;
            } else {
                __builtin_amdgcn_s_sleep(4);
            }
        }
        if (busy && a == 12345.678f && sink != nullptr) sink[0] = a;   // keeps the arithmetic alive
    }
    if (ptrs == nullptr) return;
    const int r = blockIdx.y;
    if (r >= R) return;
    char* dst = static_cast<char*>(ptrs[r]);
    const char* src = static_cast<const char*>(ptrs[R + r]);
    const int64_t stride = static_cast<int64_t>(gridDim.x) * BLOCK;
    for (int64_t i = static_cast<int64_t>(blockIdx.x) * BLOCK + threadIdx.x; i < nelem; i += stride) {
        if (es == 4) gstore<uint32_t>(dst + i * 4, gload<uint32_t>(src + i * 4));
        else gstore<uint16_t>(dst + i * 2, gload<uint16_t>(src + i * 2));
    }
}

inline hipError_t after_launch() { return hipGetLastError(); }

// Every kernel here streams through HBM and needs only a few resident blocks per
// CU to keep the memory system full; more blocks mean more interleaved request
// streams at the DRAM channels and measurably less throughput.  `lds` bytes of
// dynamic LDS that no kernel touches cap the number of resident blocks
// (a CU has 160 KiB of LDS): 0 = no cap.
constexpr unsigned kLdsNoOptIn = 64 * 1024;
constexpr unsigned kLdsPerUnit = 160 * 1024;     // gfx950

// the pair of events that the next launch through launch() on this thread carries (time_next_launch)
thread_local hipEvent_t g_time_start = nullptr, g_time_stop = nullptr;

template <typename... KArgs, typename... Args>
static hipError_t launch(void (*kernel)(KArgs...), dim3 grid, unsigned lds, hipStream_t s, Args... args) {
    if (lds > kLdsNoOptIn) {
        // allocations above 64 KiB must be allowed per kernel; once is enough
        // (per device: the attribute belongs to the kernel's code object on the current device)
        static std::mutex mu;
        static std::set<std::pair<int, const void*>> raised;
        int dev = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e != hipSuccess) return e;
        const std::pair<int, const void*> key(dev, reinterpret_cast<const void*>(kernel));
        std::lock_guard<std::mutex> lock(mu);
        if (raised.find(key) == raised.end()) {
            e = hipFuncSetAttribute(key.second, hipFuncAttributeMaxDynamicSharedMemorySize,
                                    static_cast<int>(kLdsPerUnit));
            if (e != hipSuccess) return e;
            raised.insert(key);
        }
    }
    if (g_time_start) {
        // the runtime stamps the two events with this kernel's own start and end: no packet of
        // its own sits between consecutive kernels, as an event record would
        hipEvent_t a = g_time_start, b = g_time_stop;
        g_time_start = g_time_stop = nullptr;
        hipExtLaunchKernelGGL(kernel, grid, dim3(BLOCK), lds, s, a, b, 0u, static_cast<KArgs>(args)...);
    } else {
        hipLaunchKernelGGL(kernel, grid, dim3(BLOCK), lds, s, static_cast<KArgs>(args)...);
    }
    return hipGetLastError();
}

}  // namespace

// ---- launch wrappers ---------------------------------------------------------
void time_next_launch(hipEvent_t start, hipEvent_t stop) {
    g_time_start = start;
    g_time_stop = stop;
}

bool timing_pair_unused() {
    const bool unused = g_time_start != nullptr;
    g_time_start = g_time_stop = nullptr;
    return unused;
}

hipError_t launch_pack(const SegTables& t, int64_t tile_base, int64_t ntiles, char* slab0,
                       int64_t slab_stride, int nrep, const uint8_t* local, hipStream_t s) {
    if (ntiles <= 0 || nrep <= 0) return hipSuccess;
    dim3 grid(static_cast<unsigned>(ntiles), static_cast<unsigned>(nrep));
    return launch(seg_copy_kernel<true>, grid, 0u, s, t, tile_base, slab0, slab_stride, local, 0);
}

hipError_t launch_unpack(const SegTables& t, int64_t tile_base, int64_t ntiles,
                         const char* out_slab, int nrep, const uint8_t* global_used, bool keep_unused,
                         hipStream_t s) {
    if (ntiles <= 0 || nrep <= 0) return hipSuccess;
    dim3 grid(static_cast<unsigned>(ntiles), static_cast<unsigned>(nrep));
    const int keep = keep_unused ? 1 : 0;
    return launch(seg_copy_kernel<false>, grid, 0u, s, t, tile_base, const_cast<char*>(out_slab), int64_t(0), global_used, keep);
}

// Vectors per thread and replica in the reduce kernels: a tile's worth (two), which measured
// best against one and four on both model-shaped lists.
constexpr int RU = TILE_VECS / BLOCK;

template <int DT>
static hipError_t flat_reduce_dispatch(bool nt, unsigned lds, hipStream_t s, const char* in0, int64_t stride,
                                       char* out, int64_t nvec, int R, Scale sc) {
    const int64_t nrows = (nvec + BLOCK * RU - 1) / (BLOCK * RU);
    dim3 grid(static_cast<unsigned>(nrows));
    if (nt) return launch(flat_reduce_kernel<DT, true, RU>, grid, lds, s, in0, stride, out, nvec, R, sc);
    return launch(flat_reduce_kernel<DT, false, RU>, grid, lds, s, in0, stride, out, nvec, R, sc);
}

hipError_t launch_flat_reduce(int dtype, const char* in0, int64_t stride, char* out, int64_t nvec,
                              int R, Scale sc, bool nontemporal, unsigned lds, hipStream_t s) {
    if (nvec <= 0) return hipSuccess;
    switch (dtype) {
        case 0: return flat_reduce_dispatch<0>(nontemporal, lds, s, in0, stride, out, nvec, R, sc);
        case 1: return flat_reduce_dispatch<1>(nontemporal, lds, s, in0, stride, out, nvec, R, sc);
        case 2: return flat_reduce_dispatch<2>(nontemporal, lds, s, in0, stride, out, nvec, R, sc);
        default: return hipErrorInvalidValue;
    }
}

template <int DT>
static hipError_t fused_dispatch(bool nt, int64_t ntiles, unsigned lds, hipStream_t s,
                                 const SegTables& t, int64_t tile_base, int R, int nwrite,
                                 const uint8_t* local, int keep, Scale sc, const GateRecord* gate, uint32_t tag,
                                 DispatchSignal sig) {
    dim3 grid(static_cast<unsigned>(ntiles));
    if (nt) return launch(fused_reduce_kernel<DT, true, RU>, grid, lds, s, t, tile_base, R, nwrite, local, keep, sc, gate, tag, sig);
    return launch(fused_reduce_kernel<DT, false, RU>, grid, lds, s, t, tile_base, R, nwrite, local, keep, sc, gate, tag, sig);
}

hipError_t launch_fused_reduce(int dtype, const SegTables& t, int64_t tile_base, int64_t ntiles,
                               int R, int nwrite, const uint8_t* local, bool keep_unused, Scale sc,
                               bool nontemporal, unsigned lds,
                               const GateRecord* gate, uint32_t tag, DispatchSignal sig, hipStream_t s) {
    if (ntiles <= 0) return hipSuccess;
    const int keep = keep_unused ? 1 : 0;
    if (t.out != nullptr) {
        // 16-bit gradients, binary32 averages to separate tensors
        constexpr int U = RU;
        if (nwrite != 1 || (dtype != 1 && dtype != 2)) return hipErrorInvalidValue;
        const dim3 grid(static_cast<unsigned>(ntiles));
        if (dtype == 1)
            return nontemporal ? launch(fused_reduce_kernel<1, true, U, true>, grid, lds, s, t, tile_base, R, nwrite, local, keep, sc, gate, tag, sig)
                               : launch(fused_reduce_kernel<1, false, U, true>, grid, lds, s, t, tile_base, R, nwrite, local, keep, sc, gate, tag, sig);
        return nontemporal ? launch(fused_reduce_kernel<2, true, U, true>, grid, lds, s, t, tile_base, R, nwrite, local, keep, sc, gate, tag, sig)
                           : launch(fused_reduce_kernel<2, false, U, true>, grid, lds, s, t, tile_base, R, nwrite, local, keep, sc, gate, tag, sig);
    }
    switch (dtype) {
        case 0: return fused_dispatch<0>(nontemporal, ntiles, lds, s, t, tile_base, R, nwrite, local, keep, sc, gate, tag, sig);
        case 1: return fused_dispatch<1>(nontemporal, ntiles, lds, s, t, tile_base, R, nwrite, local, keep, sc, gate, tag, sig);
        case 2: return fused_dispatch<2>(nontemporal, ntiles, lds, s, t, tile_base, R, nwrite, local, keep, sc, gate, tag, sig);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_announce(OrderState* st, unsigned long long seq, hipStream_t s) {
    hipLaunchKernelGGL(announce_kernel, dim3(1), dim3(64), 0, s, st, seq);
    return after_launch();
}

hipError_t launch_chain_wait(OrderState* st, unsigned long long chain_ord, long long chain_ticks, hipStream_t s) {
    hipLaunchKernelGGL(chain_wait_kernel, dim3(1), dim3(64), 0, s, st, chain_ord, chain_ticks);
    return after_launch();
}

hipError_t launch_done(OrderState* st, int lane, unsigned long long tag, hipStream_t s) {
    if (lane < 0 || lane >= kOrderLanes) return hipErrorInvalidValue;
    hipLaunchKernelGGL(done_kernel, dim3(1), dim3(64), 0, s, st, lane, tag);
    return after_launch();
}

hipError_t launch_join(OrderState* st, uint32_t lane_mask, unsigned long long tag, long long wait_ticks,
                       hipStream_t s) {
    if (lane_mask >> kOrderLanes) return hipErrorInvalidValue;
    hipLaunchKernelGGL(join_kernel, dim3(1), dim3(64), 0, s, st, lane_mask, tag, wait_ticks);
    return after_launch();
}

hipError_t launch_gate(OrderState* st, unsigned long long need, long long wait_ticks, GateRecord* rec,
                       GateRecord* row_summary, int32_t tile_base, int32_t ntiles, int32_t dtype, uint32_t tag,
                       unsigned long long chain_ord, long long chain_ticks, hipStream_t s) {
    hipLaunchKernelGGL(gate_kernel, dim3(1), dim3(64), 0, s, st, need, wait_ticks, rec, row_summary, tile_base,
                       ntiles, dtype, tag, chain_ord, chain_ticks);
    return after_launch();
}

hipError_t launch_repair(int dtype, const SegTables& t, OrderState* st, const GateRecord* rec, int nb, uint32_t tag,
                         int R, int nwrite, const uint8_t* local, bool keep_unused, Scale sc,
                         int blocks, bool nt, hipStream_t s) {
    if (blocks <= 0 || nb <= 0) return hipSuccess;
    constexpr int U = RU;
    const dim3 grid(static_cast<unsigned>(blocks));
    const int keep = keep_unused ? 1 : 0;
    if (t.out != nullptr) {
        if (nwrite != 1 || (dtype != 1 && dtype != 2)) return hipErrorInvalidValue;
        if (dtype == 1)
            return nt ? launch(repair_kernel<1, true, U, true>, grid, 0u, s, t, st, rec, nb, tag, R, nwrite, local, keep, sc)
                      : launch(repair_kernel<1, false, U, true>, grid, 0u, s, t, st, rec, nb, tag, R, nwrite, local, keep, sc);
        return nt ? launch(repair_kernel<2, true, U, true>, grid, 0u, s, t, st, rec, nb, tag, R, nwrite, local, keep, sc)
                  : launch(repair_kernel<2, false, U, true>, grid, 0u, s, t, st, rec, nb, tag, R, nwrite, local, keep, sc);
    }
    switch (dtype) {
        case 0: return nt ? launch(repair_kernel<0, true, U>, grid, 0u, s, t, st, rec, nb, tag, R, nwrite, local, keep, sc)
                          : launch(repair_kernel<0, false, U>, grid, 0u, s, t, st, rec, nb, tag, R, nwrite, local, keep, sc);
        case 1: return nt ? launch(repair_kernel<1, true, U>, grid, 0u, s, t, st, rec, nb, tag, R, nwrite, local, keep, sc)
                          : launch(repair_kernel<1, false, U>, grid, 0u, s, t, st, rec, nb, tag, R, nwrite, local, keep, sc);
        case 2: return nt ? launch(repair_kernel<2, true, U>, grid, 0u, s, t, st, rec, nb, tag, R, nwrite, local, keep, sc)
                          : launch(repair_kernel<2, false, U>, grid, 0u, s, t, st, rec, nb, tag, R, nwrite, local, keep, sc);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_probe(unsigned long long* word, unsigned long long value, long long wait_ticks,
                        hipStream_t waiter, hipStream_t writer) {
    hipLaunchKernelGGL(probe_wait_kernel, dim3(1), dim3(64), 0, waiter, word, value, wait_ticks);
    hipError_t e = after_launch();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(probe_write_kernel, dim3(1), dim3(64), 0, writer, word, value);
    return after_launch();
}

hipError_t launch_accumulate(const SegTables& t, int64_t ntiles, int R, int n, void* const* micro,
                             unsigned lds, hipStream_t s) {
    if (ntiles <= 0 || R <= 0) return hipSuccess;
    dim3 grid(static_cast<unsigned>(ntiles), static_cast<unsigned>(R));
    return launch(accumulate_kernel, grid, lds, s, t, n, micro);
}

hipError_t launch_bitmap_or(const uint8_t* local, uint8_t* global, int G, int R, hipStream_t s) {
    if (G <= 0) return hipSuccess;
    hipLaunchKernelGGL(bitmap_or_kernel, dim3((G + BLOCK - 1) / BLOCK), dim3(BLOCK), 0, s, local, global, G, R);
    return after_launch();
}

hipError_t launch_emit(int64_t ticks, void* const* ptrs, int R, int64_t nelem, int es,
                       int busy_blocks, float* sink, hipStream_t s) {
    // The delay and the copy are separate launches: a wait inside the copy's
    // blocks would start per block, and a grid with more blocks than fit on
    // the GPU at once would then wait several times the nominal delay.
    if (ticks > 0) {
        const unsigned bx = busy_blocks > 1 ? static_cast<unsigned>(busy_blocks) : 1u;
        hipLaunchKernelGGL(emit_kernel, dim3(bx, 1), dim3(BLOCK), 0, s, ticks,
                           static_cast<void* const*>(nullptr), R, int64_t(0), es,
                           busy_blocks > 0 ? 1 : 0, sink);
        const hipError_t e = after_launch();
        if (e != hipSuccess) return e;
    }
    if (ptrs == nullptr) return hipSuccess;
    int64_t want = (nelem + BLOCK * 8 - 1) / (BLOCK * 8);
    if (want < 1) want = 1;
    if (want > 1024) want = 1024;
    hipLaunchKernelGGL(emit_kernel, dim3(static_cast<unsigned>(want), static_cast<unsigned>(R)),
                       dim3(BLOCK), 0, s, int64_t(0), ptrs, R, nelem, es, 0, sink);
    return after_launch();
}

}  // namespace ddp
