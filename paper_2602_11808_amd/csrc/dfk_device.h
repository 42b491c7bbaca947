// Device-side helpers shared by the VALU and MFMA kernels (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "dfk_internal.h"

namespace dfk {

// 16 bytes as a native vector (what global_load_dwordx4 moves)
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// ---- bfloat16 <-> fp32 on raw bits ----------------------------------------
__device__ __forceinline__ float bf16_lo(uint32_t packed) { return __uint_as_float(packed << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t packed) { return __uint_as_float(packed & 0xFFFF0000u); }

// fp32 -> bf16 bits, round-to-nearest-even; NaN stays a quiet NaN.
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (u >> 16) | 0x0040u;
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}
// Two at once: the hardware's packed conversion (v_cvt_pk_bf16_f32, also round-to-nearest-even).
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    typedef float f32x2_t __attribute__((ext_vector_type(2)));
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    union { bf16x2_t b; uint32_t u; } c;
    c.b = __builtin_convertvector(f32x2_t{lo, hi}, bf16x2_t);
    return c.u;
}

// SiLU(g) * u  (Background, SwiGLU equations): Sigmoid(g) * g * u.
__device__ __forceinline__ float silu_mul(float g, float u) {
    return u * (g / (1.0f + expf(-g)));
}

// Same with the hardware's exp2 and reciprocal (about 1 ulp each): for results that
// are rounded to bf16 next.  exp2(+inf) -> rcp gives 0 for g << 0; no division.
__device__ __forceinline__ float silu_mul_fast(float g, float u) {
    return u * g * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.44269504088896341f * g));
}

// ---- element traits: 16-byte vectors of the storage type -------------------
struct BF16 {
    static constexpr int VEC = 8;  // elements per 16 bytes
    static constexpr int BYTES = 2;
    __device__ static __forceinline__ void widen(const u32x4& v, float (&f)[8]) {
        f[0] = bf16_lo(v.x); f[1] = bf16_hi(v.x);
        f[2] = bf16_lo(v.y); f[3] = bf16_hi(v.y);
        f[4] = bf16_lo(v.z); f[5] = bf16_hi(v.z);
        f[6] = bf16_lo(v.w); f[7] = bf16_hi(v.w);
    }
    __device__ static __forceinline__ void store(void* Y, size_t i, float v) {
        ((uint16_t*)Y)[i] = (uint16_t)f32_to_bf16_bits(v);
    }
    __device__ static __forceinline__ uint32_t pack2(float lo, float hi) { return pack_bf16x2(lo, hi); }
    __device__ static __forceinline__ void widen2(uint32_t packed, float& lo, float& hi) {
        lo = bf16_lo(packed); hi = bf16_hi(packed);
    }
    // four consecutive elements, i a multiple of 4
    __device__ static __forceinline__ void load4(const void* p, size_t i, float (&f)[4]) {
        const uint2 v = *(const uint2*)((const uint16_t*)p + i);
        widen2(v.x, f[0], f[1]); widen2(v.y, f[2], f[3]);
    }
    // four consecutive outputs, i a multiple of 4
    __device__ static __forceinline__ void store4(void* Y, size_t i, float a, float b, float c, float d) {
        uint2 v;
        v.x = pack_bf16x2(a, b);
        v.y = pack_bf16x2(c, d);
        *(uint2*)((uint16_t*)Y + i) = v;
    }
};
// IEEE binary16; conversions are the hardware's (round-to-nearest-even, exact widening).
struct FP16 {
    static constexpr int VEC = 8;
    static constexpr int BYTES = 2;
    typedef _Float16 h8 __attribute__((ext_vector_type(8)));
    __device__ static __forceinline__ void widen(const u32x4& v, float (&f)[8]) {
        union { u32x4 u; h8 h; } c;
        c.u = v;
#pragma unroll
        for (int i = 0; i < 8; ++i) f[i] = (float)c.h[i];
    }
    __device__ static __forceinline__ uint32_t bits(float v) {
        union { _Float16 h; uint16_t u; } c;
        c.h = (_Float16)v;
        return c.u;
    }
    __device__ static __forceinline__ void store(void* Y, size_t i, float v) { ((uint16_t*)Y)[i] = (uint16_t)bits(v); }
    __device__ static __forceinline__ uint32_t pack2(float lo, float hi) { return bits(lo) | (bits(hi) << 16); }
    __device__ static __forceinline__ void widen2(uint32_t packed, float& lo, float& hi) {
        union { uint32_t u; _Float16 h[2]; } c;
        c.u = packed;
        lo = (float)c.h[0]; hi = (float)c.h[1];
    }
    __device__ static __forceinline__ void load4(const void* p, size_t i, float (&f)[4]) {
        const uint2 v = *(const uint2*)((const uint16_t*)p + i);
        widen2(v.x, f[0], f[1]); widen2(v.y, f[2], f[3]);
    }
    __device__ static __forceinline__ void store4(void* Y, size_t i, float a, float b, float c, float d) {
        uint2 v;
        v.x = pack2(a, b);
        v.y = pack2(c, d);
        *(uint2*)((uint16_t*)Y + i) = v;
    }
};
struct FP32 {
    static constexpr int VEC = 4;
    static constexpr int BYTES = 4;
    __device__ static __forceinline__ void widen(const u32x4& v, float (&f)[4]) {
        f[0] = __uint_as_float(v.x); f[1] = __uint_as_float(v.y);
        f[2] = __uint_as_float(v.z); f[3] = __uint_as_float(v.w);
    }
    __device__ static __forceinline__ void store(void* Y, size_t i, float v) { ((float*)Y)[i] = v; }
    __device__ static __forceinline__ void load4(const void* p, size_t i, float (&f)[4]) {
        const float4 v = *(const float4*)((const float*)p + i);
        f[0] = v.x; f[1] = v.y; f[2] = v.z; f[3] = v.w;
    }
    __device__ static __forceinline__ void store4(void* Y, size_t i, float a, float b, float c, float d) {
        *(float4*)((float*)Y + i) = make_float4(a, b, c, d);
    }
};

__device__ __forceinline__ u32x4 ld16(const void* base, size_t vec_index) {
    return ((const u32x4*)base)[vec_index];
}
// Same for data that is read exactly once (the weight stream): non-temporal hint.
__device__ __forceinline__ u32x4 ld16_stream(const void* base, size_t vec_index) {
    return __builtin_nontemporal_load((const u32x4*)base + vec_index);
}

// ---- publishing partial sums to other workgroups ------------------------------
// Partial sums are published with device-scope (write-through) stores, so they
// are visible to the whole device once the issuing wavefront's memory counter
// has drained; no L2 write-back fence is needed on the writer side (such a fence
// executed by every wavefront was measured to dominate the kernel).  A reader
// invalidates its caches once (acquire_device) before it loads them.
//
// Hardware assumption (gfx950, and nothing else): the protocol is relaxed agent-scope
// stores, s_waitcnt vmcnt(0), a relaxed agent-scope read-modify-write on the arrival
// counter, and on the reader's side an acquire fence followed by plain loads.  There is
// no release operation, so in the language's memory model this is a data race; it is
// correct on this target because (a) an agent-scope store is issued with the sc1 bit and
// writes through the issuing XCD's L2 to memory, (b) vmcnt counts a store as complete
// only once that write has been acknowledged, and (c) agent-scope read-modify-writes are
// performed at the memory side, after the acknowledged writes.  The bitwise repeat-call
// tests of every reducer guard it; another target needs a release fence before the arrival.
#if defined(__HIP_DEVICE_COMPILE__) && !defined(__gfx950__)
#error "libdfk's cross-workgroup publish/arrive protocol is written for gfx950 only"
#endif
__device__ __forceinline__ void store2_device(float* p, float a, float b) {
    union { float f[2]; unsigned long long u; } c;
    c.f[0] = a; c.f[1] = b;
    __hip_atomic_store((unsigned long long*)p, c.u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void store4_device(float* p, float a, float b, float c, float d) {
    store2_device(p, a, b);
    store2_device(p + 2, c, d);
}
// Wait until every memory operation this wavefront has issued has completed.
__device__ __forceinline__ void drain_own_memory_ops() {
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
    asm volatile("" ::: "memory");
}
__device__ __forceinline__ void acquire_device() { __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent"); }

// Device-wide fp32 accumulate (hardware float atomic, no return) and the matching
// read-and-clear, performed at the same coherence point as the adds.
__device__ __forceinline__ void acc_add(float* p, float v) {
    __hip_atomic_fetch_add(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float acc_take(float* p) {
    return __hip_atomic_exchange(p, 0.0f, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Arrival counter: returns true for the last of `expected` arrivals, and resets
// the counter for the next call.  The caller orders its published stores before
// it (drain_own_memory_ops in every wavefront, then a workgroup barrier).
__device__ __forceinline__ bool arrive_last(unsigned* ticket, unsigned expected) {
    unsigned old = __hip_atomic_fetch_add(ticket, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (old == expected - 1u) {
        __hip_atomic_store(ticket, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return true;
    }
    return false;
}

// ---- split-d_ff reduction ----------------------------------------------------
// Every workgroup has published its fp32 partial block of Y ([m_count][d_model]
// floats, block index p) with store4_device.  Workgroups are gathered in
// first-level groups; the last of a group to arrive sums the group's blocks in
// a fixed order into the group block Q[q_slot] (or, if there is only one group
// for these columns, straight into Y); the last group to arrive sums the group
// blocks, again in a fixed order, and writes Y.  No workgroup ever waits for
// another, and the result does not depend on arrival order.
struct ReducePlan {
    float* P;
    float* Q;
    unsigned* tickets;
    int m_count, d_model;
    int c_lo, c_hi;             // columns (floats, multiples of 4) this group is responsible for
    int p_first, p_stride, n1;  // first-level members: blocks p_first + i*p_stride, i < n1
    int t1;                     // first-level counter
    int q_slot, n2, t2;         // second level: own group block, number of group blocks, counter
};

// Plan of the fused kernel (and of any kernel whose workgroup s of `S` holds a
// partial of all d_model columns): groups are the residues s mod NG, NG = ceil(S/16).
__device__ __forceinline__ ReducePlan plan_full_width(const MlpArgs& a, int s, int S) {
    ReducePlan r;
    const int ng = (S + kGroupSize - 1) / kGroupSize;
    const int g = s % ng;
    r.P = a.P; r.Q = a.Q; r.tickets = a.tickets;
    r.m_count = a.m_count; r.d_model = a.d_model;
    r.c_lo = 0; r.c_hi = a.d_model;
    r.p_first = g; r.p_stride = ng; r.n1 = (S - g + ng - 1) / ng;
    r.t1 = g;
    r.q_slot = g; r.n2 = ng; r.t2 = kTicketLevel2;
    return r;
}

// Plan of the second kernel of the two-kernel variant: workgroup (js, cb) holds
// the partial of d_ff split js for columns [c_lo, c_hi) and has stored it in those
// columns of block js (the workgroups of one split share a block); one level.
__device__ __forceinline__ ReducePlan plan_column_block(const MlpArgs& a, int cb, int c_lo, int c_hi) {
    ReducePlan r;
    r.P = a.P; r.Q = a.Q; r.tickets = a.tickets;
    r.m_count = a.m_count; r.d_model = a.d_model;
    r.c_lo = c_lo; r.c_hi = c_hi;
    r.p_first = 0; r.p_stride = 1; r.n1 = a.k2_splits;
    r.t1 = cb;
    r.q_slot = 0; r.n2 = 1; r.t2 = kTicketLevel2;
    return r;
}

// Sums, in ascending block order, the float4 at two positions (idx0 and idx0+nth of a
// [m][w4] index space) over n blocks `stride` floats apart.  All loads of a batch of
// 16 blocks for both positions are issued before the first add, so a reducer pays
// one memory round trip per 16 blocks instead of one per few loads.
__device__ __forceinline__ void sum_blocks2(const float* base, size_t stride, int n, int idx0, int nth, int total,
                                            int w4, int d_model, int c_lo, float4 (&s)[2], size_t (&off)[2]) {
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const int idx = min(idx0 + u * nth, total - 1);   // a clamped duplicate is computed and dropped by the caller
        const int m = idx / w4, c4 = idx - m * w4;
        off[u] = (size_t)m * d_model + c_lo + 4 * c4;
        s[u] = make_float4(0.f, 0.f, 0.f, 0.f);
    }
    for (int i0 = 0; i0 < n; i0 += 16) {
        float4 v[2][16];
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int k = 0; k < 16; ++k)
                v[u][k] = (i0 + k < n) ? *(const float4*)(base + (size_t)(i0 + k) * stride + off[u])
                                       : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int k = 0; k < 16; ++k) { s[u].x += v[u][k].x; s[u].y += v[u][k].y; s[u].z += v[u][k].z; s[u].w += v[u][k].w; }
    }
}

// Final store of four consecutive outputs: the sum, plus the residual input at the same
// position when there is one (it may be the output buffer itself: each element is read
// and then written by this one thread).
template <typename E>
__device__ __forceinline__ void store4_plus(void* Y, const void* resid, size_t i, const float4& v) {
    if (!resid) { E::store4(Y, i, v.x, v.y, v.z, v.w); return; }
    float r[4];
    E::load4(resid, i, r);
    E::store4(Y, i, v.x + r[0], v.y + r[1], v.z + r[2], v.w + r[3]);
}

template <typename E>
__device__ __forceinline__ void reduce_store(const ReducePlan& r, void* Y, int m_base, int* flag,
                                             unsigned long long* trace = nullptr, const void* resid = nullptr) {
    const int tid = threadIdx.x, nth = blockDim.x;
    const int w4 = (r.c_hi - r.c_lo) >> 2;
    const size_t blk = (size_t)r.m_count * r.d_model;
    // Every wavefront waits for its own published stores before the workgroup's
    // single arrival is counted.
    drain_own_memory_ops();
    __syncthreads();
    if (trace && tid == 0) trace[(size_t)blockIdx.x * 8 + 5] = wall_clock64();
    if (tid == 0) *flag = arrive_last(r.tickets + r.t1, (unsigned)r.n1) ? 1 : 0;
    __syncthreads();
    if (!*flag) { if (trace && tid == 0) trace[(size_t)blockIdx.x * 8 + 6] = wall_clock64(); return; }
    acquire_device();
    for (int idx0 = tid; idx0 < r.m_count * w4; idx0 += 2 * nth) {
        float4 s[2];
        size_t off[2];
        sum_blocks2(r.P + (size_t)r.p_first * blk, (size_t)r.p_stride * blk, r.n1, idx0, nth, r.m_count * w4, w4,
                    r.d_model, r.c_lo, s, off);
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int idx = idx0 + u * nth;
            if (idx < r.m_count * w4) {
                const int m = idx / w4, c4 = idx - m * w4;
                if (r.n2 == 1) store4_plus<E>(Y, resid, (size_t)(m_base + m) * r.d_model + r.c_lo + 4 * c4, s[u]);
                else store4_device(r.Q + (size_t)r.q_slot * blk + off[u], s[u].x, s[u].y, s[u].z, s[u].w);
            }
        }
    }
    if (r.n2 == 1) { if (trace && tid == 0) trace[(size_t)blockIdx.x * 8 + 6] = wall_clock64(); return; }
    drain_own_memory_ops();
    __syncthreads();
    if (tid == 0) *flag = arrive_last(r.tickets + r.t2, (unsigned)r.n2) ? 1 : 0;
    __syncthreads();
    if (trace && tid == 0) trace[(size_t)blockIdx.x * 8 + 6] = wall_clock64();
    if (!*flag) return;
    acquire_device();
    for (int idx0 = tid; idx0 < r.m_count * w4; idx0 += 2 * nth) {
        float4 s[2];
        size_t off[2];
        sum_blocks2(r.Q, blk, r.n2, idx0, nth, r.m_count * w4, w4, r.d_model, r.c_lo, s, off);
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int idx = idx0 + u * nth;
            if (idx < r.m_count * w4) {
                const int m = idx / w4, c4 = idx - m * w4;
                store4_plus<E>(Y, resid, (size_t)(m_base + m) * r.d_model + r.c_lo + 4 * c4, s[u]);
            }
        }
    }
    if (trace && tid == 0) trace[(size_t)blockIdx.x * 8 + 7] = wall_clock64();
}

}  // namespace dfk
