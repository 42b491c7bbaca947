// Device-side helpers shared by the VALU and MFMA kernels (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

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
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    return f32_to_bf16_bits(lo) | (f32_to_bf16_bits(hi) << 16);
}

// SiLU(g) * u  (Background, SwiGLU equations): Sigmoid(g) * g * u.
__device__ __forceinline__ float silu_mul(float g, float u) {
    return u * (g / (1.0f + expf(-g)));
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
};
struct FP32 {
    static constexpr int VEC = 4;
    static constexpr int BYTES = 4;
    __device__ static __forceinline__ void widen(const u32x4& v, float (&f)[4]) {
        f[0] = __uint_as_float(v.x); f[1] = __uint_as_float(v.y);
        f[2] = __uint_as_float(v.z); f[3] = __uint_as_float(v.w);
    }
    __device__ static __forceinline__ void store(void* Y, size_t i, float v) { ((float*)Y)[i] = v; }
};

__device__ __forceinline__ u32x4 ld16(const void* base, size_t vec_index) {
    return ((const u32x4*)base)[vec_index];
}

// ---- device-scope fp32 accumulate / drain ----------------------------------
// Hardware float atomic add without return (device scope, relaxed).
__device__ __forceinline__ void acc_add(float* p, float v) {
    __hip_atomic_fetch_add(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// Read the accumulated value and leave zero behind, at the same coherence
// point as the adds (no plain load of memory other agents' atomics touched).
__device__ __forceinline__ float acc_take(float* p) {
    return __hip_atomic_exchange(p, 0.0f, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Device-scope fences.  A release makes the calling wavefront wait until all
// of its earlier stores and atomics have been performed for the whole device; it
// must be executed by every wavefront whose writes the arrival below publishes
// (a workgroup barrier alone does not wait for other wavefronts' memory traffic).
__device__ __forceinline__ void release_device() { __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent"); }
__device__ __forceinline__ void acquire_device() { __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent"); }

// Arrival counter: returns true for the last of `expected` arrivals, and resets
// the counter for the next call.  Release/acquire at device scope orders every
// earlier accumulate of the caller before the count, and the drain after it.
__device__ __forceinline__ bool arrive_last(unsigned* ticket, unsigned expected) {
    unsigned old = __hip_atomic_fetch_add(ticket, 1u, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
    if (old == expected - 1u) {
        __hip_atomic_store(ticket, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return true;
    }
    return false;
}

}  // namespace dfk
