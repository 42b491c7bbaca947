// Pieces shared by the MFMA kernels (gfx950): vector types, the wait-counter and raw LDS
// forms that keep the compiler from draining the global->LDS tile loads, and the
// workgroup barrier that orders LDS traffic only.  Internal to libdfk.
#pragma once

#include "dfk_device.h"
#include "dfk_internal.h"

namespace dfk {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;

constexpr int kTileBytes = 4096;   // one ring slot = 4 global->LDS instructions of 1 KB
constexpr int kKC = 128;           // k extent of a stage-one tile
constexpr int kLdsLimit = 160 * 1024 - 256;   // dynamic part; a few static words (flags) come on top
constexpr int kAuxNonTemporal = 2;  // cache-policy bit "nt": the weight stream is read once



#define DFK_LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))
// s_waitcnt with only vmcnt constrained (gfx9 encoding: vmcnt[3:0] | expcnt[6:4] | lgkmcnt[11:8] | vmcnt[5:4]<<14)
#define DFK_WAIT_VM(n) __builtin_amdgcn_s_waitcnt(0x0F70 | ((n) & 15) | ((((n) >> 4) & 3) << 14))
#define DFK_WAIT_LGKM0() __builtin_amdgcn_s_waitcnt(0xC07F)
#define DFK_STAMP(k) do { if (a.trace && tid == 0) a.trace[(size_t)blockIdx.x * 8 + (k)] = wall_clock64(); } while (0)

// Wait until at most `newer_ops` of this wavefront's vector-memory operations
// are outstanding (loads complete in issue order); newer_ops is a multiple of 4.
__device__ __forceinline__ void wait_vm_ops(int newer_ops) {
    switch (newer_ops >> 2) {
        case 0: DFK_WAIT_VM(0); break;
        case 1: DFK_WAIT_VM(4); break;
        case 2: DFK_WAIT_VM(8); break;
        case 3: DFK_WAIT_VM(12); break;
        case 4: DFK_WAIT_VM(16); break;
        case 5: DFK_WAIT_VM(20); break;
        case 6: DFK_WAIT_VM(24); break;
        case 7: DFK_WAIT_VM(28); break;
        case 8: DFK_WAIT_VM(32); break;
        case 9: DFK_WAIT_VM(36); break;
        case 10: DFK_WAIT_VM(40); break;
        case 11: DFK_WAIT_VM(44); break;
        case 12: DFK_WAIT_VM(48); break;
        case 13: DFK_WAIT_VM(52); break;
        case 14: DFK_WAIT_VM(56); break;
        default: DFK_WAIT_VM(60); break;
    }
    asm volatile("" ::: "memory");
}

// LDS stores and LDS atomics issued while tile loads are in flight go through
// these raw forms: for an LDS write the compiler sees, it first waits for every
// outstanding global->LDS load (it cannot tell the ring from the other arrays),
// which would drain the stream each time.  The arrays written here are never a
// target of tile loads.  Completion is awaited in lds_barrier.
__device__ __forceinline__ unsigned lds_addr(const void* p) {
    return (unsigned)(uintptr_t)(__attribute__((address_space(3))) const void*)p;
}
__device__ __forceinline__ void lds_write_b16_raw(unsigned addr, unsigned v) {
    asm volatile("ds_write_b16 %0, %1" : : "v"(addr), "v"(v) : "memory");
}

__device__ __forceinline__ void lds_write_b32_raw(unsigned addr, unsigned v) {
    asm volatile("ds_write_b32 %0, %1" : : "v"(addr), "v"(v) : "memory");
}
__device__ __forceinline__ void lds_write_b64_raw(unsigned addr, unsigned lo, unsigned hi) {
    typedef __attribute__((__vector_size__(2 * sizeof(unsigned)))) unsigned u32x2;
    const u32x2 v = u32x2{lo, hi};
    asm volatile("ds_write_b64 %0, %1" : : "v"(addr), "v"(v) : "memory");
}
__device__ __forceinline__ void lds_write_b128_raw(unsigned addr, __attribute__((__vector_size__(4 * sizeof(float)))) float v) {
    asm volatile("ds_write_b128 %0, %1" : : "v"(addr), "v"(v) : "memory");
}
// LDS reads of flags other wavefronts raise (waited for).  Through a plain volatile
// pointer these become flat loads, whose wait also covers every tile load in flight.
__device__ __forceinline__ unsigned lds_read_b32_raw(unsigned addr) {
    unsigned v;
    asm volatile("ds_read_b32 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(v) : "v"(addr) : "memory");
    return v;
}
__device__ __forceinline__ u32x4 lds_read_b128_raw(unsigned addr) {
    u32x4 v;
    asm volatile("ds_read_b128 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(v) : "v"(addr) : "memory");
    return v;
}
// LDS counter increment that returns the previous value (waits for it).
__device__ __forceinline__ unsigned lds_inc_rtn_raw(unsigned addr) {
    unsigned old, one = 1u;
    asm volatile("ds_add_rtn_u32 %0, %1, %2\n\ts_waitcnt lgkmcnt(0)" : "=v"(old) : "v"(addr), "v"(one) : "memory");
    return old;
}

// Workgroup barrier that orders LDS traffic only: it does not wait for the
// global->LDS tile loads in flight (a full __syncthreads would drain them).
// Written raw for the same reason: a fence the compiler sees waits for the tile
// loads, which also write LDS.
__device__ __forceinline__ void lds_barrier() {
    DFK_WAIT_LGKM0();
    asm volatile("s_barrier" ::: "memory");
}

__device__ __forceinline__ bf16x8 as_bf16x8(const u32x4& v) {
    union { u32x4 u; bf16x8 b; } c;
    c.u = v;
    return c.b;
}

// v_mfma_f32_16x16x32 for the element type: operands are the same 16 bytes per lane either way.
template <typename E>
__device__ __forceinline__ f32x4 mfma16(const u32x4& a, const u32x4& b, const f32x4& c);
template <>
__device__ __forceinline__ f32x4 mfma16<BF16>(const u32x4& a, const u32x4& b, const f32x4& c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(a), as_bf16x8(b), c, 0, 0, 0);
}
template <>
__device__ __forceinline__ f32x4 mfma16<FP16>(const u32x4& a, const u32x4& b, const f32x4& c) {
    union { u32x4 u; FP16::h8 h; } x, y;
    x.u = a; y.u = b;
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(x.h, y.h, c, 0, 0, 0);
}

}  // namespace
}  // namespace dfk
