// VALU path: plain fp32 FMA kernels for any supported shape, in bf16 or in the
// fp32 test mode.  Fused single-launch kernel and the two-kernel variant share
// the two stage routines below.
//
// Stage one (Method, first stage): each wavefront owns rows j of the slice and
// streams W_gate[j,:] and W_up[j,:] with 128-bit loads, every lane keeping fp32
// partial dot products for up to MT tokens; a wavefront reduction yields
// G[m,j], U[m,j]; lane 0 applies SiLU(G)*U and leaves A_2[m,j] in LDS.
// Stage two (Method, second stage): each thread owns 16-byte column chunks of
// W_down and accumulates A_2[m,j] * W_down[j, chunk] over the slice's rows.
// The slice's fp32 partial Y is published to the workspace and is
// combined by the two-level arrival-counter reduction (reduce_store).
#include "dfk_device.h"
#include "dfk_internal.h"

namespace dfk {
namespace {

// MT * slice rows are held in LDS as fp32: dynamic LDS, which the launchers leave at the default 64 KiB
// allowance; the kernels add a static word (the reducer's flag), so the bound stays a little below it.
constexpr int kMaxLdsFloats = (64 * 1024 - 256) / 4;

template <typename E, int MT>
__device__ __forceinline__ void stage1_valu(const MlpArgs& a, int j0, int rows, int m0, int mt,
                                            float* a2s, int a2_stride) {
    constexpr int VEC = E::VEC;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int nwaves = blockDim.x >> 6;
    const int nchunk = a.d_model / VEC;
    for (int r = wave; r < rows; r += nwaves) {
        const size_t rowv = (size_t)(j0 + r) * nchunk;
        float ag[MT], au[MT];
#pragma unroll
        for (int m = 0; m < MT; ++m) { ag[m] = 0.f; au[m] = 0.f; }
#pragma unroll 4
        for (int c = lane; c < nchunk; c += 64) {
            float wg[VEC], wu[VEC];
            E::widen(ld16_stream(a.Wg, rowv + c), wg);
            E::widen(ld16_stream(a.Wu, rowv + c), wu);
#pragma unroll
            for (int m = 0; m < MT; ++m) {
                if (m < mt) {
                    float x[VEC];
                    E::widen(ld16(a.X, (size_t)(m0 + m) * nchunk + c), x);
#pragma unroll
                    for (int v = 0; v < VEC; ++v) {
                        ag[m] = fmaf(x[v], wg[v], ag[m]);
                        au[m] = fmaf(x[v], wu[v], au[m]);
                    }
                }
            }
        }
#pragma unroll
        for (int m = 0; m < MT; ++m) {
#pragma unroll
            for (int o = 32; o >= 1; o >>= 1) {
                ag[m] += __shfl_xor(ag[m], o);
                au[m] += __shfl_xor(au[m], o);
            }
            if (lane == 0) a2s[m * a2_stride + r] = (m < mt) ? silu_mul(ag[m], au[m]) : 0.f;
        }
    }
}

// Columns [c_lo, c_hi) (in 16-byte chunks) of the partial Y of rows [j0, j0+rows)
// -> partial block p of the workspace.
template <typename E, int MT>
__device__ __forceinline__ void stage2_valu(const MlpArgs& a, int j0, int rows, int mt, int p,
                                            const float* a2s, int a2_stride, int c_lo, int c_hi) {
    constexpr int VEC = E::VEC;
    const int nchunk = a.d_model / VEC;
    for (int c = c_lo + (int)threadIdx.x; c < c_hi; c += blockDim.x) {
        float acc[MT][VEC];
#pragma unroll
        for (int m = 0; m < MT; ++m)
#pragma unroll
            for (int v = 0; v < VEC; ++v) acc[m][v] = 0.f;
#pragma unroll 8
        for (int j = 0; j < rows; ++j) {
            float w[VEC];
            E::widen(ld16_stream(a.Wd, (size_t)(j0 + j) * nchunk + c), w);
#pragma unroll
            for (int m = 0; m < MT; ++m) {
                const float s = a2s[m * a2_stride + j];
#pragma unroll
                for (int v = 0; v < VEC; ++v) acc[m][v] = fmaf(s, w[v], acc[m][v]);
            }
        }
#pragma unroll
        for (int m = 0; m < MT; ++m) {
            if (m < mt) {
                float* dst = a.P + ((size_t)p * a.m_count + m) * a.d_model + (size_t)c * VEC;
#pragma unroll
                for (int v = 0; v < VEC; v += 4)
                    store4_device(dst + v, acc[m][v], acc[m][v + 1], acc[m][v + 2], acc[m][v + 3]);
            }
        }
    }
}

template <typename E, int MT>
__global__ __launch_bounds__(512) void k_fused_valu(MlpArgs a, int a2_stride) {
    extern __shared__ float a2s[];
    __shared__ int flag;
    int j0, j1;
    slice_rows(a.d_ff, a.splits, blockIdx.x, j0, j1);
    const int rows = j1 - j0;
    const int nchunk = a.d_model / E::VEC;
    stage1_valu<E, MT>(a, j0, rows, a.m_base, a.m_count, a2s, a2_stride);
    __syncthreads();
    stage2_valu<E, MT>(a, j0, rows, a.m_count, blockIdx.x, a2s, a2_stride, 0, nchunk);
    reduce_store<E>(plan_full_width(a, blockIdx.x, a.splits), a.Y, a.m_base, &flag);
}

// First kernel of the two-kernel variant: A_2 slice -> workspace.
template <typename E, int MT>
__global__ __launch_bounds__(512) void k_gateup_valu(MlpArgs a, int a2_stride) {
    extern __shared__ float a2s[];
    int j0, j1;
    slice_rows(a.d_ff, a.splits, blockIdx.x, j0, j1);
    const int rows = j1 - j0;
    stage1_valu<E, MT>(a, j0, rows, a.m_base, a.m_count, a2s, a2_stride);
    __syncthreads();
    for (int i = threadIdx.x; i < a.m_count * rows; i += blockDim.x) {
        const int m = i / rows, r = i - m * rows;
        const size_t o = (size_t)(a.m_base + m) * a.d_ff + j0 + r;
        const float v = a2s[m * a2_stride + r];
        if (a.a2_is_fp32) ((float*)a.a2)[o] = v;
        else ((uint16_t*)a.a2)[o] = (uint16_t)f32_to_bf16_bits(v);
    }
}

// Second kernel: Y = A_2 W_down over a (d_ff split) x (column block) grid.
template <typename E, int MT>
__global__ __launch_bounds__(512) void k_down_valu(MlpArgs a, int a2_stride) {
    extern __shared__ float a2s[];
    __shared__ int flag;
    const int js = blockIdx.x / a.k2_col_blocks;
    const int cb = blockIdx.x - js * a.k2_col_blocks;
    int j0, j1;
    slice_rows(a.d_ff, a.k2_splits, js, j0, j1);
    const int rows = j1 - j0;
    const int nchunk = a.d_model / E::VEC;
    const int c_lo = (int)((long long)nchunk * cb / a.k2_col_blocks);
    const int c_hi = (int)((long long)nchunk * (cb + 1) / a.k2_col_blocks);
    for (int i = threadIdx.x; i < MT * rows; i += blockDim.x) {
        const int m = i / rows, r = i - m * rows;
        float v = 0.f;
        if (m < a.m_count) {
            const size_t o = (size_t)(a.m_base + m) * a.d_ff + j0 + r;
            v = a.a2_is_fp32 ? ((const float*)a.a2)[o]
                             : __uint_as_float((uint32_t)((const uint16_t*)a.a2)[o] << 16);
        }
        a2s[m * a2_stride + r] = v;
    }
    __syncthreads();
    stage2_valu<E, MT>(a, j0, rows, a.m_count, js, a2s, a2_stride, c_lo, c_hi);
    reduce_store<E>(plan_column_block(a, cb, c_lo * E::VEC, c_hi * E::VEC), a.Y, a.m_base, &flag);
}

// Second kernel for W_down given as [d_model, d_ff] (config field kmajor = 5): row n of it is output column n over
// all of d_ff, so each wavefront owns output columns whole, streams their rows with 128-bit loads against A_2 of the
// launch's tokens and stores Y; nothing is summed across workgroups.
template <typename E, int MT>
__global__ __launch_bounds__(512) void k_down_t_valu(MlpArgs a) {
    constexpr int VEC = E::VEC;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int nwaves = blockDim.x >> 6;
    const int nchunk = a.d_ff / VEC;
    for (int n = blockIdx.x * nwaves + wave; n < a.d_model; n += gridDim.x * nwaves) {
        float acc[MT];
#pragma unroll
        for (int m = 0; m < MT; ++m) acc[m] = 0.f;
#pragma unroll 2
        for (int c = lane; c < nchunk; c += 64) {
            float w[VEC];
            E::widen(ld16_stream(a.Wd, (size_t)n * nchunk + c), w);
#pragma unroll
            for (int m = 0; m < MT; ++m) {
                if (m < a.m_count) {
                    const size_t o = (size_t)(a.m_base + m) * a.d_ff + (size_t)c * VEC;
                    float s[VEC];
                    if (a.a2_is_fp32) {
#pragma unroll
                        for (int v = 0; v < VEC; v += 4) {
                            const float4 f = *(const float4*)((const float*)a.a2 + o + v);
                            s[v] = f.x; s[v + 1] = f.y; s[v + 2] = f.z; s[v + 3] = f.w;
                        }
                    } else {     // bf16 A_2 (bf16 inputs only, VEC = 8): one 16-byte load
#pragma unroll
                        for (int v = 0; v < VEC; v += 2) {
                            const uint32_t pk = *(const uint32_t*)((const uint16_t*)a.a2 + o + v);
                            s[v] = bf16_lo(pk); s[v + 1] = bf16_hi(pk);
                        }
                    }
#pragma unroll
                    for (int v = 0; v < VEC; ++v) acc[m] = fmaf(s[v], w[v], acc[m]);
                }
            }
        }
#pragma unroll
        for (int m = 0; m < MT; ++m) {
#pragma unroll
            for (int o = 32; o >= 1; o >>= 1) acc[m] += __shfl_xor(acc[m], o);
            if (lane == 0 && m < a.m_count) E::store(a.Y, (size_t)(a.m_base + m) * a.d_model + n, acc[m]);
        }
    }
}

// smallest token-tile width that holds the launch's tokens (a launch has at most 8)
int pick_mt(int m_count) { return m_count > 4 ? 8 : m_count > 2 ? 4 : m_count > 1 ? 2 : 1; }

template <typename E, int MT>
hipError_t launch_t(const MlpArgs& a, const dfk_config_t& c, hipStream_t st) {
    const int threads = c.waves * 64;
    if (c.variant == DFK_VARIANT_FUSED) {
        if (!(g_stage_mask & 1)) return hipSuccess;
        const int stride = max_slice_rows(a.d_ff, a.splits);
        hipLaunchKernelGGL((k_fused_valu<E, MT>), dim3(a.splits), dim3(threads),
                           (size_t)MT * stride * sizeof(float), st, a, stride);
        return hipGetLastError();
    }
    if (g_stage_mask & 1) {
        const int s1 = max_slice_rows(a.d_ff, a.splits);
        hipLaunchKernelGGL((k_gateup_valu<E, MT>), dim3(a.splits), dim3(threads),
                           (size_t)MT * s1 * sizeof(float), st, a, s1);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (!(g_stage_mask & 2)) return hipSuccess;
    if (c.kmajor == 5) {
        hipLaunchKernelGGL((k_down_t_valu<E, MT>), dim3(a.k2_splits), dim3(threads), 0, st, a);
        return hipGetLastError();
    }
    const int s2 = max_slice_rows(a.d_ff, a.k2_splits);
    hipLaunchKernelGGL((k_down_valu<E, MT>), dim3(a.k2_splits * a.k2_col_blocks), dim3(threads),
                       (size_t)MT * s2 * sizeof(float), st, a, s2);
    return hipGetLastError();
}

template <typename E>
hipError_t launch_e(const MlpArgs& a, const dfk_config_t& c, hipStream_t st) {
    switch (pick_mt(a.m_count)) {
        case 8: return launch_t<E, 8>(a, c, st);
        case 4: return launch_t<E, 4>(a, c, st);
        case 2: return launch_t<E, 2>(a, c, st);
        default: return launch_t<E, 1>(a, c, st);
    }
}

}  // namespace

bool valu_config_valid(const dfk_config_t& c, int M, int d_model, int d_ff, dfk_dtype_t dtype) {
    if (c.path != DFK_PATH_VALU) return false;
    if (c.variant != DFK_VARIANT_FUSED && c.variant != DFK_VARIANT_TWO_KERNEL) return false;
    if (c.kmajor != 0 && !(c.kmajor == 5 && c.variant == DFK_VARIANT_TWO_KERNEL)) return false;   // 5: W_down as [d_model, d_ff]
    if (c.reduce != DFK_REDUCE_TICKET || c.k2_rows_by_wave != 0) return false;
    if (c.waves < 1 || c.waves > 8) return false;  // kernels are built for <= 512 threads
    if (M < 1 || d_model < 8 || d_ff < 8 || d_model % 8 || d_ff % 8) return false;
    const int ng = d_ff / 8;
    if (c.splits < 1 || c.splits > ng) return false;
    const int mt = pick_mt(M);
    const int tokens = M < 8 ? M : 8;
    if ((long long)mt * max_slice_rows(d_ff, c.splits) > kMaxLdsFloats) return false;
    if (c.variant == DFK_VARIANT_FUSED) {
        if ((c.splits + kGroupSize - 1) / kGroupSize > kTicketLevel2) return false;
        if (!partials_fit(c.splits, tokens, M, d_model)) return false;
    }
    if (c.variant == DFK_VARIANT_TWO_KERNEL && c.kmajor == 5) {
        if (c.waves < 1 || c.k2_splits < 1 || c.k2_splits > 65535 || c.k2_col_blocks != 1) return false;
        return c.a2_dtype == DFK_FP32 || (c.a2_dtype == DFK_BF16 && dtype == DFK_BF16);
    }
    if (c.variant == DFK_VARIANT_TWO_KERNEL) {
        if (c.k2_splits < 1 || c.k2_splits > ng) return false;
        const int nchunk = d_model / (dtype == DFK_FP32 ? 4 : 8);
        if (c.k2_col_blocks < 1 || c.k2_col_blocks > nchunk || c.k2_col_blocks > kTicketLevel2) return false;
        if (!partials_fit(c.k2_splits, tokens, M, d_model)) return false;
        if ((long long)c.k2_splits * c.k2_col_blocks > 65535) return false;
        if ((long long)mt * max_slice_rows(d_ff, c.k2_splits) > kMaxLdsFloats) return false;
        // A_2 between the kernels: fp32, or bf16 with bf16 inputs
        if (c.a2_dtype != DFK_FP32 && !(c.a2_dtype == DFK_BF16 && dtype == DFK_BF16)) return false;
    }
    return true;
}

int valu_max_tokens_per_launch() { return 8; }

hipError_t launch_valu(const MlpArgs& a, const dfk_config_t& c, dfk_dtype_t dtype, hipStream_t st) {
    return dtype == DFK_BF16 ? launch_e<BF16>(a, c, st) : dtype == DFK_FP16 ? launch_e<FP16>(a, c, st) : launch_e<FP32>(a, c, st);
}

}  // namespace dfk
