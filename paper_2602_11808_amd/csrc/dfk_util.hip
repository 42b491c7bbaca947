// Utility kernels: workspace zeroing, synthetic fill, and the read-stream probe.
#include "dfk_device.h"
#include "dfk_internal.h"

namespace dfk {
namespace {

__global__ void k_zero(u32x4* p, size_t n16, unsigned char* tail, size_t ntail) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride)
        p[i] = u32x4{0, 0, 0, 0};
    if (blockIdx.x == 0 && threadIdx.x < ntail) tail[threadIdx.x] = 0;
}

__device__ __forceinline__ uint32_t mix32(uint32_t x) {
    x ^= x >> 16; x *= 0x7FEB352Du;
    x ^= x >> 15; x *= 0x846CA68Bu;
    x ^= x >> 16;
    return x;
}

__global__ void k_fill(void* dst, size_t n, int dtype, float scale, uint32_t seed) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        const uint32_t h = mix32((uint32_t)i * 0x9E3779B9u + mix32(seed + (uint32_t)(i >> 32)));
        const float u = ((float)(h >> 8) * (1.0f / 8388608.0f) - 1.0f) * scale;  // (-scale, scale)
        if (dtype == DFK_FP32) ((float*)dst)[i] = u;
        else if (dtype == DFK_FP16) FP16::store(dst, i, u);
        else ((uint16_t*)dst)[i] = (uint16_t)f32_to_bf16_bits(u);
    }
}

constexpr int kReadThreads = 256;
constexpr int kReadUnroll = 8;

__global__ __launch_bounds__(kReadThreads) void k_stream_read(const u32x4* __restrict__ src, size_t n16,
                                                              unsigned* sink) {
    const size_t tile = (size_t)kReadThreads * kReadUnroll;
    const size_t full = n16 / tile;
    u32x4 acc = {0, 0, 0, 0};
    // whole tiles: kReadUnroll independent 16-byte loads per lane in flight, no bounds checks
    for (size_t t = blockIdx.x; t < full; t += gridDim.x) {
        const u32x4* p = src + t * tile + threadIdx.x;
        u32x4 v[kReadUnroll];
#pragma unroll
        for (int u = 0; u < kReadUnroll; ++u) v[u] = __builtin_nontemporal_load(p + (size_t)u * kReadThreads);
#pragma unroll
        for (int u = 0; u < kReadUnroll; ++u) acc ^= v[u];
    }
    // ragged tail
    for (size_t i = full * tile + (size_t)blockIdx.x * kReadThreads + threadIdx.x; i < n16;
         i += (size_t)gridDim.x * kReadThreads)
        acc ^= src[i];
    // Keep the loads alive without a contended atomic: the fold is compared with a
    // value it practically never takes.
    const unsigned a = acc.x ^ acc.z, b = acc.y ^ acc.w;
    if (a == 0x9E3779B9u && b == 0x7F4A7C15u) sink[0] = 1u;
}

// out[m,:] = in[m,:] / rms(in[m,:]) in bf16 (fp32 arithmetic), one workgroup per token.
// Keeps chained random layers from shrinking the activations to zero in benchmarks.
// in and out may be the same buffer (no restrict): each element is read twice, then written, by one thread.
__global__ __launch_bounds__(256) void k_rms_normalize(const uint16_t* in, uint16_t* out, int d_model) {
    __shared__ float part[4];
    const uint16_t* x = in + (size_t)blockIdx.x * d_model;
    uint16_t* y = out + (size_t)blockIdx.x * d_model;
    float s = 0.f;
    for (int i = threadIdx.x; i < d_model; i += 256) {
        const float v = __uint_as_float((uint32_t)x[i] << 16);
        s += v * v;
    }
    for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = s;
    __syncthreads();
    const float scale = rsqrtf((part[0] + part[1] + part[2] + part[3]) / (float)d_model + 1e-12f);
    for (int i = threadIdx.x; i < d_model; i += 256)
        y[i] = (uint16_t)f32_to_bf16_bits(__uint_as_float((uint32_t)x[i] << 16) * scale);
}

// out[m,:] = round16(in[m,:] * w * rsqrt(mean(in[m,:]^2) + eps)), 16-bit element type E, fp32 arithmetic;
// one workgroup per token, 16-byte accesses.  The normalisation ahead of the 256-token kernel pair in
// dfk_mlp_block (there the in-kernel form costs more than this pass).
template <typename E>
__global__ __launch_bounds__(256) void k_rmsnorm_weighted(const void* __restrict__ in, const void* __restrict__ w,
                                                          void* __restrict__ out, int d_model, float eps) {
    __shared__ float part[4];
    const u32x4* x = (const u32x4*)((const uint16_t*)in + (size_t)blockIdx.x * d_model);
    const u32x4* wv = (const u32x4*)w;
    u32x4* y = (u32x4*)((uint16_t*)out + (size_t)blockIdx.x * d_model);
    const int nv = d_model / 8;
    float s = 0.f;
    for (int i = threadIdx.x; i < nv; i += 256) {
        float f[8];
        E::widen(x[i], f);
#pragma unroll
        for (int k = 0; k < 8; ++k) s = fmaf(f[k], f[k], s);
    }
    for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = s;
    __syncthreads();
    const float scale = __builtin_amdgcn_rsqf((part[0] + part[1] + part[2] + part[3]) / (float)d_model + eps);
    for (int i = threadIdx.x; i < nv; i += 256) {
        float f[8], g[8];
        E::widen(x[i], f);
        E::widen(wv[i], g);
        u32x4 o;
#pragma unroll
        for (int k = 0; k < 4; ++k) o[k] = E::pack2(f[2 * k] * g[2 * k] * scale, f[2 * k + 1] * g[2 * k + 1] * scale);
        y[i] = o;
    }
}

// out[c][r] = in[r][c] for a [rows][cols] matrix of 16- or 32-bit elements: 32 x 32 tiles through LDS (padded
// against bank conflicts), reads and writes both along rows.
template <typename T>
__global__ __launch_bounds__(256) void k_transpose(const T* in, T* out, int rows, int cols) {
    __shared__ T tile[32][33];
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;   // 32 x 8 threads
    const int c0 = blockIdx.x * 32, r0 = blockIdx.y * 32;
    for (int i = ty; i < 32; i += 8)
        if (r0 + i < rows && c0 + tx < cols) tile[i][tx] = in[(size_t)(r0 + i) * cols + c0 + tx];
    __syncthreads();
    for (int i = ty; i < 32; i += 8)
        if (c0 + i < cols && r0 + tx < rows) out[(size_t)(c0 + i) * rows + r0 + tx] = tile[tx][i];
}

}  // namespace

hipError_t launch_transpose(const void* in, void* out, int rows, int cols, dfk_dtype_t dtype, hipStream_t st) {
    const dim3 grid((unsigned)((cols + 31) / 32), (unsigned)((rows + 31) / 32));
    if (dtype == DFK_FP32)
        hipLaunchKernelGGL(k_transpose<uint32_t>, grid, dim3(256), 0, st, (const uint32_t*)in, (uint32_t*)out, rows, cols);
    else
        hipLaunchKernelGGL(k_transpose<uint16_t>, grid, dim3(256), 0, st, (const uint16_t*)in, (uint16_t*)out, rows, cols);
    return hipGetLastError();
}

hipError_t launch_rmsnorm_weighted(const void* in, const void* w, void* out, int M, int d_model, float eps, dfk_dtype_t dtype,
                                   hipStream_t st) {
    if (dtype == DFK_FP16)
        hipLaunchKernelGGL(k_rmsnorm_weighted<FP16>, dim3((unsigned)M), dim3(256), 0, st, in, w, out, d_model, eps);
    else
        hipLaunchKernelGGL(k_rmsnorm_weighted<BF16>, dim3((unsigned)M), dim3(256), 0, st, in, w, out, d_model, eps);
    return hipGetLastError();
}

hipError_t launch_zero(void* p, size_t bytes, hipStream_t st) {
    const size_t n16 = bytes / 16, ntail = bytes % 16;
    size_t blocks = (n16 + 255) / 256;
    if (blocks < 1) blocks = 1;
    if (blocks > 2048) blocks = 2048;
    hipLaunchKernelGGL(k_zero, dim3((unsigned)blocks), dim3(256), 0, st, (u32x4*)p, n16,
                       (unsigned char*)p + n16 * 16, ntail);
    return hipGetLastError();
}

hipError_t launch_fill(void* dst, size_t elems, dfk_dtype_t dtype, float scale, unsigned seed,
                       hipStream_t st) {
    size_t blocks = (elems + 255) / 256;
    if (blocks < 1) blocks = 1;
    if (blocks > 8192) blocks = 8192;
    hipLaunchKernelGGL(k_fill, dim3((unsigned)blocks), dim3(256), 0, st, dst, elems,
                       (int)dtype, scale, seed);
    return hipGetLastError();
}

hipError_t launch_rms_normalize(const void* in, void* out, int M, int d_model, hipStream_t st) {
    hipLaunchKernelGGL(k_rms_normalize, dim3((unsigned)M), dim3(256), 0, st, (const uint16_t*)in, (uint16_t*)out, d_model);
    return hipGetLastError();
}

// Reads W_gate and W_up the way the gate/up kernel for up to 64 tokens does, and nothing else:
// workgroup s takes the d_ff slice s of both matrices, wavefront w the k range w of every row,
// a load instruction covers 4 rows x 256 bytes (one quarter of a 16-row x 128-k tile; rows 0..7
// of a tile from W_gate, 8..15 the same rows of W_up), the tiles are walked k chunk by k chunk
// over all row tiles of the slice, 16 instructions (4 tiles) in flight per wavefront.  No X, no
// MFMA, no LDS, no stores: what is left is the memory pattern's own time.
template <int NW>
__global__ __launch_bounds__(NW * 64) void k_read_gateup_pattern(const char* __restrict__ Wg, const char* __restrict__ Wu,
                                                                  int d_model, int d_ff, int splits, unsigned* sink) {
    constexpr int kInFlight = 16;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int j0, j1;
    slice_rows(d_ff, splits, blockIdx.x, j0, j1);
    const int nt = (j1 - j0) / 8;                       // row tiles of 8 rows of each matrix
    const size_t row_bytes = (size_t)d_model * 2;
    const int kw_bytes = d_model * 2 / NW;              // this wavefront's bytes of every row
    const int nkc = kw_bytes / 256;
    const size_t base = (size_t)j0 * row_bytes + (size_t)wave * kw_bytes + (size_t)(lane & 15) * 16;
    const int tiles = nkc * nt;                         // 16-row x 128-k tiles of this wavefront, k chunk by k chunk
    const char* gl = Wg + base + (size_t)(lane >> 4) * row_bytes;   // this lane in rows 0..3 of the slice
    const char* ul = Wu + base + (size_t)(lane >> 4) * row_bytes;
    u32x4 acc = {0, 0, 0, 0};
    int kc = 0, rt = 0;                                 // (wave-uniform counters: no division per load)
    for (int t0 = 0; t0 < tiles; t0 += kInFlight / 4) {
        u32x4 v[kInFlight];
#pragma unroll
        for (int t = 0; t < kInFlight / 4; ++t) {
            const size_t off = (size_t)rt * 8 * row_bytes + (size_t)kc * 256;
            v[4 * t + 0] = __builtin_nontemporal_load((const u32x4*)(gl + off));
            v[4 * t + 1] = __builtin_nontemporal_load((const u32x4*)(gl + off + 4 * row_bytes));
            v[4 * t + 2] = __builtin_nontemporal_load((const u32x4*)(ul + off));
            v[4 * t + 3] = __builtin_nontemporal_load((const u32x4*)(ul + off + 4 * row_bytes));
            if (t0 + t + 1 < tiles) {                   // past the last tile: it is read again
                if (++rt == nt) { rt = 0; ++kc; }
            }
        }
#pragma unroll
        for (int u = 0; u < kInFlight; ++u) acc ^= v[u];
    }
    const unsigned a = acc.x ^ acc.z, b = acc.y ^ acc.w;
    if (a == 0x9E3779B9u && b == 0x7F4A7C15u) sink[0] = 1u;
}

hipError_t launch_read_gateup_pattern(const void* Wg, const void* Wu, int d_model, int d_ff, int splits, int waves,
                                      void* sink, hipStream_t st) {
    if (waves == 8)
        hipLaunchKernelGGL(k_read_gateup_pattern<8>, dim3(splits), dim3(512), 0, st, (const char*)Wg, (const char*)Wu,
                           d_model, d_ff, splits, (unsigned*)sink);
    else
        hipLaunchKernelGGL(k_read_gateup_pattern<4>, dim3(splits), dim3(256), 0, st, (const char*)Wg, (const char*)Wu,
                           d_model, d_ff, splits, (unsigned*)sink);
    return hipGetLastError();
}

hipError_t launch_stream_read(const void* src, size_t bytes, void* sink, hipStream_t st) {
    const size_t n16 = bytes / 16;
    const size_t tile = (size_t)kReadThreads * kReadUnroll;
    size_t blocks = (n16 + tile - 1) / tile;
    if (blocks < 1) blocks = 1;
    if (blocks > 256 * 8) blocks = 256 * 8;
    hipLaunchKernelGGL(k_stream_read, dim3((unsigned)blocks), dim3(kReadThreads), 0, st,
                       (const u32x4*)src, n16, (unsigned*)sink);
    return hipGetLastError();
}

}  // namespace dfk
