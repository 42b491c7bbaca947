// The deeply fused single launch (Figure 1c; Method, second paragraph) on the k-major stage one of
// the pair for up to 64 tokens per launch: gate/up projection, SiLU (x) up and down projection of
// the whole block in one kernel; A_2 never leaves LDS.  gfx950 only.
//
// Work split ("column-major tiling" of the Method section): workgroup s owns the d_ff slice
// [j0, j1) (at most 8 row tiles of 8 rows) for BOTH stages, so nothing it needs ever comes from
// another workgroup and no workgroup waits for another.
//
// Every wavefront consumes ONE in-order stream of 4 KB tiles through its private LDS ring
// (asynchronous 16-byte global->LDS loads, counted waits): first the stage-one tiles in k-major
// order (per 128-k chunk of the wavefront's k range the X tile, then the weight tile of every row
// tile: 8 rows of W_gate and the same 8 of W_up), then without a gap the stage-two tiles (W_down
// rows of the slice for the wavefront's 128-column blocks), whose addresses do not depend on stage
// one: HBM stays busy across the stage boundary.
//
// Stage boundary: the wavefronts' k-partial sums of G and U meet in a small LDS stage beside the
// rings (not over them: W_down tiles are landing there), one LDS-only barrier, all threads finish
// SiLU(G) * U into A_2 (16-bit, [token][row] in LDS), one more LDS-only barrier.  Stage two:
// wavefront w owns 128-column blocks of d_model; A_2 from LDS is the MFMA A operand, W_down tiles
// are regrouped per lane with v_perm_b32 as in the down kernels.  Rows past the slice in its last
// 32-row block are not fetched at all (those lanes are masked off in the load; the first fused
// kernel fetched whole blocks, 64 rows for a slice of 56).
//
// Reduction over the 256 slices.  A workgroup's result is a partial of ALL of Y, so the partial
// traffic grows with slices x tokens: this form is for the smallest token counts, which is where
// the Method section places deep fusion.  DFK_REDUCE_ATOMIC: every wavefront adds each finished
// [tokens][128] block into the fp32 accumulator with device-wide float atomics while it streams the
// next block; the workgroup counts in once at the end, and the last of the launch turns the
// accumulator into Y.  DFK_REDUCE_TICKET: partial blocks and the two-level fixed-order sum
// (reduce_store), run-to-run bitwise reproducible.
#include <atomic>
#include "dfk_mfma_common.h"

namespace dfk {
namespace {

constexpr int kLocalRowTiles = 8;        // row tiles of a slice (stage-one accumulators)
constexpr int kLocalTokensPerLaunch = 16;
constexpr int kLocalDoneTicket = 1023;   // arrival counter of the atomic mode (word index in the counter area)

struct LocalGeom {
    int depth;
    int stage_off;   // LDS byte offset of the k-partial sums [row tile][wavefront][mp][16] fp32
    int mp;          // tokens the stage holds
    int a2_off;      // LDS byte offset of A_2 [16 tokens][a2_stride] in the 16-bit type
    int a2_stride;   // elements
};

// ---------------------------------------------------------------- the tile stream of a wavefront
template <int NW>
struct LocalStream {
    const char *Wg, *Wu, *Wd, *X;
    unsigned row_bytes;          // d_model * 2
    size_t w_base;               // byte offset of (row j0, this wavefront's first k) in W_gate / W_up
    size_t x_base;               // byte offset of (first token of the launch, this wavefront's first k) in X
    int nt, nkc, m_count;
    int j0, rows, njb;           // the slice; its 32-row blocks
    int blk_first, my_blocks;    // this wavefront's 128-column blocks: blk_first .. blk_first + my_blocks - 1
    int q, g;
    unsigned off1[4], xo[4];
    unsigned char* ring;
    int depth, T1, T, issued, issue_slot, take_slot;
    int p_a, p_b, p_c;           // producer: stage one (chunk, position in chunk); stage two (block, 32-row block, half)

    __device__ __forceinline__ void start() {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int i = 4 * u + g;
            off1[u] = (unsigned)((i & 7) * row_bytes + (q ^ i) * 16);
            xo[u] = (unsigned)(min(i, m_count - 1) * row_bytes + (q ^ i) * 16);
        }
        T1 = nkc * (1 + nt);
        T = T1 + my_blocks * njb * 2;
        issued = 0; issue_slot = 0; take_slot = 0; p_a = 0; p_b = 0; p_c = 0;
        const int ahead = min(depth - 1, T);
        for (int i = 0; i < ahead; ++i) issue();
    }
    __device__ __forceinline__ void issue() {
        unsigned char* slot = ring + issue_slot * kTileBytes;
        if (issued < T1) {
            if (p_b == 0) {        // X tile of chunk p_a: 16 tokens x 128 k
                const char* xb = X + x_base + (size_t)p_a * (kKC * 2);
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    __builtin_amdgcn_global_load_lds(xb + xo[u], DFK_LDS_PTR(slot + u * 1024), 16, 0, 0);
            } else {               // weight tile of row tile p_b - 1
                const size_t tb = w_base + (size_t)(p_b - 1) * 8 * row_bytes + (size_t)p_a * (kKC * 2);
                const char* gb = Wg + tb;
                const char* ub = Wu + tb;
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    __builtin_amdgcn_global_load_lds((u < 2 ? gb : ub) + off1[u], DFK_LDS_PTR(slot + u * 1024), 16, 0,
                                                     kAuxNonTemporal);
            }
            if (++p_b == 1 + nt) { p_b = 0; ++p_a; }
            if (issued + 1 == T1) { p_a = 0; p_b = 0; p_c = 0; }
        } else {                   // W_down: column block p_a of this wavefront, 32-row block p_b, half p_c
            const int r0 = p_b * 32 + 4 * p_c;                       // lane adds 8g + u
            const char* base = Wd + (size_t)(j0 + r0) * row_bytes + (size_t)(blk_first + p_a) * 256 + 16 * q;
            // rows past the slice are not fetched: their lanes are masked off (the slot keeps stale bytes there,
            // which the consumer replaces by zeros)
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (r0 + 8 * g + u < rows)
                    __builtin_amdgcn_global_load_lds(base + (size_t)(8 * g + u) * row_bytes, DFK_LDS_PTR(slot + u * 1024), 16, 0,
                                                     kAuxNonTemporal);
            if (++p_c == 2) { p_c = 0; if (++p_b == njb) { p_b = 0; ++p_a; } }
        }
        ++issued;
        if (++issue_slot == depth) issue_slot = 0;
    }
    __device__ __forceinline__ const unsigned char* acquire() {
        DFK_WAIT_LGKM0();   // reads of the slot about to be refilled have returned
        asm volatile("" ::: "memory");
        if (issued < T) {
            issue();
            wait_vm_ops(4 * (depth - 1));
        } else {
            wait_vm_ops(0);
        }
        const unsigned char* slot = ring + take_slot * kTileBytes;
        if (++take_slot == depth) take_slot = 0;
        return slot;
    }
};

template <int NW, typename E>
__global__ __launch_bounds__(NW * 64) void k_fused_local(MlpArgs a, LocalGeom geo) {
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    __shared__ int flag;
    constexpr int NTHREADS = NW * 64;
    constexpr int NT = kLocalRowTiles;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int q = lane & 15, g = lane >> 4;
    int j0, j1;
    slice_rows(a.d_ff, a.splits, blockIdx.x, j0, j1);
    const int rows = j1 - j0;
    const int nt = rows / 8;                              // <= NT, checked on the host
    const int njb = (rows + 31) / 32;
    const int nchunks = a.d_model / kKC;
    const int c0 = wave * nchunks / NW, c1 = (wave + 1) * nchunks / NW;
    const int nblk = a.d_model / 128;
    const int b0 = wave * nblk / NW, b1 = (wave + 1) * nblk / NW;
    const bool atomic_mode = a.reduce_mode == DFK_REDUCE_ATOMIC;
    const int MP = geo.mp;
    const unsigned stage_addr = lds_addr(lds + geo.stage_off);
    const float* stage = (const float*)(lds + geo.stage_off);
    const unsigned a2_addr = lds_addr(lds + geo.a2_off);
    const uint16_t* a2s = (const uint16_t*)(lds + geo.a2_off);
    const int a2_stride = geo.a2_stride;

    LocalStream<NW> ts;
    ts.Wg = (const char*)a.Wg; ts.Wu = (const char*)a.Wu; ts.Wd = (const char*)a.Wd; ts.X = (const char*)a.X;
    ts.row_bytes = (unsigned)a.d_model * 2u;
    ts.w_base = (size_t)j0 * ts.row_bytes + (size_t)c0 * (kKC * 2);
    ts.x_base = (size_t)a.m_base * ts.row_bytes + (size_t)c0 * (kKC * 2);
    ts.nt = nt; ts.nkc = c1 - c0; ts.m_count = a.m_count;
    ts.j0 = j0; ts.rows = rows; ts.njb = njb;
    ts.blk_first = b0; ts.my_blocks = b1 - b0;
    ts.q = q; ts.g = g;
    ts.ring = lds + wave * geo.depth * kTileBytes;
    ts.depth = geo.depth;
    DFK_STAMP(0);
    ts.start();                                          // the stream starts first: nothing it needs depends on LDS contents

    // A_2 rows past the slice (up to the next multiple of 32) must read as zero: clear the whole array once.
    for (int i = tid; i < 16 * a2_stride / 2; i += NTHREADS) lds_write_b32_raw(a2_addr + 4u * (unsigned)i, 0u);

    // ---- stage one: every row tile accumulates over this wavefront's k range
    {
        f32x4 acc[NT];
#pragma unroll
        for (int rt = 0; rt < NT; ++rt) acc[rt] = f32x4{0.f, 0.f, 0.f, 0.f};
        for (int kc = 0; kc < ts.nkc; ++kc) {
            u32x4 xk[4];
            {
                const unsigned char* slot = ts.acquire();
#pragma unroll
                for (int c = 0; c < 4; ++c) xk[c] = *(const u32x4*)(slot + (q * 16 + ((4 * c + g) ^ q)) * 16);
            }
#pragma unroll
            for (int rt = 0; rt < NT; ++rt) {
                if (rt < nt) {
                    const unsigned char* slot = ts.acquire();
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        const u32x4 av = *(const u32x4*)(slot + (q * 16 + ((4 * c + g) ^ q)) * 16);
                        acc[rt] = mfma16<E>(av, xk[c], acc[rt]);
                    }
                }
            }
        }
        DFK_STAMP(2);
        // the wavefronts' k-partial sums meet in LDS: [row tile][wavefront][token][16 rows]
#pragma unroll
        for (int rt = 0; rt < NT; ++rt) {
            if (rt < nt) {
                asm volatile("s_nop 7\n\ts_nop 7\n\ts_nop 7" : "+v"(acc[rt]));   // MFMA result -> LDS store wait states
                if (q < MP) lds_write_b128_raw(stage_addr + 4u * (unsigned)((((rt * NW + wave) * MP + q) * 16) + 4 * g), acc[rt]);
            }
        }
    }
    lds_barrier();
    // A_2[m, j] = SiLU(G) * U, wavefronts' blocks added in wavefront order; task (row tile r, token m, row pair pr)
    for (int t = tid; t < nt * a.m_count * 4; t += NTHREADS) {
        const int r = t / (a.m_count * 4), rem = t - r * (a.m_count * 4);
        const int m = rem >> 2, pr = rem & 3;
        const float* src = stage + ((size_t)(r * NW) * MP + m) * 16 + 2 * pr;
        float g0 = 0.f, g1 = 0.f, u0 = 0.f, u1 = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            const float2 gv = *(const float2*)(src + (size_t)w * MP * 16);
            const float2 uv = *(const float2*)(src + (size_t)w * MP * 16 + 8);
            g0 += gv.x; g1 += gv.y; u0 += uv.x; u1 += uv.y;
        }
        lds_write_b32_raw(a2_addr + 2u * (unsigned)(m * a2_stride + r * 8 + 2 * pr),
                          E::pack2(silu_mul_fast(g0, u0), silu_mul_fast(g1, u1)));
    }
    lds_barrier();
    DFK_STAMP(3);

    // ---- stage two: this wavefront's column blocks, one after the other
    const int pblk = (int)blockIdx.x;
    for (int bi = 0; bi < ts.my_blocks; ++bi) {
        f32x4 acc2[8];
#pragma unroll
        for (int c = 0; c < 8; ++c) acc2[c] = f32x4{0.f, 0.f, 0.f, 0.f};
        for (int jb = 0; jb < njb; ++jb) {
            u32x4 w[8];
            const unsigned char* sa = ts.acquire();
#pragma unroll
            for (int u = 0; u < 4; ++u) w[u] = *(const u32x4*)(sa + u * 1024 + lane * 16);
            const unsigned char* sb = ts.acquire();
#pragma unroll
            for (int u = 0; u < 4; ++u) w[4 + u] = *(const u32x4*)(sb + u * 1024 + lane * 16);
            if (jb * 32 + 32 > rows) {   // rows past the slice were not fetched
#pragma unroll
                for (int r = 0; r < 8; ++r)
                    if (jb * 32 + 8 * g + r >= rows) w[r] = u32x4{0, 0, 0, 0};
            }
            const u32x4 av = *(const u32x4*)(a2s + q * a2_stride + jb * 32 + 8 * g);
#pragma unroll
            for (int c = 0; c < 8; ++c) {
                const uint32_t sel = (c & 1) ? 0x07060302u : 0x05040100u;
                u32x4 bb;
#pragma unroll
                for (int p = 0; p < 4; ++p) bb[p] = __builtin_amdgcn_perm(w[2 * p + 1][c >> 1], w[2 * p][c >> 1], sel);
                acc2[c] = mfma16<E>(av, bb, acc2[c]);
            }
        }
        // the finished [tokens][128] block leaves the wavefront: lane (q, g) holds tokens 4g+i, columns 8q .. 8q+7
        const int nb = (b0 + bi) * 128;
        if (atomic_mode) {
            // Regrouped through lane permutes so that one atomic instruction covers 64 consecutive floats of one
            // token (lane L adds columns nb+L and nb+64+L): in the MFMA layout an instruction touches 16 separate
            // 32-byte pieces and the adds run an order of magnitude slower.
            for (int token = 0; token < a.m_count; ++token) {
                const int gsrc = token >> 2, i = token & 3;
                float lo = 0.f, hi = 0.f;
#pragma unroll
                for (int c = 0; c < 8; ++c) {
                    const float v = i == 0 ? acc2[c][0] : i == 1 ? acc2[c][1] : i == 2 ? acc2[c][2] : acc2[c][3];
                    const float va = __shfl(v, 16 * gsrc + (lane >> 3));
                    const float vb = __shfl(v, 16 * gsrc + 8 + (lane >> 3));
                    if ((lane & 7) == c) { lo = va; hi = vb; }
                }
                float* dst = a.yacc + (size_t)token * a.d_model + nb + lane;
                acc_add(dst, lo);
                acc_add(dst + 64, hi);
            }
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int token = 4 * g + i;
                if (token < a.m_count) {
                    float* dst = a.P + ((size_t)pblk * a.m_count + token) * a.d_model + nb + 8 * q;
                    store4_device(dst, acc2[0][i], acc2[1][i], acc2[2][i], acc2[3][i]);
                    store4_device(dst + 4, acc2[4][i], acc2[5][i], acc2[6][i], acc2[7][i]);
                }
            }
        }
    }
    DFK_STAMP(4);

    // ---- reduction over the slices and the store of Y
    if (!atomic_mode) {
        reduce_store<E>(plan_full_width(a, blockIdx.x, a.splits), a.Y, a.m_base, &flag, a.trace);
        return;
    }
    drain_own_memory_ops();                                // this wavefront's adds have been performed
    __syncthreads();
    DFK_STAMP(5);
    if (tid == 0) flag = arrive_last(a.tickets + kLocalDoneTicket, gridDim.x) ? 1 : 0;
    __syncthreads();
    DFK_STAMP(6);
    if (!flag) return;
    for (int idx = tid; idx < a.m_count * (a.d_model / 2); idx += NTHREADS) {
        const int m = idx / (a.d_model / 2), c2 = idx - m * (a.d_model / 2);
        float* src = a.yacc + (size_t)m * a.d_model + 2 * c2;
        const float v0 = acc_take(src), v1 = acc_take(src + 1);
        *(uint32_t*)((uint16_t*)a.Y + (size_t)(a.m_base + m) * a.d_model + 2 * c2) = E::pack2(v0, v1);
    }
    DFK_STAMP(7);
}

// ---------------------------------------------------------------- host side
size_t local_lds(const dfk_config_t& c, int m_count, int d_ff, LocalGeom* geo) {
    const int nt_max = max_slice_rows(d_ff, c.splits) / 8;
    const size_t ring = (size_t)c.waves * c.depth * kTileBytes;
    geo->depth = c.depth;
    geo->mp = std::min(16, m_count);
    geo->stage_off = (int)ring;
    const size_t stage = (size_t)nt_max * c.waves * geo->mp * 16 * 4;
    geo->a2_off = (int)(ring + stage);
    geo->a2_stride = ((nt_max * 8 + 31) & ~31) + 8;      // whole 32-row blocks, padded against bank conflicts
    return ring + stage + (size_t)16 * geo->a2_stride * 2;
}

template <int NW, typename E>
hipError_t launch_local_e(const MlpArgs& a, const dfk_config_t& c, hipStream_t st) {
    static LdsAllowance allowed;
    if (!(g_stage_mask & 1)) return hipSuccess;
    LocalGeom geo;
    const size_t lds = local_lds(c, a.m_count, a.d_ff, &geo);
    if (hipError_t e = allow_lds(allowed, (const void*)k_fused_local<NW, E>, lds); e != hipSuccess) return e;
    hipLaunchKernelGGL((k_fused_local<NW, E>), dim3(a.splits), dim3(NW * 64), lds, st, a, geo);
    return hipGetLastError();
}

}  // namespace

int mfma_fused_km_tokens_per_launch() { return kLocalTokensPerLaunch; }

bool mfma_fused_km_config_valid(const dfk_config_t& c, int M, int d_model, int d_ff, dfk_dtype_t dtype) {
    if (c.path != DFK_PATH_MFMA || (dtype != DFK_BF16 && dtype != DFK_FP16) || c.variant != DFK_VARIANT_FUSED) return false;
    if (c.kmajor != 1 || c.k2_rows_by_wave != 0) return false;
    if (c.reduce != DFK_REDUCE_TICKET && c.reduce != DFK_REDUCE_ATOMIC) return false;
    if ((c.waves != 4 && c.waves != 8) || c.depth < 2 || c.depth > 16) return false;
    if (M < 1 || d_model < 8 || d_ff < 8 || d_ff % 8 || d_model > kMaxDModel) return false;
    if (d_model % kKC || d_model / kKC < c.waves) return false;    // every wavefront owns whole 128-k chunks and column blocks
    const int G = d_ff / 8;
    if (c.splits < 1 || c.splits > G || c.splits > 65535) return false;
    if (max_slice_rows(d_ff, c.splits) / 8 > kLocalRowTiles) return false;   // stage-one accumulators
    const int tokens = std::min(M, kLocalTokensPerLaunch);
    if (c.reduce == DFK_REDUCE_TICKET &&
        ((c.splits + kGroupSize - 1) / kGroupSize > kTicketLevel2 - 1 || !partials_fit(c.splits, tokens, M, d_model)))
        return false;
    if (c.reduce == DFK_REDUCE_ATOMIC && (size_t)tokens * d_model * 4 > kYaccBytes) return false;
    LocalGeom geo;
    return local_lds(c, tokens, d_ff, &geo) <= (size_t)kLdsLimit;
}

hipError_t launch_mfma_fused_km(const MlpArgs& a, const dfk_config_t& c, hipStream_t st) {
    if (c.waves == 8) return a.dtype == DFK_FP16 ? launch_local_e<8, FP16>(a, c, st) : launch_local_e<8, BF16>(a, c, st);
    if (c.waves == 4) return a.dtype == DFK_FP16 ? launch_local_e<4, FP16>(a, c, st) : launch_local_e<4, BF16>(a, c, st);
    return hipErrorInvalidValue;
}

}  // namespace dfk
