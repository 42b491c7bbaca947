// MFMA kernels of the two-kernel variant for up to 64 tokens per launch (gfx950).
//
// The kernels of dfk_mfma.hip keep the activations a wavefront needs (its k range
// of X; A_2 for its rows) in registers for the whole launch, which caps a launch at
// 32 tokens; more tokens mean further launches that stream the weights again.  Here
// the activations ride the same per-wavefront LDS ring as the weight tiles, 4 KB
// tiles fetched by the same asynchronous global->LDS loads in one in-order stream,
// so their register cost is one tile at a time and a launch takes up to 4 token tiles of
// 16 ("row-major" end of the Method section's tiling choice: X stays local while
// more of it is reused per weight tile).
//
// Gate/up kernel (A_2 = (X W_up) (x) SiLU(X W_gate), same split as before: workgroup s
// owns a d_ff slice of at most 8 row tiles of 8 rows, wavefront w a contiguous run of the
// 128-k chunks of every row).  The stream is k-major: for every 128-k chunk first the X tiles
// (16 tokens x 128 k each, same shape and swizzle as a weight tile; they become the
// MFMA B operand registers of the chunk), then the weight tile of every row tile.
// All row tiles accumulate in registers until the stream ends; the wavefronts' sums
// then meet in LDS (over the drained rings, a few row tiles per pass) and all
// threads of the workgroup finish SiLU(G)*U and store A_2 to the workspace.
//
// Down kernel (Y = A_2 W_down): workgroup (js, cb) owns CB adjacent 128-column blocks
// over d_ff split js, its wavefronts divide the split's 32-row blocks.  Per pair of 32-row
// blocks the stream holds the A_2 tiles (64 rows x 32 tokens: whole 128-byte lines per token;
// [token][8 rows] per lane is the MFMA A operand) and then two W_down tiles per block and
// column block, regrouped per lane with v_perm_b32.
// The end (per-wavefront LDS stages, ticket or atomic reduction) is that of
// k_down_rows, one token tile at a time.
//
// Rows of X / A_2 past the launch's tokens are fetched from the last real token:
// they only feed output rows that are never stored.
#include <atomic>
#include <cstdlib>
#include "dfk_mfma_common.h"

namespace dfk {
namespace {

constexpr int kKmMaxRowTiles = 8;   // row tiles per workgroup of the gate/up kernel (accumulators)
constexpr int kKmTokensPerLaunch = 64;

struct KmGeom {
    int depth;   // ring slots per wavefront
    int pass;    // gate/up kernel: row tiles whose partial sums LDS holds per pass at the end
    int norm_off;  // gate/up kernel with the normalisation: byte offset in LDS of the weight slices, past rings and stage
    // the single launch of both kernels' workgroups:
    int n_gateup;            // workgroups of the gate/up kernel at the head of the grid
    int role_publish;        // gate/up workgroups count themselves done
    int role_wait;           // down workgroups wait for the gate/up workgroups of their rows
    int role_stride;         // words between the counters of adjacent d_ff splits
    int depth_down;          // ring slots per wavefront of the down workgroups
    int role_spin_limit;     // polls of the done counter before a down workgroup gives up (its outputs become NaN)
};

// Counter words of the single launch of both kernels' workgroups, in the counter area of the workspace (column
// block counters occupy [0, 512), the second reduction level word 512, the slice-local fused kernel word 1023).
constexpr int kRolePassed = 1022;   // down workgroups that are past their wait: the last one clears the counters below
constexpr int kRoleCount0 = 520;    // per d_ff split of the down projection: gate/up workgroups that have published
constexpr int kRoleCountEnd = 1020; //   A_2 rows of that split; geo.role_stride words apart (spread over cache lines)

// the slice (of S) that holds 8-row group gidx of ng: the inverse of slice_rows
__device__ __forceinline__ int slice_of_group(int ng, int S, int gidx) { return (int)((((long long)gidx + 1) * S - 1) / ng); }

// Bytes between the wavefronts' slices of the normalisation weight in LDS: the longest run of
// chunks a wavefront can own, 1 KB-aligned (one load instruction writes 1 KB).
__host__ __device__ inline int km_norm_stride(int d_model, int waves) {
    const int nchunks = d_model / kKC;
    return (((nchunks + waves - 1) / waves) * (kKC * 2) + 1023) & ~1023;
}

// ---------------------------------------------------------------- gate/up kernel
template <int NW, int TT>
struct KmStream1 {
    const char *Wg, *Wu, *X;
    size_t row_bytes;          // d_model * 2
    size_t w_base;             // byte offset of (row j0, this wavefront's first k)
    size_t x_base;             // byte offset of (token m_base, this wavefront's first k)
    int nt, nkc, m_count;
    int tile_rows;             // weight rows between consecutive row tiles (8: gate and up rows side by side; 16: one matrix)
    int q, g;
    unsigned off1[4];
    unsigned char* ring;
    int depth, T, issued, issue_slot, take_slot;
    int p_kc, p_idx;           // producer: chunk, position in the chunk (X tiles, then row tiles)

    __device__ __forceinline__ void issue() {
        unsigned char* slot = ring + issue_slot * kTileBytes;
        if (p_idx < TT) {      // X tile: lane (q, g), instruction u -> token row 4u+g, chunk q ^ row
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int i = 4 * u + g;
                const int token = min(p_idx * 16 + i, m_count - 1);
                const char* src = X + x_base + (size_t)token * row_bytes + (size_t)p_kc * (kKC * 2) + ((q ^ i) * 16);
                __builtin_amdgcn_global_load_lds(src, DFK_LDS_PTR(slot + u * 1024), 16, 0, 0);
            }
        } else {               // weight tile of row tile p_idx - TT: 8 rows of W_gate, the same 8 of W_up
            const size_t tb = w_base + (size_t)(p_idx - TT) * tile_rows * row_bytes + (size_t)p_kc * (kKC * 2);
            const char* gb = Wg + tb;
            const char* ub = Wu + tb;
#pragma unroll
            for (int u = 0; u < 4; ++u)
                __builtin_amdgcn_global_load_lds((u < 2 ? gb : ub) + off1[u], DFK_LDS_PTR(slot + u * 1024), 16, 0,
                                                 kAuxNonTemporal);
        }
        if (++p_idx == TT + nt) { p_idx = 0; ++p_kc; }
        ++issued;
        if (++issue_slot == depth) issue_slot = 0;
    }
    __device__ __forceinline__ void start() {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int i = 4 * u + g;
            off1[u] = (unsigned)((i & 7) * row_bytes + (q ^ i) * 16);
        }
        T = nkc * (TT + nt);
        issued = 0; issue_slot = 0; take_slot = 0; p_kc = 0; p_idx = 0;
        const int ahead = min(depth - 1, T);
        for (int i = 0; i < ahead; ++i) issue();
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

// NORM: X is the un-normalised residual stream H and the kernel computes the gate/up sums of
// RMSNorm(H; w, eps) = H (x) w * s_m, s_m = 1/sqrt(mean_k H[m,k]^2 + eps).  The per-token
// scalar s_m factors out of both sums, so the B operand becomes round16(H[m,k] * w[k])
// (one rounding to the 16-bit type, as a separate normalisation kernel's store would do),
// every lane adds up the squares of the H values it holds anyway, and the end scales the
// summed G and U by s_m in fp32 before the activation.  Each workgroup reads all of X, so
// it has the whole sum of squares of every token by itself.
//
// PUBLISH (the single launch that holds both kernels' workgroups, further down): A_2 is stored
// with device-scope stores and the workgroup ends by counting itself done on kRoleDone.
//
// DOWN_T: the same stream and accumulation computes the down projection from W_down given as [d_model, d_ff]
// (a linear layer's own [out, in] layout): Y^T = W_down^T A_2^T has the shape of stage one, with d_ff as the k
// range, a row tile = 16 rows of one matrix, A_2 in X's place, and workgroup s owning a slice of d_model whole:
// nothing is summed across workgroups, the end just adds the wavefronts' k-partial sums and stores Y.
template <int NW, int TT, typename E, bool NORM, bool PUBLISH, bool DOWN_T = false>
__device__ __forceinline__ void gateup_km_body(const MlpArgs& a, const KmGeom& geo, const int wg, unsigned char* lds) {
    constexpr int TOK = 16 * TT;
    constexpr int NTHREADS = NW * 64;
    constexpr int NT = kKmMaxRowTiles;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int q = lane & 15, g = lane >> 4;
    int j0, j1;
    if (DOWN_T) {            // slices of d_model, in whole 16-row tiles
        const long long t16 = a.d_model / 16;
        j0 = (int)(t16 * wg / a.k2_splits) * 16;
        j1 = (int)(t16 * (wg + 1) / a.k2_splits) * 16;
    } else {
        slice_rows(a.d_ff, a.splits, wg, j0, j1);
    }
    const int nt = (j1 - j0) / (DOWN_T ? 16 : 8);   // <= NT, checked on the host
    // The 128-k chunks of a row are dealt out to the wavefronts in contiguous runs, as evenly as
    // their number allows (equal runs when the k range is a multiple of 128 * NW).
    const int kdim = DOWN_T ? a.d_ff : a.d_model;
    const int nchunks = kdim / kKC;
    const int c0 = wave * nchunks / NW, c1 = (wave + 1) * nchunks / NW;
    const size_t kbase = (size_t)c0 * (kKC * 2);          // bytes into a row

    KmStream1<NW, TT> ts;
    ts.row_bytes = (size_t)kdim * 2;
    if (DOWN_T) {
        ts.Wg = (const char*)a.Wd; ts.Wu = (const char*)a.Wd + 8 * ts.row_bytes; ts.X = (const char*)a.a2;
        ts.tile_rows = 16;
    } else {
        ts.Wg = (const char*)a.Wg; ts.Wu = (const char*)a.Wu; ts.X = (const char*)a.X;
        ts.tile_rows = 8;
    }
    ts.w_base = (size_t)j0 * ts.row_bytes + kbase;
    ts.x_base = (size_t)a.m_base * ts.row_bytes + kbase;
    ts.nt = nt; ts.nkc = c1 - c0; ts.m_count = a.m_count;
    ts.q = q; ts.g = g;
    ts.ring = lds + wave * geo.depth * kTileBytes;
    ts.depth = geo.depth;
    DFK_STAMP(DOWN_T ? 3 : 0);
    // The wavefront's slice of the normalisation weight travels to LDS by the same asynchronous
    // loads as the tiles, issued ahead of them: they are the oldest in the queue, so the first
    // tile's counted wait covers them and no register or extra wait is involved.  Slices sit
    // 1 KB-aligned (one load instruction writes 1 KB); lanes past a short slice re-read its end.
    const int wbytes = ts.nkc * (kKC * 2);
    const int wstride = km_norm_stride(a.d_model, NW);
    unsigned char* wslice = lds + geo.norm_off + (size_t)wave * wstride;
    float* ssq = (float*)(lds + geo.norm_off + (size_t)NW * wstride);   // [NW][TOK] sums of squares
    float ss[TT];
#pragma unroll
    for (int tt = 0; tt < TT; ++tt) ss[tt] = 0.f;
    if (NORM) {
        const char* src = (const char*)a.norm_w + kbase;
        for (int o = 0; o < wbytes; o += 1024)
            __builtin_amdgcn_global_load_lds(src + min(o + lane * 16, wbytes - 16), DFK_LDS_PTR(wslice + o), 16, 0, 0);
    }
    ts.start();

    f32x4 acc[NT][TT];
#pragma unroll
    for (int rt = 0; rt < NT; ++rt)
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) acc[rt][tt] = f32x4{0.f, 0.f, 0.f, 0.f};

    for (int kc = 0; kc < ts.nkc; ++kc) {
        u32x4 xk[TT][4];       // B operand of this chunk: token q of each token tile, k group g of step c
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) {
            const unsigned char* slot = ts.acquire();
#pragma unroll
            for (int c = 0; c < 4; ++c) xk[tt][c] = *(const u32x4*)(slot + (q * 16 + ((4 * c + g) ^ q)) * 16);
            if (NORM) {   // one token tile at a time, the weight re-read from LDS: few registers live
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const u32x4 wv = *(const u32x4*)(wslice + ((size_t)kc * kKC + (4 * c + g) * 8) * 2);
#pragma unroll
                    for (int p = 0; p < 4; ++p) {
                        float w0, w1, h0, h1;
                        E::widen2(wv[p], w0, w1);
                        E::widen2(xk[tt][c][p], h0, h1);
                        ss[tt] = fmaf(h0, h0, ss[tt]);
                        ss[tt] = fmaf(h1, h1, ss[tt]);
                        uint32_t packed = E::pack2(h0 * w0, h1 * w1);
                        asm volatile("" : "+v"(packed));
                        xk[tt][c][p] = packed;
                    }
                    // pin the sum here: otherwise the adds sink to the end of the chunk and the
                    // widened values stay live across all its MFMAs
                    asm volatile("" : "+v"(ss[tt]));
                }
            }
        }
#pragma unroll
        for (int rt = 0; rt < NT; ++rt) {
            if (rt < nt) {
                const unsigned char* slot = ts.acquire();
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const u32x4 av = *(const u32x4*)(slot + (q * 16 + ((4 * c + g) ^ q)) * 16);
#pragma unroll
                    for (int tt = 0; tt < TT; ++tt) acc[rt][tt] = mfma16<E>(av, xk[tt][c], acc[rt][tt]);
                }
            }
        }
    }
    DFK_STAMP(DOWN_T ? 4 : 2);
    if (NORM) {   // lanes (q, 0..3) hold the four k groups' shares of token q's squares
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) {
            float v = ss[tt];
            v += __shfl_xor(v, 16);
            v += __shfl_xor(v, 32);
            if (g == 0) ssq[wave * TOK + tt * 16 + q] = v;
        }
    }

    // Every wavefront's tile loads have landed (its last acquire waited for all of them), so
    // after this barrier the rings are free.  The wavefronts' k-partial sums meet there,
    // geo.pass row tiles at a time: [row tile][wavefront][token][16 rows] fp32.
    __syncthreads();
    float* stage = (float*)lds;
    for (int rt0 = 0; rt0 < nt; rt0 += geo.pass) {
        const int cnt = min(geo.pass, nt - rt0);
#pragma unroll
        for (int rt = 0; rt < NT; ++rt) {
            if (rt >= rt0 && rt < rt0 + cnt) {
#pragma unroll
                for (int tt = 0; tt < TT; ++tt)
                    *(f32x4*)(stage + ((size_t)((rt - rt0) * NW + wave) * TOK + tt * 16 + q) * 16 + 4 * g) = acc[rt][tt];
            }
        }
        __syncthreads();
        if (DOWN_T) {
            // task (row tile r of the pass, token m, row quad): four adjacent outputs of Y's row m
            for (int t = tid; t < cnt * TOK * 4; t += NTHREADS) {
                const int r = t / (TOK * 4), rem = t - r * (TOK * 4);
                const int m = rem >> 2, quad = rem & 3;
                if (m < a.m_count) {
                    const float* src = stage + ((size_t)(r * NW) * TOK + m) * 16 + 4 * quad;
                    f32x4 v = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int w = 0; w < NW; ++w) v += *(const f32x4*)(src + (size_t)w * TOK * 16);
                    const size_t o = (size_t)(a.m_base + m) * a.d_model + j0 + (rt0 + r) * 16 + 4 * quad;
                    if (a.resid) {
                        float rr[4];
                        E::load4(a.resid, o, rr);
                        v[0] += rr[0]; v[1] += rr[1]; v[2] += rr[2]; v[3] += rr[3];
                    }
                    E::store4(a.Y, o, v[0], v[1], v[2], v[3]);
                }
            }
            __syncthreads();
            continue;
        }
        // task (row tile r of the pass, token m, row pair pr): rows 2pr, 2pr+1 (gate) and 8 further on (up)
        for (int t = tid; t < cnt * TOK * 4; t += NTHREADS) {
            const int r = t / (TOK * 4), rem = t - r * (TOK * 4);
            const int m = rem >> 2, pr = rem & 3;
            if (m < a.m_count) {
                const float* src = stage + ((size_t)(r * NW) * TOK + m) * 16 + 2 * pr;
                float g0 = 0.f, g1 = 0.f, u0 = 0.f, u1 = 0.f;
#pragma unroll
                for (int w = 0; w < NW; ++w) {
                    const float2 gv = *(const float2*)(src + (size_t)w * TOK * 16);
                    const float2 uv = *(const float2*)(src + (size_t)w * TOK * 16 + 8);
                    g0 += gv.x; g1 += gv.y; u0 += uv.x; u1 += uv.y;
                }
                if (NORM) {
                    float sq = 0.f;
#pragma unroll
                    for (int w = 0; w < NW; ++w) sq += ssq[w * TOK + m];
                    const float sm = __builtin_amdgcn_rsqf(sq / (float)a.d_model + a.eps);
                    g0 *= sm; g1 *= sm; u0 *= sm; u1 *= sm;
                }
                const size_t o = (size_t)(a.m_base + m) * a.d_ff + j0 + (rt0 + r) * 8 + 2 * pr;
                const uint32_t v = E::pack2(silu_mul_fast(g0, u0), silu_mul_fast(g1, u1));
                if (PUBLISH) __hip_atomic_store((uint32_t*)((uint16_t*)a.a2 + o), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                else *(uint32_t*)((uint16_t*)a.a2 + o) = v;
            }
        }
        __syncthreads();
    }
    DFK_STAMP(DOWN_T ? 6 : 1);   // A_2 (or Y) stored
    if (PUBLISH && geo.role_publish) {
        drain_own_memory_ops();                  // this wavefront's A_2 stores are acknowledged
        __syncthreads();
        if (tid == 0) {                          // one count on every split of the down projection these rows belong to
            const int ng = a.d_ff / 8;
            const int lo = slice_of_group(ng, a.k2_splits, j0 / 8), hi = slice_of_group(ng, a.k2_splits, j1 / 8 - 1);
            for (int js = lo; js <= hi; ++js)
                __hip_atomic_fetch_add(a.tickets + kRoleCount0 + js * geo.role_stride, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

template <int NW, int TT, typename E, bool NORM>
__global__ __launch_bounds__(NW * 64) void k_gateup_km(MlpArgs a, KmGeom geo) {
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    gateup_km_body<NW, TT, E, NORM, false>(a, geo, blockIdx.x, lds);
}

// Down projection from W_down given as [d_model, d_ff]: k2_splits workgroups, a slice of d_model each.
template <int NW, int TT, typename E>
__global__ __launch_bounds__(NW * 64) void k_down_t_km(MlpArgs a, KmGeom geo) {
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    gateup_km_body<NW, TT, E, false, false, true>(a, geo, blockIdx.x, lds);
}

// ---------------------------------------------------------------- down kernel
template <int NW, int TT>
struct KmStream2 {
    // A_2 travels in tiles of 64 d_ff rows x 32 tokens: per token 128 contiguous bytes, one whole cache line per
    // request (a 32-row tile would be 64-byte pieces, twice the requests for the same bytes).  One tile serves
    // two 32-row blocks; NA tiles cover the launch's token tiles.
    static constexpr int NA = TT > 2 ? 2 : 1;
    const char *Wd, *A2;
    size_t row_bytes;          // d_model * 2
    size_t a2_row_bytes;       // d_ff * 2
    size_t a2_base;            // byte offset of (token m_base, row j0)
    int d_ff, j0, rows, m_count;
    int blk_first, CB;
    int jb_lo, njb;
    int q, g;
    unsigned off2;
    unsigned char* ring;
    int depth, T, issued, issue_slot, take_slot;
    int p_grp, p_idx;          // producer: pair of 32-row blocks, position in the pair's tile sequence
    int a_pos;                 // position of the pair's A tiles: 0, or 2 CB = behind the first block's weight tiles

    __device__ __forceinline__ void issue() {
        unsigned char* slot = ring + issue_slot * kTileBytes;
        const int jb0 = jb_lo + 2 * p_grp;
        const bool two = 2 * p_grp + 1 < njb;
        if (p_idx >= a_pos && p_idx < a_pos + NA) {
            // A tile `half`: instruction u = tokens 32 half + 8u .. +7; lanes 8t .. 8t+7 = the 128 bytes of token t,
            // the 16-byte chunks of odd tokens swapped by four so that the operand reads spread over the banks
            const int half = p_idx - a_pos;
            const int lane = 16 * g + q;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int tl = 32 * half + 8 * u + (lane >> 3);
                const int chunk = (lane & 7) ^ ((tl & 1) << 2);
                const int token = min(min(tl, 16 * TT - 1), m_count - 1);
                const int j = min(jb0 * 32 + 8 * chunk, rows - 8);   // past the split: any valid address (masked at use)
                const char* src = A2 + a2_base + (size_t)token * a2_row_bytes + (size_t)j * 2;
                __builtin_amdgcn_global_load_lds(src, DFK_LDS_PTR(slot + u * 1024), 16, 0, 0);
            }
        } else {
            const int wi = p_idx - (p_idx > a_pos ? NA : 0);   // index among the pair's weight tiles
            const int jb = jb0 + (wi >= 2 * CB ? 1 : 0);
            const int wj = wi - (wi >= 2 * CB ? 2 * CB : 0);
            const int b = wj >> 1, h = wj & 1;
            const int row0 = j0 + jb * 32 + 4 * h;           // lane adds 8g + u
            const size_t colb = (size_t)(blk_first + b) * 256;
            if (row0 + 28 <= d_ff) {
                const char* base = Wd + (size_t)row0 * row_bytes + colb;
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    __builtin_amdgcn_global_load_lds(base + (size_t)u * row_bytes + off2, DFK_LDS_PTR(slot + u * 1024), 16,
                                                     0, kAuxNonTemporal);
            } else {           // last rows of W_down: clamp per lane (values are masked later)
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int row = min(row0 + 8 * g + u, d_ff - 1);
                    __builtin_amdgcn_global_load_lds(Wd + (size_t)row * row_bytes + colb + 16 * q,
                                                     DFK_LDS_PTR(slot + u * 1024), 16, 0, kAuxNonTemporal);
                }
            }
        }
        if (++p_idx == NA + 2 * CB * (two ? 2 : 1)) { p_idx = 0; ++p_grp; }
        ++issued;
        if (++issue_slot == depth) issue_slot = 0;
    }
    // limit: most tiles to request now (the single launch holds back the first A tile until A_2 is complete)
    __device__ __forceinline__ void start(const int limit) {
        off2 = (unsigned)(8 * g * row_bytes + 16 * q);
        T = ((njb + 1) / 2) * NA + njb * 2 * CB;
        issued = 0; issue_slot = 0; take_slot = 0; p_grp = 0; p_idx = 0;
        const int ahead = min(min(depth - 1, T), limit);
        for (int i = 0; i < ahead; ++i) issue();
    }
    __device__ __forceinline__ void top_up() {
        const int ahead = min(depth - 1, T);
        while (issued < ahead) issue();
    }
    __device__ __forceinline__ const unsigned char* acquire() {
        DFK_WAIT_LGKM0();
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

__host__ __device__ constexpr int km_col_blocks(int tt) { return tt >= 3 ? 1 : 2; }   // accumulator budget

//
// WAIT (the single launch of both kernels' workgroups): the stream carries the A tile of a 32-row block behind the
// first column block's weight tiles and starts with those alone; then the workgroup waits until every gate/up
// workgroup has counted itself done, drops what its caches hold of A_2's lines, and goes on as the kernel does.
template <int NW, int TT, typename E, bool WAIT>
__device__ __forceinline__ void down_km_body(const MlpArgs& a, const KmGeom& geo, const int wg, unsigned char* lds) {
    __shared__ int flag;
    constexpr int NTHREADS = NW * 64;
    constexpr int CBM = km_col_blocks(TT);
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int q = lane & 15, g = lane >> 4;
    const int js = wg / a.k2_col_blocks;
    const int cb = wg - js * a.k2_col_blocks;
    int j0, j1;
    slice_rows(a.d_ff, a.k2_splits, js, j0, j1);
    const int rows = j1 - j0;
    const int CB = a.d_model / 128 / a.k2_col_blocks;      // <= CBM, checked on the host
    const int blk_lo = cb * CB;
    const int njb_all = (rows + 31) / 32;
    const int jb_lo = (int)((long long)njb_all * wave / NW);
    const int njb = (int)((long long)njb_all * (wave + 1) / NW) - jb_lo;

    KmStream2<NW, TT> ts;
    ts.Wd = (const char*)a.Wd; ts.A2 = (const char*)a.a2;
    ts.row_bytes = (size_t)a.d_model * 2;
    ts.a2_row_bytes = (size_t)a.d_ff * 2;
    ts.a2_base = ((size_t)a.m_base * a.d_ff + j0) * 2;
    ts.d_ff = a.d_ff; ts.j0 = j0; ts.rows = rows; ts.m_count = a.m_count;
    ts.blk_first = blk_lo; ts.CB = CB;
    ts.jb_lo = jb_lo; ts.njb = njb;
    ts.q = q; ts.g = g;
    const int depth = WAIT ? geo.depth_down : geo.depth;
    ts.ring = lds + wave * depth * kTileBytes;
    ts.depth = depth;
    // the single launch: with one token tile every column block's weight tiles of a pair's first block precede the
    // A tiles (more to request before the wait); with more token tiles only the first column block's (registers)
    constexpr int PRE = TT == 1 ? CBM : 1;
    const int pre = min(PRE, CB);
    ts.a_pos = WAIT ? 2 * pre : 0;
    DFK_STAMP(3);
    bool gave_up = false;
    unsigned passed_before = 0;
    if (WAIT) {
        ts.start(2 * pre);                 // weight tiles only: nothing of A_2 yet
        if (geo.role_wait > 0) {
            if (tid == 0) {
                int polls = 0, ok = 1;
                const int ng = a.d_ff / 8;
                const unsigned expected = (unsigned)(slice_of_group(ng, a.splits, j1 / 8 - 1) - slice_of_group(ng, a.splits, j0 / 8) + 1);
                const unsigned* cnt = a.tickets + kRoleCount0 + js * geo.role_stride;
                while (__hip_atomic_load(cnt, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < expected) {
                    if (++polls > geo.role_spin_limit) { ok = 0; break; }
                    __builtin_amdgcn_s_sleep(8);
                }
                // gate/up workgroups of other XCDs wrote parts of lines this XCD's L2 may hold: drop them
                acquire_device();
                flag = ok;
            }
            __syncthreads();
            gave_up = flag == 0;
            __syncthreads();               // flag is used again by the reduction
            DFK_STAMP(7);
            // this workgroup is past its wait; the answer is looked at when the stream has ended
            if (tid == 0) passed_before = __hip_atomic_fetch_add(a.tickets + kRolePassed, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        ts.top_up();
    } else {
        ts.start(1 << 30);
    }

    f32x4 acc2[CBM][8][TT];
#pragma unroll
    for (int b = 0; b < CBM; ++b)
#pragma unroll
        for (int c = 0; c < 8; ++c)
#pragma unroll
            for (int tt = 0; tt < TT; ++tt) acc2[b][c][tt] = f32x4{0.f, 0.f, 0.f, 0.f};

    for (int grp = 0; 2 * grp < njb; ++grp) {
        const int jb0 = jb_lo + 2 * grp;
        const bool two = 2 * grp + 1 < njb;
        u32x4 av[2][TT];       // A operands of the pair's two blocks: A_2[token q of tile tt][rows 8g .. 8g+7 of the block]
        auto take_a = [&]() {
#pragma unroll
            for (int half = 0; half < KmStream2<NW, TT>::NA; ++half) {
                const unsigned char* slot = ts.acquire();
#pragma unroll
                for (int t2 = 0; t2 < 2; ++t2) {
                    const int tt = 2 * half + t2;
                    if (tt < TT) {
#pragma unroll
                        for (int h = 0; h < 2; ++h) {
                            const int idx = (2 * t2 + (q >> 3)) * 64 + (q & 7) * 8 + ((4 * h + g) ^ ((q & 1) << 2));
                            const u32x4 v = *(const u32x4*)(slot + idx * 16);
                            av[h][tt] = (jb0 + h) * 32 + 8 * g >= rows ? u32x4{0, 0, 0, 0} : v;
                        }
                    }
                }
            }
        };
        auto take_w = [&](const int jb, u32x4 (&w)[8]) {
            const unsigned char* sa = ts.acquire();
#pragma unroll
            for (int u = 0; u < 4; ++u) w[u] = *(const u32x4*)(sa + u * 1024 + lane * 16);
            const unsigned char* sb = ts.acquire();
#pragma unroll
            for (int u = 0; u < 4; ++u) w[4 + u] = *(const u32x4*)(sb + u * 1024 + lane * 16);
            if (jb * 32 + 32 > rows) {   // rows past the split contribute nothing
#pragma unroll
                for (int r = 0; r < 8; ++r)
                    if (jb * 32 + 8 * g + r >= rows) w[r] = u32x4{0, 0, 0, 0};
            }
        };
        auto multiply = [&](const int b, const int h, const u32x4 (&w)[8]) {
#pragma unroll
            for (int c = 0; c < 8; ++c) {
                const uint32_t sel = (c & 1) ? 0x07060302u : 0x05040100u;
                u32x4 bb;
#pragma unroll
                for (int p = 0; p < 4; ++p) bb[p] = __builtin_amdgcn_perm(w[2 * p + 1][c >> 1], w[2 * p][c >> 1], sel);
#pragma unroll
                for (int tt = 0; tt < TT; ++tt)
                    acc2[b][c][tt] = mfma16<E>(av[h][tt], bb, acc2[b][c][tt]);
            }
        };
        if (WAIT) {            // weight tiles of the first block's first `pre` column blocks come first in the stream, then the pair's A tiles
            u32x4 w[PRE][8];
#pragma unroll
            for (int b = 0; b < PRE; ++b)
                if (b < pre) take_w(jb0, w[b]);
            take_a();
#pragma unroll
            for (int b = 0; b < PRE; ++b)
                if (b < pre) multiply(b, 0, w[b]);
#pragma unroll
            for (int b = PRE; b < CBM; ++b) {
                if (b < CB) {
                    u32x4 w2[8];
                    take_w(jb0, w2);
                    multiply(b, 0, w2);
                }
            }
        } else {
            take_a();
#pragma unroll
            for (int b = 0; b < CBM; ++b) {
                if (b < CB) {
                    u32x4 w[8];
                    take_w(jb0, w);
                    multiply(b, 0, w);
                }
            }
        }
        if (two) {
#pragma unroll
            for (int b = 0; b < CBM; ++b) {
                if (b < CB) {
                    u32x4 w[8];
                    take_w(jb0 + 1, w);
                    multiply(b, 1, w);
                }
            }
        }
    }
    if (WAIT && gave_up) {   // the wait ran out (never, unless a gate/up workgroup cannot run): make the failure visible in Y
#pragma unroll
        for (int b = 0; b < CBM; ++b)
#pragma unroll
            for (int c = 0; c < 8; ++c)
#pragma unroll
                for (int tt = 0; tt < TT; ++tt) acc2[b][c][tt] = f32x4{NAN, NAN, NAN, NAN};
    }
    DFK_STAMP(4);

    // The wavefronts' sums over their rows meet in LDS, one column block and one token tile
    // at a time: per-wavefront stages [16 tokens][128] over the drained rings.
    const bool atomic_mode = a.reduce_mode == DFK_REDUCE_ATOMIC;
    float* stage = (float*)lds;                           // [NW][16][128]
    __syncthreads();
#pragma unroll
    for (int b = 0; b < CBM; ++b) {
        if (b < CB) {
            const int nb = (blk_lo + b) * 128;
#pragma unroll
            for (int tt = 0; tt < TT; ++tt) {
                if (tt * 16 < a.m_count) {                // uniform: token tiles past the launch's tokens hold nothing
                    float* mine = stage + (size_t)wave * 16 * 128;
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        float* dst = mine + (4 * g + i) * 128 + 8 * q;
                        *(f32x4*)dst = f32x4{acc2[b][0][tt][i], acc2[b][1][tt][i], acc2[b][2][tt][i], acc2[b][3][tt][i]};
                        *(f32x4*)(dst + 4) = f32x4{acc2[b][4][tt][i], acc2[b][5][tt][i], acc2[b][6][tt][i], acc2[b][7][tt][i]};
                    }
                    __syncthreads();
                    const int mt = min(16, a.m_count - tt * 16);   // tokens of this tile
                    if (atomic_mode) {
                        for (int idx = tid; idx < mt * 128; idx += NTHREADS) {
                            float v = 0.f;
#pragma unroll
                            for (int w = 0; w < NW; ++w) v += stage[w * 16 * 128 + idx];
                            acc_add(a.yacc + (size_t)(tt * 16 + (idx >> 7)) * a.d_model + nb + (idx & 127), v);
                        }
                    } else {
                        for (int idx = tid; idx < mt * 32; idx += NTHREADS) {
                            f32x4 v = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                            for (int w = 0; w < NW; ++w) v += *(const f32x4*)(stage + w * 16 * 128 + 4 * idx);
                            const int m = tt * 16 + (idx >> 5), c4 = idx & 31;
                            store4_device(a.P + ((size_t)js * a.m_count + m) * a.d_model + nb + 4 * c4, v[0], v[1], v[2], v[3]);
                        }
                    }
                    __syncthreads();
                }
            }
        }
    }
    const int width = CB * 128;
    if (WAIT && geo.role_wait > 0 && tid == 0) {
        // every down workgroup is past its wait once the last one has said so: that one clears the counters for the next launch
        const unsigned n_down = (unsigned)(a.k2_splits * a.k2_col_blocks);
        if (passed_before == n_down - 1u) {
            __hip_atomic_store(a.tickets + kRolePassed, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            for (int x = 0; x < a.k2_splits; ++x)
                __hip_atomic_store(a.tickets + kRoleCount0 + x * geo.role_stride, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    if (atomic_mode) {
        drain_own_memory_ops();
        __syncthreads();
        if (tid == 0) flag = arrive_last(a.tickets + cb, (unsigned)a.k2_splits) ? 1 : 0;
        __syncthreads();
        if (!flag) return;
        for (int idx = tid; idx < a.m_count * (width / 2); idx += NTHREADS) {
            const int m = idx / (width / 2), c2 = idx - m * (width / 2);
            float* src = a.yacc + (size_t)m * a.d_model + blk_lo * 128 + 2 * c2;
            float v0 = acc_take(src), v1 = acc_take(src + 1);
            const size_t o = (size_t)(a.m_base + m) * a.d_model + blk_lo * 128 + 2 * c2;
            if (a.resid) {
                float r0, r1;
                E::widen2(*(const uint32_t*)((const uint16_t*)a.resid + o), r0, r1);
                v0 += r0; v1 += r1;
            }
            *(uint32_t*)((uint16_t*)a.Y + o) = E::pack2(v0, v1);
        }
        return;
    }
    reduce_store<E>(plan_column_block(a, cb, blk_lo * 128, blk_lo * 128 + width), a.Y, a.m_base, &flag, a.trace, a.resid);
}

template <int NW, int TT, typename E>
__global__ __launch_bounds__(NW * 64) void k_down_km(MlpArgs a, KmGeom geo) {
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    down_km_body<NW, TT, E, false>(a, geo, blockIdx.x, lds);
}

// ---------------------------------------------------------------- both kernels' workgroups in one launch
// Grid = the gate/up kernel's workgroups followed by the down kernel's.  Workgroups are dispatched in index
// order, so no down workgroup starts before every gate/up workgroup (of its XCD's share of the grid) has, and a
// gate/up workgroup waits for nothing: the down workgroups' wait always ends.  What the single launch buys over
// two: no launch boundary (drain, dispatch and ramp with HBM idle), and the down workgroups request their first
// W_down tiles while the last gate/up workgroups are still streaming.  A_2 crosses between workgroups through
// device memory (2 bytes per token and d_ff row), as between the two kernels.
template <int NW, int TT, typename E>
__global__ __launch_bounds__(NW * 64) void k_roles_km(MlpArgs a, KmGeom geo) {
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    if ((int)blockIdx.x < geo.n_gateup) gateup_km_body<NW, TT, E, false, true>(a, geo, blockIdx.x, lds);
    else down_km_body<NW, TT, E, true>(a, geo, blockIdx.x - geo.n_gateup, lds);
}

// ---------------------------------------------------------------- host side
int km_token_tiles(int m_count) { return m_count <= 16 ? 1 : m_count <= 32 ? 2 : m_count <= 48 ? 3 : 4; }

// norm: the kernel also keeps the normalisation weight (d_model 16-bit values, a 1 KB-aligned
// slice per wavefront) and the wavefronts' sums of squares behind rings and stage.
size_t km_lds_gateup(const dfk_config_t& c, int TT, int d_model, int d_ff, bool norm, KmGeom* geo) {
    const int nt_max = max_slice_rows(d_ff, c.splits) / 8;
    const size_t ring = (size_t)c.waves * c.depth * kTileBytes;
    const size_t per_tile = (size_t)c.waves * 16 * TT * 16 * 4;   // partial sums of one row tile
    const size_t wstride = (size_t)km_norm_stride(d_model, c.waves);
    const size_t extra = norm ? (size_t)c.waves * wstride + (size_t)c.waves * 16 * TT * 4 : 0;
    const size_t room = (size_t)kLdsLimit > extra ? (size_t)kLdsLimit - extra : 0;
    const int fit = (int)(room / per_tile);
    geo->depth = c.depth;
    geo->pass = std::max(1, std::min(nt_max, fit));
    const size_t base = std::max(ring, (size_t)geo->pass * per_tile);
    geo->norm_off = (int)base;
    return base + extra;
}
size_t km_lds_down(const dfk_config_t& c, KmGeom* geo) {
    geo->depth = c.depth;
    geo->pass = 0;
    geo->norm_off = 0;
    return std::max((size_t)c.waves * c.depth * kTileBytes, (size_t)c.waves * 16 * 128 * 4);
}

// down kernel on W_down as [d_model, d_ff]: rings, or the k-partial sums of as many 16-row tiles as fit
int km_down_t_max_tiles(int d_model, int k2_splits) { return (d_model / 16 + k2_splits - 1) / k2_splits; }
size_t km_lds_down_t(const dfk_config_t& c, int TT, int d_model, KmGeom* geo) {
    const int nt_max = km_down_t_max_tiles(d_model, c.k2_splits);
    const size_t ring = (size_t)c.waves * c.depth * kTileBytes;
    const size_t per_tile = (size_t)c.waves * 16 * TT * 16 * 4;
    geo->depth = c.depth;
    geo->pass = std::max(1, std::min(nt_max, (int)((size_t)kLdsLimit / per_tile)));
    geo->norm_off = 0;
    return std::max(ring, (size_t)geo->pass * per_tile);
}

template <int NW, int TT, typename E>
hipError_t launch_km_te(const MlpArgs& a, const dfk_config_t& c, hipStream_t st) {
    static LdsAllowance allowed1, allowed1n, allowed2;   // of the three kernels of this instantiation, per device
    if ((g_stage_mask & 1) && !a.norm_w) {
        KmGeom geo{};
        const size_t lds = km_lds_gateup(c, TT, a.d_model, a.d_ff, false, &geo);
        if (hipError_t e = allow_lds(allowed1, (const void*)k_gateup_km<NW, TT, E, false>, lds); e != hipSuccess) return e;
        hipLaunchKernelGGL((k_gateup_km<NW, TT, E, false>), dim3(a.splits), dim3(NW * 64), lds, st, a, geo);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if ((g_stage_mask & 1) && a.norm_w) {
        KmGeom geo{};
        const size_t lds = km_lds_gateup(c, TT, a.d_model, a.d_ff, true, &geo);
        if (hipError_t e = allow_lds(allowed1n, (const void*)k_gateup_km<NW, TT, E, true>, lds); e != hipSuccess) return e;
        hipLaunchKernelGGL((k_gateup_km<NW, TT, E, true>), dim3(a.splits), dim3(NW * 64), lds, st, a, geo);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if ((g_stage_mask & 2) && c.kmajor == 5) {
        static LdsAllowance allowed2t;
        KmGeom geo{};
        const size_t lds = km_lds_down_t(c, TT, a.d_model, &geo);
        if (hipError_t e = allow_lds(allowed2t, (const void*)k_down_t_km<NW, TT, E>, lds); e != hipSuccess) return e;
        hipLaunchKernelGGL((k_down_t_km<NW, TT, E>), dim3(a.k2_splits), dim3(NW * 64), lds, st, a, geo);
        return hipGetLastError();
    }
    if (g_stage_mask & 2) {
        KmGeom geo{};
        const size_t lds = km_lds_down(c, &geo);
        if (hipError_t e = allow_lds(allowed2, (const void*)k_down_km<NW, TT, E>, lds); e != hipSuccess) return e;
        hipLaunchKernelGGL((k_down_km<NW, TT, E>), dim3(a.k2_splits * a.k2_col_blocks), dim3(NW * 64), lds, st, a, geo);
        return hipGetLastError();
    }
    return hipSuccess;
}

template <int NW, int TT>
hipError_t launch_km_t(const MlpArgs& a, const dfk_config_t& c, hipStream_t st) {
    return a.dtype == DFK_FP16 ? launch_km_te<NW, TT, FP16>(a, c, st) : launch_km_te<NW, TT, BF16>(a, c, st);
}

// Both kernels' workgroups in one launch.  The stage mask of the per-kernel timer maps to the head of the grid
// alone (gate/up workgroups, nothing counted) and to the tail alone (down workgroups that wait for nobody).
template <int NW, int TT, typename E>
hipError_t launch_km_roles_te(const MlpArgs& a, const dfk_config_t& c, hipStream_t st) {
    static LdsAllowance allowed;
    if (a.norm_w) return hipErrorInvalidValue;
    KmGeom geo{}, gd{};
    size_t lds = std::max(km_lds_gateup(c, TT, a.d_model, a.d_ff, false, &geo), km_lds_down(c, &gd));
    const bool head = g_stage_mask & 1, tail = g_stage_mask & 2;
    geo.n_gateup = head ? a.splits : 0;
    geo.role_publish = head && tail;
    geo.role_wait = head && tail ? a.splits : 0;
    geo.role_stride = 1;
    while (geo.role_stride < 32 && a.k2_splits * geo.role_stride * 2 <= kRoleCountEnd - kRoleCount0) geo.role_stride *= 2;
    geo.depth_down = std::max(c.depth, std::min(c.depth + 1, (int)((size_t)kLdsLimit / ((size_t)NW * kTileBytes))));
    lds = std::max(lds, (size_t)NW * geo.depth_down * kTileBytes);
    geo.role_spin_limit = 1 << 21;          // seconds; a healthy launch needs a handful of polls
    if (const char* e = std::getenv("DFK_DEBUG_SPIN_LIMIT")) geo.role_spin_limit = std::atoi(e);
    const int grid = geo.n_gateup + (tail ? a.k2_splits * a.k2_col_blocks : 0);
    if (grid == 0) return hipSuccess;
    if (hipError_t e = allow_lds(allowed, (const void*)k_roles_km<NW, TT, E>, lds); e != hipSuccess) return e;
    hipLaunchKernelGGL((k_roles_km<NW, TT, E>), dim3(grid), dim3(NW * 64), lds, st, a, geo);
    return hipGetLastError();
}
template <int NW, int TT>
hipError_t launch_km_roles_t(const MlpArgs& a, const dfk_config_t& c, hipStream_t st) {
    return a.dtype == DFK_FP16 ? launch_km_roles_te<NW, TT, FP16>(a, c, st) : launch_km_roles_te<NW, TT, BF16>(a, c, st);
}

}  // namespace

int mfma_km_tokens_per_launch() { return kKmTokensPerLaunch; }

bool mfma_km_config_valid(const dfk_config_t& c, int M, int d_model, int d_ff, dfk_dtype_t dtype) {
    if (c.path != DFK_PATH_MFMA || (dtype != DFK_BF16 && dtype != DFK_FP16) || c.variant != DFK_VARIANT_TWO_KERNEL) return false;
    if (c.kmajor != 1 || c.k2_rows_by_wave != 0 || c.a2_dtype != (int)dtype) return false;   // A_2 in the inputs' 16-bit type
    if (c.reduce != DFK_REDUCE_TICKET && c.reduce != DFK_REDUCE_ATOMIC) return false;
    if ((c.waves != 4 && c.waves != 8) || c.depth < 2 || c.depth > 16) return false;
    if (M < 1 || d_model < 8 || d_ff < 8 || d_ff % 8 || d_model > kMaxDModel) return false;
    if (d_model % kKC || d_model / kKC < c.waves) return false;   // each wavefront owns whole 128-k chunks, at least one
    const int ng = d_ff / 8;
    if (c.splits < 1 || c.splits > ng || c.splits > 65535) return false;
    if (max_slice_rows(d_ff, c.splits) / 8 > kKmMaxRowTiles) return false;   // accumulators of the row tiles
    if (c.k2_splits < 1 || c.k2_splits > ng) return false;
    const int nblk = d_model / 128;
    if (c.k2_col_blocks < 1 || nblk % c.k2_col_blocks) return false;
    if ((long long)c.k2_splits * c.k2_col_blocks > 65535 || c.k2_col_blocks > kTicketLevel2) return false;
    const int tokens = std::min(M, kKmTokensPerLaunch);
    const int TT = km_token_tiles(tokens);
    if (nblk / c.k2_col_blocks > km_col_blocks(TT)) return false;
    if (c.reduce == DFK_REDUCE_TICKET && !partials_fit(c.k2_splits, tokens, M, d_model)) return false;
    KmGeom geo{};
    return km_lds_gateup(c, TT, d_model, d_ff, false, &geo) <= (size_t)kLdsLimit && km_lds_down(c, &geo) <= (size_t)kLdsLimit;
}

// The pair whose down kernel takes W_down as [d_model, d_ff] (kmajor = 5): the gate/up kernel of the pair above, then
// k2_splits workgroups that own a slice of d_model each.  d_ff is that kernel's k range: whole 128-k chunks, at
// least one per wavefront.
bool mfma_km_t_config_valid(const dfk_config_t& c, int M, int d_model, int d_ff, dfk_dtype_t dtype) {
    if (c.path != DFK_PATH_MFMA || (dtype != DFK_BF16 && dtype != DFK_FP16) || c.variant != DFK_VARIANT_TWO_KERNEL) return false;
    if (c.kmajor != 5 || c.k2_rows_by_wave != 0 || c.a2_dtype != (int)dtype || c.reduce != DFK_REDUCE_TICKET) return false;
    if ((c.waves != 4 && c.waves != 8) || c.depth < 2 || c.depth > 16) return false;
    if (M < 1 || d_model < 16 || d_ff < 8 || d_ff % 8 || d_model > kMaxDModel) return false;
    if (d_model % kKC || d_model / kKC < c.waves) return false;          // gate/up kernel
    if (d_ff % kKC || d_ff / kKC < c.waves || d_model % 16) return false; // down kernel
    const int ng = d_ff / 8;
    if (c.splits < 1 || c.splits > ng || c.splits > 65535) return false;
    if (max_slice_rows(d_ff, c.splits) / 8 > kKmMaxRowTiles) return false;
    if (c.k2_col_blocks != 1 || c.k2_splits < 1 || c.k2_splits > d_model / 16 || c.k2_splits > 65535) return false;
    if (km_down_t_max_tiles(d_model, c.k2_splits) > kKmMaxRowTiles) return false;
    const int TT = km_token_tiles(std::min(M, kKmTokensPerLaunch));
    KmGeom geo{};
    return km_lds_gateup(c, TT, d_model, d_ff, false, &geo) <= (size_t)kLdsLimit && km_lds_down_t(c, TT, d_model, &geo) <= (size_t)kLdsLimit;
}

// The pre-norm residual form runs on this kernel pair only; its gate/up kernel needs a
// little more LDS (weight of the normalisation, sums of squares).
bool mfma_km_block_config_valid(const dfk_config_t& c, int M, int d_model, int d_ff, dfk_dtype_t dtype) {
    if (c.kmajor == 5 ? !mfma_km_t_config_valid(c, M, d_model, d_ff, dtype) : !mfma_km_config_valid(c, M, d_model, d_ff, dtype)) return false;
    KmGeom geo{};
    return km_lds_gateup(c, km_token_tiles(std::min(M, kKmTokensPerLaunch)), d_model, d_ff, true, &geo) <= (size_t)kLdsLimit;
}

// The single launch of both kernels' workgroups (variant FUSED, kmajor = 4): everything the pair asks of the
// configuration, and a grid small enough that its 16-bit-safe index arithmetic holds.
static dfk_config_t roles_as_pair(const dfk_config_t& c) { dfk_config_t p = c; p.variant = DFK_VARIANT_TWO_KERNEL; p.kmajor = 1; return p; }
bool mfma_km_roles_config_valid(const dfk_config_t& c, int M, int d_model, int d_ff, dfk_dtype_t dtype) {
    if (c.variant != DFK_VARIANT_FUSED || c.kmajor != 4 || c.waves != 8) return false;
    if ((long long)c.splits + (long long)c.k2_splits * c.k2_col_blocks > 65535) return false;
    if (c.k2_splits > kRoleCountEnd - kRoleCount0) return false;   // one counter per d_ff split of the down projection
    return mfma_km_config_valid(roles_as_pair(c), M, d_model, d_ff, dtype);
}
hipError_t launch_mfma_km_roles(const MlpArgs& a, const dfk_config_t& c, hipStream_t st) {
    const dfk_config_t p = roles_as_pair(c);
    switch (km_token_tiles(a.m_count)) {
        case 1: return launch_km_roles_t<8, 1>(a, p, st);
        case 2: return launch_km_roles_t<8, 2>(a, p, st);
        case 3: return launch_km_roles_t<8, 3>(a, p, st);
        case 4: return launch_km_roles_t<8, 4>(a, p, st);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_mfma_km(const MlpArgs& a, const dfk_config_t& c, hipStream_t st) {
    switch (c.waves * 10 + km_token_tiles(a.m_count)) {
        case 41: return launch_km_t<4, 1>(a, c, st);
        case 42: return launch_km_t<4, 2>(a, c, st);
        case 43: return launch_km_t<4, 3>(a, c, st);
        case 44: return launch_km_t<4, 4>(a, c, st);
        case 81: return launch_km_t<8, 1>(a, c, st);
        case 82: return launch_km_t<8, 2>(a, c, st);
        case 83: return launch_km_t<8, 3>(a, c, st);
        case 84: return launch_km_t<8, 4>(a, c, st);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace dfk
