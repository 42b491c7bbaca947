// MFMA path (bf16 inputs, fp32 accumulation) for gfx950: the deeply fused single
// launch, and the first generation of the two-kernel variant (at most 32 tokens
// per launch; dfk_mfma_km.hip holds the pair for up to 64).
//
// k_mfma<NW, TT, MODE> covers the fused launch (MODE_FUSED) and the two launches of
// the two-kernel variant (MODE_GATEUP, MODE_DOWN); k_down_rows is a second form of
// the down kernel.
//
// Work split ("column-major tiling" of the Method section: a workgroup owns a
// block of weight rows and reuses it for every token): workgroup s owns the
// d_ff slice [j0, j1).  Inside it, every wavefront consumes its own stream of
// 4 KB weight tiles that it brings from HBM straight into a private LDS ring
// with asynchronous 128-bit global->LDS loads (no VGPR staging, no workgroup
// barrier in the streaming loops).  The stream holds first the stage-one tiles
// (W_gate / W_up) and then, without a gap, the stage-two tiles (W_down), whose
// addresses do not depend on stage one, so HBM stays busy across the SiLU
// epilogue.
//
// Stage one (A_2 = (X W_up) (x) SiLU(X W_gate)): wavefront w owns the k-range
// [w*KW, (w+1)*KW) of d_model.  A tile is 16 weight rows (8 of W_gate, the same
// 8 of W_up) x 128 k; it is the A operand of v_mfma_f32_16x16x32_bf16 (4 k-steps
// per tile), X^T (tokens padded to 16 per token tile) is the B operand; the
// wavefront's whole k-range of X is loaded into registers once.  16-byte chunks
// are XOR-swizzled by row on the way into LDS (by permuting which global chunk
// each lane fetches), so the operand reads are bank-conflict free.  The
// wavefronts' k-partial sums meet in LDS without atomics: each wavefront stores
// its block and counts its arrival at the row tile; the one that arrives last
// adds the blocks, applies SiLU(G)*U and hands A_2 on (bf16 [token][j] in LDS and
// a ready flag in the fused kernel, so there is no workgroup barrier between the
// stages; the workspace in MODE_GATEUP).
//
// Stage two (Y += A_2 W_down over the slice): wavefront w owns 128-column blocks
// of d_model.  A tile is 4 row-groups of W_down: lane (q, g) fetches 16 bytes
// (8 consecutive columns) of row 8g+r.  After two tiles a lane holds an 8x8
// block (8 rows x 8 columns); v_perm_b32 regroups it into, per column, the 8
// consecutive-j values the MFMA B operand wants - a per-lane transpose, no
// cross-lane traffic.  A_2 (bf16, from LDS) is the A operand.  Stage two first
// does the slice's first 32 rows for all of the wavefront's column blocks (they
// need only row tiles whose flags were raised long ago, which absorbs the skew
// between wavefronts), then finishes and flushes one block after the other.
// The fp32 block of partial Y is published to the workspace with device-scope
// stores and combined by the two-level arrival-counter reduction (reduce_store),
// or added into the workspace accumulator with device-wide float atomics, one
// instruction per 64 consecutive floats (DFK_REDUCE_ATOMIC).
#include <atomic>
#include "dfk_mfma_common.h"

namespace dfk {
namespace {

constexpr int MODE_FUSED = 0, MODE_GATEUP = 1, MODE_DOWN = 2, MODE_DOWN_ROWS = 3;
constexpr int kMaxPartialSlots = 4;  // row tiles whose k-partial sums LDS holds at a time, at most

struct Geom {
    int depth;      // ring slots per wavefront
    int gu_off;     // LDS byte offset of the fp32 k-partial gate/up sums [slots][wavefronts][16*TT tokens][16 rows]
    int slots;      // row tiles whose partial sums LDS holds at a time
    int a2s_off;    // LDS byte offset of A_2 as bf16 [16*TT][a2_stride]
    int a2_stride;  // elements
    int sync_off;   // LDS byte offset of the row-tile arrival counters and ready flags
    int sync_cap;   // entries in each of the two (a multiple of 4, > row tiles)
};


// 16-byte B-operand registers a wavefront may spend on X: cap * 4 per lane.
__host__ __device__ constexpr int x_chunk_cap(int) { return 8; }
// 128-column blocks whose stage-two accumulators a wavefront holds at once.
__host__ __device__ constexpr int block_group(int tt) { return 4 / tt; }

// Per-wavefront producer/consumer of the weight-tile stream.
// Stage-one tiles come row-tile-major (tile (rt, kc): 16 rows x 128 k).  Stage-two
// tiles (16 rows x 128 columns; two per 32-row block jb) come per group of BG
// column blocks: first jb = 0 of every block of the group, then, block by block,
// jb = 1 .. njb-1.
template <int NW, int MODE, int BG>
struct TileStream {
    const char *Wg, *Wu, *Wd;
    int d_model, d_ff;
    int j0, nt, njb;          // slice start row, stage-one row tiles, stage-two 32-row blocks
    int nkc;                  // 128-k chunks of this wavefront's k range
    int blk_first, blk_step, my_blocks;   // stage two: this wavefront's 128-column blocks: blk_first + i*blk_step
    int jb_lo;                // stage two: first 32-row block of the slice this wavefront handles
    bool jb_major;            // stage two order: every column block of the group per 32-row block (rows-split kernel)
    int wave, q, g;
    // per-lane byte offsets inside a tile, fixed for the whole kernel
    unsigned off1[4];         // stage one, instruction u
    unsigned off2;            // stage two: (8g)*row_bytes + 16q
    size_t base1;             // stage one: byte offset of tile (0, 0) of this wavefront
    size_t row_bytes;
    // ring
    unsigned char* ring;
    int depth;
    int T1, T;                // stage-one tiles, all tiles
    int issued, issue_slot;   // producer position
    int take_slot;            // consumer position
    int p_rt, p_kc;           // producer coordinates, stage one
    int p_bg, p_phase, p_b, p_jb, p_h;   // producer coordinates, stage two

    __device__ __forceinline__ void init(int kbase) {
        row_bytes = (size_t)d_model * 2;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int i = 4 * u + g;   // row of the 16-row tile this lane fetches
            const int c = q ^ i;       // logical 16-byte chunk stored at position q of row i
            off1[u] = (unsigned)((i & 7) * row_bytes + c * 16);
        }
        off2 = (unsigned)(8 * g * row_bytes + 16 * q);
        base1 = (size_t)j0 * row_bytes + (size_t)kbase * 2;
    }

    __device__ __forceinline__ void issue() {
        unsigned char* slot = ring + issue_slot * kTileBytes;
        if (MODE != MODE_DOWN && issued < T1) {
            const size_t tb = base1 + (size_t)p_rt * 8 * row_bytes + (size_t)p_kc * (kKC * 2);
            const char* gb = Wg + tb;   // uniform
            const char* ub = Wu + tb;
#pragma unroll
            for (int u = 0; u < 4; ++u)
                __builtin_amdgcn_global_load_lds((u < 2 ? gb : ub) + off1[u], DFK_LDS_PTR(slot + u * 1024), 16, 0,
                                                 kAuxNonTemporal);
            if (++p_kc == nkc) { p_kc = 0; ++p_rt; }
        } else if (MODE != MODE_GATEUP) {
            const int jb = (p_phase || jb_major) ? p_jb : 0;
            const int row0 = j0 + (jb_lo + jb) * 32 + 4 * p_h;   // first row of this half (lane adds 8g + u)
            const size_t colb = (size_t)(blk_first + (p_bg + p_b) * blk_step) * 256;
            if (row0 + 28 <= d_ff) {     // every row of the tile exists: uniform base + lane offset
                const char* b = Wd + (size_t)row0 * row_bytes + colb;
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    __builtin_amdgcn_global_load_lds(b + (size_t)u * row_bytes + off2, DFK_LDS_PTR(slot + u * 1024), 16,
                                                     0, kAuxNonTemporal);
            } else {                     // last rows of W_down: clamp per lane (values are masked later)
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int row = min(row0 + 8 * g + u, d_ff - 1);
                    __builtin_amdgcn_global_load_lds(Wd + (size_t)row * row_bytes + colb + 16 * q,
                                                     DFK_LDS_PTR(slot + u * 1024), 16, 0, kAuxNonTemporal);
                }
            }
            p_h ^= 1;
            if (p_h == 0) {              // a 32-row chunk is complete: advance (phase, block, jb)
                const int nbk = min(BG, my_blocks - p_bg);
                if (jb_major) {
                    if (++p_b == nbk) {
                        p_b = 0;
                        if (++p_jb == njb) { p_jb = 0; p_bg += BG; }
                    }
                } else if (p_phase == 0) {
                    if (++p_b == nbk) {
                        p_b = 0;
                        if (njb > 1) { p_phase = 1; p_jb = 1; } else { p_bg += BG; }
                    }
                } else if (++p_jb == njb) {
                    p_jb = 1;
                    if (++p_b == nbk) { p_b = 0; p_phase = 0; p_bg += BG; }
                }
            }
        }
        ++issued;
        if (++issue_slot == depth) issue_slot = 0;
    }

    __device__ __forceinline__ void start() {
        issued = 0; issue_slot = 0; take_slot = 0;
        p_rt = 0; p_kc = 0; p_bg = 0; p_phase = 0; p_b = 0; p_jb = jb_major ? 0 : 1; p_h = 0;
        const int ahead = min(depth - 1, T);
        for (int i = 0; i < ahead; ++i) issue();
    }

    // Returns the LDS address of the next tile, landed and readable by this wavefront.
    // Only loads count: with at most 4*(depth-1) operations outstanding, at most that
    // many loads are, and loads complete in issue order, so the wanted tile is in.
    __device__ __forceinline__ const unsigned char* acquire() {
        // Reads of the slot about to be refilled must have returned before its refill is issued.
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

template <int NW, int TT, int MODE>
__global__ __launch_bounds__(NW * 64) void k_mfma(MlpArgs a, Geom geo) {
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    constexpr int TOK = 16 * TT;
    constexpr int NTHREADS = NW * 64;
    constexpr int NKC = x_chunk_cap(NW) / TT;   // 128-k chunks of X a wavefront can hold
    constexpr int BG = block_group(TT);
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int q = lane & 15, g = lane >> 4;
    const float* part = (const float*)(lds + geo.gu_off);   // k-partial sums [slot][wavefront][token][16 rows]
    uint16_t* a2s = (uint16_t*)(lds + geo.a2s_off);
    unsigned* sync = (unsigned*)(lds + geo.sync_off);   // [0, cap): arrivals per row tile, [cap, 2cap): ready flags
    const unsigned part_addr = lds_addr(part), a2s_addr = lds_addr(a2s), sync_addr = lds_addr(sync);
    const uint16_t* X = (const uint16_t*)a.X;

    // ---- geometry
    int j0, j1, blk_lo = 0, blk_cnt = a.d_model / 128;
    if (MODE == MODE_DOWN) {
        const int js = blockIdx.x / a.k2_col_blocks;
        const int cb = blockIdx.x - js * a.k2_col_blocks;
        slice_rows(a.d_ff, a.k2_splits, js, j0, j1);
        blk_cnt = blk_cnt / a.k2_col_blocks;
        blk_lo = cb * blk_cnt;
    } else {
        slice_rows(a.d_ff, a.splits, blockIdx.x, j0, j1);
    }
    const int rows = j1 - j0;
    const int nt = rows / 8;
    const int rows_pad = (rows + 31) & ~31;
    const int njb = rows_pad / 32;
    const int KW = a.d_model / NW;
    const int nkc = KW / kKC;
    const int my_blocks = wave < blk_cnt ? (blk_cnt - wave + NW - 1) / NW : 0;
    const bool atomic_mode = a.reduce_mode == DFK_REDUCE_ATOMIC;
    // block of the partial-sum area: one per slice (fused), one per d_ff split (down kernel)
    const int pblk = MODE == MODE_DOWN ? (int)blockIdx.x / a.k2_col_blocks : (int)blockIdx.x;

    TileStream<NW, MODE, BG> ts;
    ts.Wg = (const char*)a.Wg; ts.Wu = (const char*)a.Wu; ts.Wd = (const char*)a.Wd;
    ts.d_model = a.d_model; ts.d_ff = a.d_ff;
    ts.j0 = j0; ts.nt = nt; ts.njb = njb;
    ts.nkc = nkc;
    ts.blk_first = blk_lo + wave; ts.blk_step = NW; ts.my_blocks = my_blocks; ts.jb_lo = 0; ts.jb_major = false;
    ts.wave = wave; ts.q = q; ts.g = g;
    ts.ring = lds + wave * geo.depth * kTileBytes;
    ts.depth = geo.depth;
    ts.T1 = (MODE != MODE_DOWN) ? nt * nkc : 0;
    ts.T = ts.T1 + ((MODE != MODE_GATEUP) ? my_blocks * njb * 2 : 0);
    ts.init(wave * KW);

    // The tile stream starts first: nothing it needs depends on the LDS arrays below.
    DFK_STAMP(0);
    ts.start();

    // Everything in LDS that must start from a known value (raw stores: see dfk_mfma_common.h).
    if (MODE != MODE_DOWN) {
        for (int i = tid; i < 2 * geo.sync_cap; i += NTHREADS)
            lds_write_b32_raw(sync_addr + 4u * (unsigned)i, (i >= geo.sync_cap + nt) ? 1u : 0u);
        if (MODE == MODE_FUSED)
            for (int i = tid; i < TOK * geo.a2_stride / 2; i += NTHREADS) lds_write_b32_raw(a2s_addr + 4u * (unsigned)i, 0u);
        lds_barrier();
    }

    // ---- stage one
    if (MODE != MODE_DOWN) {
        // B operand: this wavefront's k range of X^T for every token tile, loaded once.
        // (The first use waits for everything issued so far, i.e. for the first
        // tiles of the stream too, which are needed at that point anyway.)
        u32x4 x[TT][NKC][4];
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) {
            const int token = tt * 16 + q;
#pragma unroll
            for (int kc = 0; kc < NKC; ++kc)
#pragma unroll
                for (int s = 0; s < 4; ++s) {
                    x[tt][kc][s] = u32x4{0, 0, 0, 0};
                    if (token < a.m_count && kc < nkc)
                        x[tt][kc][s] = ld16(X, ((size_t)(a.m_base + token) * a.d_model + wave * KW + kc * kKC) / 8 + 4 * s + g);
                }
        }
        int pslot = 0;   // rt % slots
        for (int rt = 0; rt < nt; ++rt) {
            if (rt == 1) DFK_STAMP(1);
            f32x4 acc[TT];
#pragma unroll
            for (int tt = 0; tt < TT; ++tt) acc[tt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kc = 0; kc < NKC; ++kc) {
                if (kc < nkc) {
                    const unsigned char* slot = ts.acquire();
#pragma unroll
                    for (int s = 0; s < 4; ++s) {
                        const bf16x8 av = *(const bf16x8*)(slot + (q * 16 + ((4 * s + g) ^ q)) * 16);
#pragma unroll
                        for (int tt = 0; tt < TT; ++tt)
                            acc[tt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, as_bf16x8(x[tt][kc][s]), acc[tt], 0, 0, 0);
                    }
                }
            }

            // The k-partial sums of the NW wavefronts meet in LDS without atomics (LDS float
            // atomics take about a cycle per lane and hold up the tile loads that land in
            // LDS meanwhile): each wavefront stores its [token][16 rows] block in a place
            // of its own in slot rt % slots, then counts its arrival at row tile rt; LDS
            // executes a wavefront's instructions in order, so the block is in before the
            // count.  The raw LDS stores are invisible to the compiler's hazard handling,
            // so the wait states an MFMA result needs before an LDS instruction may read
            // it are inserted by hand.
            if (rt >= geo.slots) {   // the slot's previous row tile must have been summed
                const unsigned freed = sync_addr + 4u * (unsigned)(geo.sync_cap + rt - geo.slots);
                while (__builtin_amdgcn_readfirstlane(lds_read_b32_raw(freed)) == 0u) __builtin_amdgcn_s_sleep(1);
            }
#pragma unroll
            for (int tt = 0; tt < TT; ++tt) asm volatile("s_nop 7\n\ts_nop 7\n\ts_nop 7" : "+v"(acc[tt]));
            const unsigned slot_floats = (unsigned)(pslot * NW * TOK * 16);
#pragma unroll
            for (int tt = 0; tt < TT; ++tt)
                lds_write_b128_raw(part_addr + 4u * (slot_floats + (unsigned)(((wave * TOK + tt * 16 + q) * 16) + 4 * g)), acc[tt]);
            unsigned old = 0;
            if (lane == 0) old = lds_inc_rtn_raw(sync_addr + 4u * (unsigned)rt);
            old = __builtin_amdgcn_readfirstlane(old);
            if (old == NW - 1) {
                // Last arrival: add the NW blocks in wavefront order, apply SiLU(G)*U and hand
                // A_2 on (LDS in the fused kernel, the workspace in the two-kernel variant),
                // then raise the row tile's flag: A_2 ready / slot free.
                // Task (token m, row quad h): rows 4h .. 4h+3 of the row tile (gate) and 8 further
                // on (up).  Two lanes share a task: lane p adds the blocks of wavefronts
                // [p*NW/2, (p+1)*NW/2), the halves are exchanged, and lane p finishes rows 2p, 2p+1.
                for (int t = lane; t < 4 * TOK; t += 64) {   // 4*TOK is a multiple of 64: no lane idles
                    const int p = t & 1, m = t >> 2, h = (t >> 1) & 1;
                    const float* src = part + slot_floats + (p * (NW / 2) * TOK + m) * 16 + 4 * h;
                    f32x4 gs = f32x4{0.f, 0.f, 0.f, 0.f}, us = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int w = 0; w < NW / 2; ++w) {
                        gs += *(const f32x4*)(src + w * TOK * 16);
                        us += *(const f32x4*)(src + w * TOK * 16 + 8);
                    }
                    // lane p keeps rows 2p, 2p+1: it sends the other pair and receives its own
                    const float g0 = (p ? gs[2] : gs[0]) + __shfl_xor(p ? gs[0] : gs[2], 1);
                    const float g1 = (p ? gs[3] : gs[1]) + __shfl_xor(p ? gs[1] : gs[3], 1);
                    const float u0 = (p ? us[2] : us[0]) + __shfl_xor(p ? us[0] : us[2], 1);
                    const float u1 = (p ? us[3] : us[1]) + __shfl_xor(p ? us[1] : us[3], 1);
                    const int jr = rt * 8 + 4 * h + 2 * p;   // first of this lane's two rows, inside the slice
                    if (MODE == MODE_FUSED) {
                        lds_write_b32_raw(a2s_addr + 2u * (unsigned)(m * geo.a2_stride + jr),
                                          pack_bf16x2(silu_mul_fast(g0, u0), silu_mul_fast(g1, u1)));
                    } else if (m < a.m_count) {
                        const size_t o = (size_t)(a.m_base + m) * a.d_ff + j0 + jr;
                        if (a.a2_is_fp32) *(float2*)((float*)a.a2 + o) = make_float2(silu_mul(g0, u0), silu_mul(g1, u1));
                        else *(uint32_t*)((uint16_t*)a.a2 + o) = pack_bf16x2(silu_mul_fast(g0, u0), silu_mul_fast(g1, u1));
                    }
                }
                DFK_WAIT_LGKM0();
                if (lane == 0) lds_write_b32_raw(sync_addr + 4u * (unsigned)(geo.sync_cap + rt), 1u);
            }
            if (++pslot == geo.slots) pslot = 0;
        }
        DFK_STAMP(2);
        if (MODE == MODE_GATEUP) return;   // every row tile's A_2 went out with its last arrival
    }

    // ---- stage two
    if (MODE == MODE_DOWN) {
        if (!a.a2_is_fp32) {
            // eight bf16 per load; slices start and end on multiples of 8 rows
            const int groups = rows_pad / 8;
            for (int idx = tid; idx < groups * TOK; idx += NTHREADS) {
                const int m = idx / groups, j = (idx - m * groups) * 8;
                u32x4 v = u32x4{0, 0, 0, 0};
                if (j < rows && m < a.m_count)
                    v = ld16((const uint16_t*)a.a2, ((size_t)(a.m_base + m) * a.d_ff + j0 + j) / 8);
                *(u32x4*)(a2s + m * geo.a2_stride + j) = v;
            }
        } else {
            for (int idx = tid; idx < rows_pad * TOK; idx += NTHREADS) {
                const int m = idx / rows_pad, j = idx - m * rows_pad;
                uint16_t v = 0;
                if (j < rows && m < a.m_count)
                    v = (uint16_t)f32_to_bf16_bits(((const float*)a.a2)[(size_t)(a.m_base + m) * a.d_ff + j0 + j]);
                lds_write_b16_raw(a2s_addr + 2u * (unsigned)(m * geo.a2_stride + j), v);
            }
        }
        lds_barrier();
    }

    // Waits (fused kernel only) until the row tiles feeding the 32-row block jb have their A_2.
    auto wait_rows_ready = [&](int jb) {
        if (MODE != MODE_FUSED) return;
        const unsigned ready = sync_addr + 4u * (unsigned)(geo.sync_cap + 4 * jb);   // 16-byte aligned
        for (;;) {
            const u32x4 f = lds_read_b128_raw(ready);
            if (__builtin_amdgcn_readfirstlane(f[0] & f[1] & f[2] & f[3]) != 0u) break;
            __builtin_amdgcn_s_sleep(1);
        }
    };

    for (int bg = 0; bg < my_blocks; bg += BG) {
        f32x4 acc2[BG][8][TT];
#pragma unroll
        for (int b = 0; b < BG; ++b)
#pragma unroll
            for (int c = 0; c < 8; ++c)
#pragma unroll
                for (int tt = 0; tt < TT; ++tt) acc2[b][c][tt] = f32x4{0.f, 0.f, 0.f, 0.f};

        // One 32-row chunk (two tiles) of one column block.
        auto chunk = [&](f32x4 (&acc)[8][TT], int jb) {
            u32x4 w[8];
            const unsigned char* sa = ts.acquire();
#pragma unroll
            for (int u = 0; u < 4; ++u) w[u] = *(const u32x4*)(sa + u * 1024 + lane * 16);
            const unsigned char* sb = ts.acquire();
#pragma unroll
            for (int u = 0; u < 4; ++u) w[4 + u] = *(const u32x4*)(sb + u * 1024 + lane * 16);
            if (jb * 32 + 32 > rows) {   // rows past the slice contribute nothing
#pragma unroll
                for (int r = 0; r < 8; ++r)
                    if (jb * 32 + 8 * g + r >= rows) w[r] = u32x4{0, 0, 0, 0};
            }
            bf16x8 av[TT];
#pragma unroll
            for (int tt = 0; tt < TT; ++tt)
                av[tt] = *(const bf16x8*)(a2s + (tt * 16 + q) * geo.a2_stride + jb * 32 + 8 * g);
#pragma unroll
            for (int c = 0; c < 8; ++c) {
                const uint32_t sel = (c & 1) ? 0x07060302u : 0x05040100u;
                u32x4 b;
#pragma unroll
                for (int p = 0; p < 4; ++p)
                    b[p] = __builtin_amdgcn_perm(w[2 * p + 1][c >> 1], w[2 * p][c >> 1], sel);
#pragma unroll
                for (int tt = 0; tt < TT; ++tt)
                    acc[c][tt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av[tt], as_bf16x8(b), acc[c][tt], 0, 0, 0);
            }
        };

        // The finished fp32 block of partial Y of one column block leaves the wavefront.
        auto flush = [&](f32x4 (&acc)[8][TT], int bi) {
            const int nb = (blk_lo + wave + bi * NW) * 128;
            if (atomic_mode) {
                // Regroup through lane permutes so that one atomic instruction covers 64
                // consecutive floats: lane L adds columns nb+L and nb+64+L of one token.
                // (Column 8q'+c of token 4g'+i sits in lane 16g'+q', register [c][tt][i].)
                for (int token = 0; token < a.m_count; ++token) {
                    const int tt = token >> 4, gsrc = (token >> 2) & 3, i = token & 3;
                    float lo = 0.f, hi = 0.f;
#pragma unroll
                    for (int c = 0; c < 8; ++c) {
                        float v = 0.f;
#pragma unroll
                        for (int t2 = 0; t2 < TT; ++t2)
#pragma unroll
                            for (int i2 = 0; i2 < 4; ++i2)
                                if (t2 == tt && i2 == i) v = acc[c][t2][i2];
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
                for (int tt = 0; tt < TT; ++tt)
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const int token = tt * 16 + 4 * g + i;
                        if (token < a.m_count) {
                            float* dst = a.P + ((size_t)pblk * a.m_count + token) * a.d_model + nb + 8 * q;
                            store4_device(dst, acc[0][tt][i], acc[1][tt][i], acc[2][tt][i], acc[3][tt][i]);
                            store4_device(dst + 4, acc[4][tt][i], acc[5][tt][i], acc[6][tt][i], acc[7][tt][i]);
                        }
                    }
            }
        };

        // first 32 rows of every block of the group
        wait_rows_ready(0);
#pragma unroll
        for (int b = 0; b < BG; ++b)
            if (bg + b < my_blocks) chunk(acc2[b], 0);
        if (bg == 0) DFK_STAMP(3);
        // then each block to its end
#pragma unroll
        for (int b = 0; b < BG; ++b) {
            if (bg + b < my_blocks) {
                for (int jb = 1; jb < njb; ++jb) {
                    if (bg == 0 && b == 0) wait_rows_ready(jb);
                    chunk(acc2[b], jb);
                }
                flush(acc2[b], bg + b);
            }
        }
    }
    DFK_STAMP(4);

    // ---- split-d_ff reduction and the bf16 store of Y
    if (atomic_mode) {
        // Per wavefront, no workgroup barrier: once its adds have been performed, the
        // wavefront counts one arrival for each 128-column block it owns (one lane per
        // block); whoever arrives last at a block reads-and-clears its accumulator
        // columns and writes them to Y.
        drain_own_memory_ops();
        const unsigned expected = MODE == MODE_DOWN ? (unsigned)a.k2_splits : (unsigned)a.splits;
        int blk = -1;
        bool won = false;
        if (lane < my_blocks) {
            blk = blk_lo + wave + lane * NW;
            won = arrive_last(a.tickets + blk, expected);
        }
        unsigned long long mask = __ballot(won);
        while (mask) {
            const int b = __builtin_ctzll(mask);
            mask &= mask - 1;
            const int nb = __shfl(blk, b) * 128;
            for (int m = 0; m < a.m_count; ++m) {
                float* src = a.yacc + (size_t)m * a.d_model + nb + 2 * lane;
                const float v0 = acc_take(src), v1 = acc_take(src + 1);
                *(uint32_t*)((uint16_t*)a.Y + (size_t)(a.m_base + m) * a.d_model + nb + 2 * lane) = pack_bf16x2(v0, v1);
            }
        }
        if (a.trace && tid == 0) a.trace[(size_t)blockIdx.x * 8 + 7] = wall_clock64();
        return;
    }
    __shared__ int flag;
    if (MODE == MODE_DOWN) {
        const int cb = blockIdx.x % a.k2_col_blocks;
        reduce_store<BF16>(plan_column_block(a, cb, blk_lo * 128, (blk_lo + blk_cnt) * 128), a.Y, a.m_base, &flag, a.trace);
    } else {
        reduce_store<BF16>(plan_full_width(a, blockIdx.x, a.splits), a.Y, a.m_base, &flag, a.trace);
    }
}

// Second kernel of the two-kernel variant, rows split over the wavefronts: workgroup
// (js, cb) owns CB <= 4 adjacent 128-column blocks of W_down over the d_ff split js;
// its wavefronts share the columns and divide the split's 32-row blocks among
// themselves.  A_2 (bf16, from the workspace) for a wavefront's rows sits in its
// registers as the MFMA A operand; the wavefronts' fp32 results meet in LDS and the
// workgroup publishes one [tokens][CB*128] block.  With few d_ff splits (8..16) the
// cross-workgroup sum is short for any number of tokens.
constexpr int kRowsModeMaxJb = 8;   // 32-row blocks per wavefront (A operand registers)

template <int NW, int TT>
__global__ __launch_bounds__(NW * 64) void k_down_rows(MlpArgs a, Geom geo) {
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    constexpr int TOK = 16 * TT;
    constexpr int NTHREADS = NW * 64;
    constexpr int BG = block_group(TT);
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int q = lane & 15, g = lane >> 4;

    const int js = blockIdx.x / a.k2_col_blocks;
    const int cb = blockIdx.x - js * a.k2_col_blocks;
    int j0, j1;
    slice_rows(a.d_ff, a.k2_splits, js, j0, j1);
    const int rows = j1 - j0;
    const int CB = a.d_model / 128 / a.k2_col_blocks;      // <= BG, checked on the host
    const int blk_lo = cb * CB;
    const int njb_all = (rows + 31) / 32;
    const int jb_lo = (int)((long long)njb_all * wave / NW);
    const int njb = (int)((long long)njb_all * (wave + 1) / NW) - jb_lo;   // <= kRowsModeMaxJb, checked on the host
    const int width = CB * 128;

    TileStream<NW, MODE_DOWN, BG> ts;
    ts.Wg = ts.Wu = nullptr; ts.Wd = (const char*)a.Wd;
    ts.d_model = a.d_model; ts.d_ff = a.d_ff;
    ts.j0 = j0; ts.nt = 0; ts.njb = njb; ts.nkc = 0;
    ts.blk_first = blk_lo; ts.blk_step = 1; ts.my_blocks = njb > 0 ? CB : 0; ts.jb_lo = jb_lo; ts.jb_major = true;
    ts.wave = wave; ts.q = q; ts.g = g;
    ts.ring = lds + wave * geo.depth * kTileBytes;
    ts.depth = geo.depth;
    ts.T1 = 0;
    ts.T = ts.my_blocks * njb * 2;
    ts.init(0);
    DFK_STAMP(3);   // the down kernel starts where A_2 is ready
    ts.start();

    // A operand: A_2[token][8 consecutive j] for every 32-row block of this wavefront
    u32x4 av[TT][kRowsModeMaxJb];
#pragma unroll
    for (int tt = 0; tt < TT; ++tt) {
        const int token = tt * 16 + q;
#pragma unroll
        for (int jbi = 0; jbi < kRowsModeMaxJb; ++jbi) {
            av[tt][jbi] = u32x4{0, 0, 0, 0};
            const int j = (jb_lo + jbi) * 32 + 8 * g;
            if (jbi < njb && token < a.m_count && j < rows)
                av[tt][jbi] = ld16((const uint16_t*)a.a2, ((size_t)(a.m_base + token) * a.d_ff + j0 + j) / 8);
        }
    }

    f32x4 acc2[BG][8][TT];
#pragma unroll
    for (int b = 0; b < BG; ++b)
#pragma unroll
        for (int c = 0; c < 8; ++c)
#pragma unroll
            for (int tt = 0; tt < TT; ++tt) acc2[b][c][tt] = f32x4{0.f, 0.f, 0.f, 0.f};

    auto chunk = [&](f32x4 (&acc)[8][TT], int jb, const u32x4 (&avj)[TT]) {
        u32x4 w[8];
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
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            const uint32_t sel = (c & 1) ? 0x07060302u : 0x05040100u;
            u32x4 b;
#pragma unroll
            for (int p = 0; p < 4; ++p) b[p] = __builtin_amdgcn_perm(w[2 * p + 1][c >> 1], w[2 * p][c >> 1], sel);
#pragma unroll
            for (int tt = 0; tt < TT; ++tt)
                acc[c][tt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(avj[tt]), as_bf16x8(b), acc[c][tt], 0, 0, 0);
        }
    };

    // same order as the tile stream: 32-row block after 32-row block, every column block each time
    for (int jbi = 0; jbi < njb; ++jbi) {
        u32x4 avj[TT];
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) {
            avj[tt] = av[tt][0];
#pragma unroll
            for (int k = 1; k < kRowsModeMaxJb; ++k)
                if (jbi == k) avj[tt] = av[tt][k];
        }
#pragma unroll
        for (int b = 0; b < BG; ++b)
            if (b < CB) chunk(acc2[b], jb_lo + jbi, avj);
    }
    DFK_STAMP(4);

    // The wavefronts' sums over their rows meet in LDS, one column block at a time:
    // each wavefront stores its [TOK][128] block into a stage of its own (the tile
    // rings are drained by now and the stages lie over them), then the workgroup adds
    // the NW stages in wavefront order and publishes the result.
    const bool atomic_mode = a.reduce_mode == DFK_REDUCE_ATOMIC;
    float* stage = (float*)lds;                           // [NW][TOK][128]
    __syncthreads();                                      // every wavefront is done with its ring
#pragma unroll
    for (int b = 0; b < BG; ++b) {
        if (b < CB) {
            float* mine = stage + (size_t)wave * TOK * 128;
#pragma unroll
            for (int tt = 0; tt < TT; ++tt)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int token = tt * 16 + 4 * g + i;
                    float* dst = mine + token * 128 + 8 * q;
                    *(f32x4*)dst = f32x4{acc2[b][0][tt][i], acc2[b][1][tt][i], acc2[b][2][tt][i], acc2[b][3][tt][i]};
                    *(f32x4*)(dst + 4) = f32x4{acc2[b][4][tt][i], acc2[b][5][tt][i], acc2[b][6][tt][i], acc2[b][7][tt][i]};
                }
            __syncthreads();
            const int nb = (blk_lo + b) * 128;
            if (atomic_mode) {
                for (int idx = tid; idx < a.m_count * 128; idx += NTHREADS) {
                    float v = 0.f;
#pragma unroll
                    for (int w = 0; w < NW; ++w) v += stage[w * TOK * 128 + idx];
                    acc_add(a.yacc + (size_t)(idx >> 7) * a.d_model + nb + (idx & 127), v);
                }
            } else {
                for (int idx = tid; idx < a.m_count * 32; idx += NTHREADS) {
                    f32x4 v = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int w = 0; w < NW; ++w) v += *(const f32x4*)(stage + w * TOK * 128 + 4 * idx);
                    const int m = idx >> 5, c4 = idx & 31;
                    store4_device(a.P + ((size_t)js * a.m_count + m) * a.d_model + nb + 4 * c4, v[0], v[1], v[2], v[3]);
                }
            }
            __syncthreads();                              // stages are rewritten by the next column block
        }
    }
    __shared__ int flag;
    if (atomic_mode) {
        drain_own_memory_ops();
        __syncthreads();
        if (tid == 0) flag = arrive_last(a.tickets + cb, (unsigned)a.k2_splits) ? 1 : 0;
        __syncthreads();
        if (!flag) return;
        for (int idx = tid; idx < a.m_count * (width / 2); idx += NTHREADS) {
            const int m = idx / (width / 2), c2 = idx - m * (width / 2);
            float* src = a.yacc + (size_t)m * a.d_model + blk_lo * 128 + 2 * c2;
            const float v0 = acc_take(src), v1 = acc_take(src + 1);
            *(uint32_t*)((uint16_t*)a.Y + (size_t)(a.m_base + m) * a.d_model + blk_lo * 128 + 2 * c2) = pack_bf16x2(v0, v1);
        }
        return;
    }
    reduce_store<BF16>(plan_column_block(a, cb, blk_lo * 128, blk_lo * 128 + width), a.Y, a.m_base, &flag, a.trace);
}

struct Sizes {
    Geom geo;
    size_t lds;
};

// token tiles (of 16) per launch: two if the wavefront can hold X for both, else one
int max_token_tiles(const dfk_config_t& c, int d_model) {
    const int nkc = d_model / c.waves / kKC;
    return 2 * nkc <= x_chunk_cap(c.waves) ? 2 : 1;
}
int token_tiles(const dfk_config_t& c, int m_count) { return m_count <= 16 ? 1 : 2; }

Sizes sizes(const dfk_config_t& c, int mode, int TT, int d_ff, int d_model) {
    Sizes s;
    const int S = (mode == MODE_DOWN || mode == MODE_DOWN_ROWS) ? c.k2_splits : c.splits;
    const int maxrows = max_slice_rows(d_ff, S);
    const int rows_pad = (maxrows + 31) & ~31;
    const int TOK = 16 * TT;
    size_t off = (size_t)c.waves * c.depth * kTileBytes;
    s.geo.depth = c.depth;
    s.geo.gu_off = (int)off;
    if (mode == MODE_DOWN_ROWS) {   // the [waves][TOK][128] fp32 stages overlay the drained rings
        off = std::max(off, (size_t)c.waves * TOK * 128 * 4);
        s.geo.a2s_off = s.geo.sync_off = (int)off;
        s.geo.a2_stride = 0;
        s.geo.sync_cap = 0;
        s.lds = off;
        return s;
    }
    // stage one: what is left of LDS after rings, A_2 and flags holds the k-partial sums of as
    // many row tiles as fit (at most kMaxPartialSlots; at least two, or the configuration is invalid)
    const size_t slot_bytes = (size_t)c.waves * TOK * 16 * 4;
    const size_t a2s_bytes = (size_t)TOK * (rows_pad + 8) * 2;
    s.geo.sync_cap = ((maxrows / 8 + 4) + 3) & ~3;
    const size_t sync_bytes = (size_t)2 * s.geo.sync_cap * 4;
    s.geo.slots = 0;
    if (mode != MODE_DOWN) {
        const size_t fixed = off + (mode == MODE_FUSED ? a2s_bytes : 0) + sync_bytes + 16;
        const int nt_max = maxrows / 8;
        const size_t fit = (size_t)kLdsLimit > fixed ? ((size_t)kLdsLimit - fixed) / slot_bytes : 0;
        s.geo.slots = (int)std::min<size_t>((size_t)std::min(nt_max, kMaxPartialSlots), fit);
        if (s.geo.slots < std::min(nt_max, 2)) { s.lds = (size_t)-1; return s; }   // does not fit
        off += (size_t)s.geo.slots * slot_bytes;
    }
    s.geo.a2s_off = (int)off;
    s.geo.a2_stride = rows_pad + 8;
    if (mode != MODE_GATEUP) off += a2s_bytes;
    off = (off + 15) & ~(size_t)15;
    s.geo.sync_off = (int)off;
    if (mode != MODE_DOWN) off += sync_bytes;
    s.lds = off;
    return s;
}

template <int NW, int TT, int MODE>
hipError_t launch_one(const MlpArgs& a, const dfk_config_t& c, int grid, hipStream_t st) {
    static LdsAllowance allowed;   // of this instantiation, per device
    const Sizes s = sizes(c, MODE, TT, a.d_ff, a.d_model);
    const void* fn = MODE == MODE_DOWN_ROWS ? (const void*)k_down_rows<NW, TT> : (const void*)k_mfma<NW, TT, MODE == MODE_DOWN_ROWS ? MODE_DOWN : MODE>;
    if (hipError_t e = allow_lds(allowed, fn, s.lds); e != hipSuccess) return e;
    if (MODE == MODE_DOWN_ROWS)
        hipLaunchKernelGGL((k_down_rows<NW, TT>), dim3(grid), dim3(NW * 64), s.lds, st, a, s.geo);
    else
        hipLaunchKernelGGL((k_mfma<NW, TT, MODE == MODE_DOWN_ROWS ? MODE_DOWN : MODE>), dim3(grid), dim3(NW * 64), s.lds, st, a, s.geo);
    return hipGetLastError();
}

template <int NW, int TT>
hipError_t launch_nt(const MlpArgs& a, const dfk_config_t& c, hipStream_t st) {
    if (c.variant == DFK_VARIANT_FUSED)
        return (g_stage_mask & 1) ? launch_one<NW, TT, MODE_FUSED>(a, c, a.splits, st) : hipSuccess;
    if (g_stage_mask & 1) {
        hipError_t e = launch_one<NW, TT, MODE_GATEUP>(a, c, a.splits, st);
        if (e != hipSuccess) return e;
    }
    if (!(g_stage_mask & 2)) return hipSuccess;
    if (c.k2_rows_by_wave) return launch_one<NW, TT, MODE_DOWN_ROWS>(a, c, a.k2_splits * a.k2_col_blocks, st);
    return launch_one<NW, TT, MODE_DOWN>(a, c, a.k2_splits * a.k2_col_blocks, st);
}

}  // namespace

// The mixed pair for 33..64 tokens (kmajor = 3): gate/up kernel with workgroup-shared weight tiles (four
// wavefronts, one token tile each), down kernel of the 64-token pair.
dfk_config_t mixed_gateup_cfg(const dfk_config_t& c) { dfk_config_t g = c; g.waves = 4; g.kmajor = 2; return g; }
dfk_config_t mixed_down_cfg(const dfk_config_t& c) { dfk_config_t d = c; d.kmajor = 1; return d; }

bool mfma_mixed_config_valid(const dfk_config_t& c, int M, int d_model, int d_ff, dfk_dtype_t dtype) {
    if (c.variant != DFK_VARIANT_TWO_KERNEL || c.kmajor != 3 || c.waves != 8) return false;
    return mfma_km_config_valid(mixed_down_cfg(c), M, d_model, d_ff, dtype) && big_gateup_64_fits(mixed_gateup_cfg(c), d_model, d_ff);
}

hipError_t launch_mfma_mixed(const MlpArgs& a, const dfk_config_t& c, hipStream_t st) {
    if (g_stage_mask & 1) {
        if (hipError_t e = launch_big_gateup_64(a, mixed_gateup_cfg(c), st); e != hipSuccess) return e;
    }
    if (!(g_stage_mask & 2)) return hipSuccess;
    const int saved = g_stage_mask;
    g_stage_mask = 2;                                  // the down kernel only
    const hipError_t e = launch_mfma_km(a, mixed_down_cfg(c), st);
    g_stage_mask = saved;
    return e;
}

int mfma_max_tokens_per_launch(const dfk_config_t& c, int d_model) {
    if (c.kmajor == 4 || c.kmajor == 5) return mfma_km_tokens_per_launch();
    if (c.kmajor == 3) return mfma_km_tokens_per_launch();
    if (c.kmajor == 2) return mfma_big_tokens_per_launch();
    if (c.kmajor == 1 && c.variant == DFK_VARIANT_FUSED) return mfma_fused_km_tokens_per_launch();
    return c.kmajor ? mfma_km_tokens_per_launch() : 16 * max_token_tiles(c, d_model);
}

bool mfma_config_valid(const dfk_config_t& c, int M, int d_model, int d_ff, dfk_dtype_t dtype) {
    if (c.kmajor == 4) return mfma_km_roles_config_valid(c, M, d_model, d_ff, dtype);
    if (c.kmajor == 5) return mfma_km_t_config_valid(c, M, d_model, d_ff, dtype);
    if (c.kmajor == 3) return mfma_mixed_config_valid(c, M, d_model, d_ff, dtype);
    if (c.kmajor == 2) return mfma_big_config_valid(c, M, d_model, d_ff, dtype);
    if (c.kmajor == 1 && c.variant == DFK_VARIANT_FUSED) return mfma_fused_km_config_valid(c, M, d_model, d_ff, dtype);
    if (c.kmajor) return mfma_km_config_valid(c, M, d_model, d_ff, dtype);
    if (c.path != DFK_PATH_MFMA || dtype != DFK_BF16) return false;
    if (c.variant != DFK_VARIANT_FUSED && c.variant != DFK_VARIANT_TWO_KERNEL) return false;
    if (c.reduce != DFK_REDUCE_TICKET && c.reduce != DFK_REDUCE_ATOMIC) return false;
    if (d_model > kMaxDModel) return false;
    if (c.waves != 4 && c.waves != 8) return false;   // one or two wavefronts per SIMD
    if (c.depth < 2 || c.depth > 16) return false;
    if (M < 1 || d_model < 8 || d_ff < 8 || d_ff % 8) return false;
    if (d_model % (kKC * c.waves)) return false;   // each wavefront owns whole 128-k chunks
    const int ng = d_ff / 8;
    if (c.splits < 1 || c.splits > ng) return false;
    if (d_model / c.waves / kKC > x_chunk_cap(c.waves)) return false;   // X of a wavefront's k range must fit its registers
    const int per = mfma_max_tokens_per_launch(c, d_model);
    const int TT = token_tiles(c, M < per ? M : per);
    const int tokens = M < per ? M : per;
    const bool ticket = c.reduce == DFK_REDUCE_TICKET;
    if (c.variant == DFK_VARIANT_FUSED)
        return (!ticket || ((c.splits + kGroupSize - 1) / kGroupSize <= kTicketLevel2 &&
                            partials_fit(c.splits, tokens, M, d_model))) &&
               sizes(c, MODE_FUSED, TT, d_ff, d_model).lds <= (size_t)kLdsLimit;
    if (c.k2_splits < 1 || c.k2_splits > ng) return false;
    const int nblk = d_model / 128;
    if (c.k2_col_blocks < 1 || nblk % c.k2_col_blocks) return false;
    if ((long long)c.k2_splits * c.k2_col_blocks > 65535 || c.k2_col_blocks > kTicketLevel2) return false;
    if (ticket && !partials_fit(c.k2_splits, tokens, M, d_model)) return false;
    if (c.a2_dtype != DFK_BF16 && c.a2_dtype != DFK_FP32) return false;
    if (sizes(c, MODE_GATEUP, TT, d_ff, d_model).lds > (size_t)kLdsLimit) return false;
    if (c.k2_rows_by_wave) {
        if (c.k2_rows_by_wave != 1 || c.a2_dtype != DFK_BF16) return false;
        if (nblk / c.k2_col_blocks > block_group(TT)) return false;             // accumulators of the column blocks
        const int njb_all = (max_slice_rows(d_ff, c.k2_splits) + 31) / 32;
        if ((njb_all + c.waves - 1) / c.waves > kRowsModeMaxJb) return false;   // A operand registers
        return sizes(c, MODE_DOWN_ROWS, TT, d_ff, d_model).lds <= (size_t)kLdsLimit;
    }
    return sizes(c, MODE_DOWN, TT, d_ff, d_model).lds <= (size_t)kLdsLimit;
}

hipError_t launch_mfma(const MlpArgs& a, const dfk_config_t& c, hipStream_t st) {
    if (c.kmajor == 4) return launch_mfma_km_roles(a, c, st);
    if (c.kmajor == 3) return launch_mfma_mixed(a, c, st);
    if (c.kmajor == 2) return launch_mfma_big(a, c, st);
    if (c.kmajor == 1 && c.variant == DFK_VARIANT_FUSED) return launch_mfma_fused_km(a, c, st);
    if (c.kmajor) return launch_mfma_km(a, c, st);
    const int TT = token_tiles(c, a.m_count);
    switch (c.waves * 10 + TT) {
        case 41: return launch_nt<4, 1>(a, c, st);
        case 42: return launch_nt<4, 2>(a, c, st);
        case 81: return launch_nt<8, 1>(a, c, st);
        case 82: return launch_nt<8, 2>(a, c, st);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace dfk
