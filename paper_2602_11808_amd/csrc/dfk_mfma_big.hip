// MFMA kernels of the two-kernel variant for 65..256 tokens per launch (gfx950).
//
// With more than 64 tokens the block stops being a matrix-vector stream: per weight tile
// there are 8..16 token tiles of MFMA work, too many accumulators for one wavefront and too
// much operand traffic if every wavefront fetched its own copy of the weights.  These
// kernels are the "row-major" end of the Method section's tiling choice carried through:
// the wavefronts of a workgroup (four or eight in the gate/up kernel, eight in the down kernel) share
// every weight tile through LDS, each wavefront owns its share of the launch's tokens (1, 2
// or 4 token tiles of 16) and keeps the whole reduction for them, so there is no
// cross-wavefront sum at the end.
//
// Data movement is the same asynchronous global->LDS tile load as in the other MFMA kernels,
// organised as a workgroup pipeline instead of per-wavefront rings:
//   * shared tiles (weights): 4 KB tiles of the usual layout; the 1 KB load instructions of a
//     step's tiles are dealt out evenly, so the wavefronts fill the tiles together and issue
//     the same number of loads.  `nb` buffers of one pipeline step each.
//   * private tiles (activations of the wavefront's own tokens): loaded and read by one
//     wavefront only, `pl` buffers per wavefront.
//   * one LDS-only barrier per step: before it every wavefront waits, by count, for its own
//     loads of the step (loads complete in issue order; the kernel keeps the running count of
//     issued loads and the count at which each step's loads were complete); after it the
//     step's shared tiles are whole and the buffer of the step before is free to refill.
//
// Gate/up kernel: workgroup s owns a d_ff slice of at most 8 row tiles (8 rows of W_gate and
// the same 8 of W_up per tile); a step is one 128-k chunk: the slice's weight tiles (shared)
// and the wavefront's token tiles of X (private, read into registers as MFMA B operands at
// the start of the step).  The D tile of a row tile holds gate rows in lanes 0..31 and up
// rows in lanes 32..63 of the same token: one cross-lane exchange, SiLU(G)*U, store of A_2.
//
// Down kernel: workgroup (js, cb) owns one 128-column block over d_ff split js; a step is
// two 32-row blocks of W_down (shared, regrouped per lane with v_perm_b32 as in the other
// down kernels) and the wavefront's A_2 tiles for those rows (private).  Each wavefront
// publishes its finished [tokens x 128] sums itself (partial block of the split, or the
// fp32 accumulator); the cross-workgroup reduction is that of the other kernels.
#include <atomic>
#include <algorithm>

#include "dfk_mfma_common.h"

namespace dfk {
namespace {

constexpr int kBigWaves = 4;          // gate/up kernel: 4 or 8; token tiles per wavefront are counted for 4
constexpr int kBigDownWaves = 8;      // down kernel: two wavefronts per SIMD, so that one's operand shuffles
                                      // (v_perm_b32) run under the other's MFMAs
constexpr int kBigMaxRowTiles = 8;
constexpr int kBigTokensPerLaunch = 256;
constexpr int kBigSB = 2;            // 32-row blocks of W_down per step of the down kernel (the A_2 tile layout assumes 2)

constexpr size_t kL2BytesPerXcd = (size_t)4 << 20;

struct BigGeom {
    int nb;          // buffers of shared tiles (steps)
    int pl;          // private buffers per wavefront (1 or 2)
    int shared_step; // bytes of one shared buffer
    int priv_off;    // byte offset of the private region
    int priv_step;   // bytes of one private buffer
    int by_xcd;      // down kernel: place the workgroups of a d_ff split on one XCD (see down_tile_of)
};

// s_waitcnt vmcnt(n) for a run-time n (uniform); more than 63 waits for 63.
__device__ __forceinline__ void wait_vm_exact(int n) {
#define DFK_VM_CASE(k) case k: DFK_WAIT_VM(k); break;
#define DFK_VM_CASE8(k) DFK_VM_CASE(k) DFK_VM_CASE(k + 1) DFK_VM_CASE(k + 2) DFK_VM_CASE(k + 3) \
                        DFK_VM_CASE(k + 4) DFK_VM_CASE(k + 5) DFK_VM_CASE(k + 6) DFK_VM_CASE(k + 7)
    switch (n) {
        DFK_VM_CASE8(0) DFK_VM_CASE8(8) DFK_VM_CASE8(16) DFK_VM_CASE8(24)
        DFK_VM_CASE8(32) DFK_VM_CASE8(40) DFK_VM_CASE8(48)
        DFK_VM_CASE(56) DFK_VM_CASE(57) DFK_VM_CASE(58) DFK_VM_CASE(59) DFK_VM_CASE(60) DFK_VM_CASE(61) DFK_VM_CASE(62)
        default: DFK_WAIT_VM(63); break;
    }
#undef DFK_VM_CASE8
#undef DFK_VM_CASE
    asm volatile("" ::: "memory");
}

// Bookkeeping of the workgroup pipeline, plain wave-uniform ints in the kernels (kept out of
// any struct that is passed around: that ended up in scratch memory, whose loads drain the
// tile loads): `issued` counts this wavefront's tile-load instructions; p_mark<i> / s_mark<i> is
// that count right after the loads of the private / shared tiles of step (current + i) were
// issued (0: none issued, nothing to wait for).
#define DFK_PIPE_DECL() int issued = 0, p_mark0 = 0, p_mark1 = 0, s_mark0 = 0, s_mark1 = 0, s_mark2 = 0
#define DFK_PIPE_SET_P(ahead) do { if ((ahead) == 0) p_mark0 = issued; else p_mark1 = issued; } while (0)
#define DFK_PIPE_SET_S(ahead) do { if ((ahead) == 0) s_mark0 = issued; else if ((ahead) == 1) s_mark1 = issued; else s_mark2 = issued; } while (0)
// Wait for this wavefront's loads of the current step, meet the other wavefronts, move on one step.
#define DFK_PIPE_ENTER_STEP() do {                                             \
        wait_vm_exact(issued - max(p_mark0, s_mark0));                          \
        lds_barrier();                                                          \
        p_mark0 = p_mark1; p_mark1 = 0;                                         \
        s_mark0 = s_mark1; s_mark1 = s_mark2; s_mark2 = 0;                      \
    } while (0)

// ---------------------------------------------------------------- gate/up kernel
template <int TT, int NW>
struct BigLoads1 {
    const char* wsrc;          // this lane's address in the slice's first weight tile, chunk 0
    const char* xsrc[TT][4];   // this lane's addresses in the wavefront's X tiles, chunk 0
    size_t row_bytes;
    int nt, wave;
    unsigned char *lds, *xpriv;
    int shared_step, priv_step;

    __device__ __forceinline__ int issue_x(int kc, int buf) {
        unsigned char* dst = xpriv + (size_t)buf * priv_step;
#pragma unroll
        for (int tt = 0; tt < TT; ++tt)
#pragma unroll
            for (int u = 0; u < 4; ++u)
                __builtin_amdgcn_global_load_lds(xsrc[tt][u] + (size_t)kc * (kKC * 2), DFK_LDS_PTR(dst + tt * kTileBytes + u * 1024), 16, 0, 0);
        return 4 * TT;
    }
    // 4 wavefronts: each issues its instruction (wave) of every tile; 8: instruction wave % 4 of
    // the tiles of parity wave / 4
    __device__ __forceinline__ int issue_w(int kc, int buf) {
        unsigned char* dst = lds + (size_t)buf * shared_step + (wave & 3) * 1024;
        int n = 0;
        for (int rt = NW == 8 ? (wave >> 2) : 0; rt < nt; rt += NW == 8 ? 2 : 1) {
            __builtin_amdgcn_global_load_lds(wsrc + (size_t)rt * 8 * row_bytes + (size_t)kc * (kKC * 2), DFK_LDS_PTR(dst + rt * kTileBytes), 16, 0,
                                             kAuxNonTemporal);
            ++n;
        }
        return n;
    }
};

// MFMAs of one 128-k chunk for NTC row tiles: the A operands (weight tile rows) are read from
// LDS one row tile ahead of their use, so that the read latency hides behind the MFMAs of the
// tile before.  wt points at this lane's row (q) of the chunk's first weight tile.
template <int NTC, int TT, typename E>
__device__ __forceinline__ void gateup_chunk(f32x4 (&acc)[NTC][TT], const u32x4 (&xk)[TT][4], const unsigned char* wt, int q, int g,
                                             bool last_present) {
    u32x4 av[2][4];
#pragma unroll
    for (int c = 0; c < 4; ++c) av[0][c] = *(const u32x4*)(wt + (((4 * c + g) ^ q)) * 16);
#pragma unroll
    for (int rt = 0; rt < NTC; ++rt) {
        if (rt + 1 < NTC) {   // (the last tile's buffer exists in every workgroup; its data is used only where present)
#pragma unroll
            for (int c = 0; c < 4; ++c) av[(rt + 1) & 1][c] = *(const u32x4*)(wt + (rt + 1) * kTileBytes + (((4 * c + g) ^ q)) * 16);
        }
        // keep the four reads above ahead of this tile's MFMAs (the scheduler otherwise moves each
        // read next to its use, two MFMAs before a full LDS wait)
        __builtin_amdgcn_sched_barrier(0);
        if (rt + 1 < NTC || last_present) {
#pragma unroll
            for (int c = 0; c < 4; ++c)
#pragma unroll
                for (int tt = 0; tt < TT; ++tt) acc[rt][tt] = mfma16<E>(av[rt & 1][c], xk[tt][c], acc[rt][tt]);
        }
        __builtin_amdgcn_sched_barrier(0);
    }
}

// NTC: the largest row-tile count of a d_ff slice of the launch (a compile-time constant so that
// the chunk body is straight-line code); every slice has NTC or NTC - 1 row tiles.
template <int TT, typename E, int NTC, int NW>
__global__ __launch_bounds__(NW * 64) void k_gateup_big(MlpArgs a, BigGeom geo) {
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    constexpr int NT = NTC;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int q = lane & 15, g = lane >> 4;
    int j0, j1;
    slice_rows(a.d_ff, a.splits, blockIdx.x, j0, j1);
    const int nt = (j1 - j0) / 8;                  // NTC or NTC - 1 (slices differ by at most one 8-row group)
    const int nkc = a.d_model / kKC;
    const size_t row_bytes = (size_t)a.d_model * 2;
    const int tile0 = wave * TT;                   // this wavefront's first token tile

    BigLoads1<TT, NW> ld;
    ld.row_bytes = row_bytes; ld.nt = nt; ld.wave = wave; ld.lds = lds;
    ld.shared_step = geo.shared_step; ld.priv_step = geo.priv_step;
    // this wavefront's instruction of a weight tile: tile row i = 4*wave + g, 16-byte chunk q ^ i
    const int iw = 4 * (wave & 3) + g;
    ld.wsrc = (const char*)((wave & 3) < 2 ? a.Wg : a.Wu) + (size_t)j0 * row_bytes + (size_t)(iw & 7) * row_bytes + ((q ^ iw) * 16);
    // X tile: instruction u covers tile rows (tokens) 4u + g
#pragma unroll
    for (int tt = 0; tt < TT; ++tt)
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int i = 4 * u + g;
            const int token = min((tile0 + tt) * 16 + i, a.m_count - 1);
            ld.xsrc[tt][u] = (const char*)a.X + (size_t)(a.m_base + token) * row_bytes + ((q ^ i) * 16);
        }
    unsigned char* xpriv = lds + geo.priv_off + (size_t)wave * geo.pl * geo.priv_step;
    ld.xpriv = xpriv;

    DFK_PIPE_DECL();
    DFK_STAMP(0);
    // Every workgroup walks the k chunks in its own rotation: all of them read the same X, and in
    // lock-step they would ask the same few L2 channels for the same lines at the same moment.
    const int rot = (int)((blockIdx.x * 7u) % (unsigned)nkc);
#define DFK_KC(step) (((step) + rot) < nkc ? (step) + rot : (step) + rot - nkc)
    // prologue: X of the first pl steps, weights of the first nb - 1, earliest needs first
    {
        int xs = 0, ws = 0;
        for (int s = 0; s < 3; ++s) {
            if (xs < geo.pl && xs < nkc && xs <= s) { issued += ld.issue_x(DFK_KC(xs), xs); DFK_PIPE_SET_P(xs); ++xs; }
            if (ws < geo.nb - 1 && ws < nkc && ws <= s) { issued += ld.issue_w(DFK_KC(ws), ws); DFK_PIPE_SET_S(ws); ++ws; }
        }
    }

    f32x4 acc[NT][TT];
#pragma unroll
    for (int rt = 0; rt < NT; ++rt)
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) acc[rt][tt] = f32x4{0.f, 0.f, 0.f, 0.f};

    int xbuf = 0, wbuf = 0;                        // buffers of the current step
    int wfree = geo.nb - 1;                        // shared buffer the step nb-1 ahead goes to
    for (int kc = 0; kc < nkc; ++kc) {
        DFK_PIPE_ENTER_STEP();
        u32x4 xk[TT][4];       // B operands of the chunk: token q of each of the wavefront's token tiles
        {
            const unsigned char* xs = xpriv + (size_t)xbuf * geo.priv_step;
#pragma unroll
            for (int tt = 0; tt < TT; ++tt)
#pragma unroll
                for (int c = 0; c < 4; ++c) xk[tt][c] = *(const u32x4*)(xs + tt * kTileBytes + (q * 16 + ((4 * c + g) ^ q)) * 16);
        }
        DFK_WAIT_LGKM0();      // the X buffer has been read: it may be refilled
        asm volatile("" ::: "memory");
        if (kc + geo.pl < nkc) { issued += ld.issue_x(DFK_KC(kc + geo.pl), xbuf); DFK_PIPE_SET_P(geo.pl - 1); }
        if (kc + geo.nb - 1 < nkc) { issued += ld.issue_w(DFK_KC(kc + geo.nb - 1), wfree); DFK_PIPE_SET_S(geo.nb - 2); }
        const unsigned char* wt = lds + (size_t)wbuf * geo.shared_step + (q * 16) * 16;
        gateup_chunk<NTC, TT, E>(acc, xk, wt, q, g, nt == NTC);
        if (++xbuf == geo.pl) xbuf = 0;
        if (++wbuf == geo.nb) wbuf = 0;
        if (++wfree == geo.nb) wfree = 0;
    }
#undef DFK_KC
    DFK_STAMP(2);

    // D tile of (row tile, token tile): lane (q, g) holds token q, tile rows 4g .. 4g+3; rows 0..7
    // are the gate rows, 8..15 the up rows of the same 8 d_ff rows: lanes 32 apart pair up.
#pragma unroll
    for (int rt = 0; rt < NT; ++rt) {
        if (rt < nt) {
#pragma unroll
            for (int tt = 0; tt < TT; ++tt) {
                const f32x4 v = acc[rt][tt];
                float o[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) o[i] = __shfl_xor(v[i], 32);
                const int m = (tile0 + tt) * 16 + q;
                if (g < 2 && m < a.m_count) {
                    uint2 pk;
                    pk.x = E::pack2(silu_mul_fast(v[0], o[0]), silu_mul_fast(v[1], o[1]));
                    pk.y = E::pack2(silu_mul_fast(v[2], o[2]), silu_mul_fast(v[3], o[3]));
                    *(uint2*)((uint16_t*)a.a2 + (size_t)(a.m_base + m) * a.d_ff + j0 + rt * 8 + 4 * g) = pk;
                }
            }
        }
    }
    DFK_STAMP(1);
}

// ---------------------------------------------------------------- down kernel
template <int TT, int NW>
struct BigLoads2 {
    const char* asrc[TT][2];   // this lane's token rows of A_2 at the split's first row (per load instruction)
    const char* Wd;
    size_t row_bytes, colb;
    int j0, rows, njb, d_ff, wave, q, g, lane;
    unsigned char *lds, *apriv;
    int shared_step, priv_step;

    // A_2 of a step (64 rows = 128 contiguous bytes per token), 2 KB per token tile: instruction h
    // covers tokens 8h .. 8h+7 of the tile, 8 consecutive lanes one token's 128 bytes (a whole
    // cache line per token); within a token the eight 16-byte chunks sit XOR-swizzled by the
    // token so that the operand reads below spread over the LDS banks.
    __device__ __forceinline__ int issue_a(int s, int buf) {
        unsigned char* dst = apriv + (size_t)buf * priv_step;
        const int chunk = (lane & 7) ^ ((lane >> 3) & 7);
        const int j = min(s * 64 + 8 * chunk, rows - 8);   // past the split: any valid address (masked at use)
#pragma unroll
        for (int tt = 0; tt < TT; ++tt)
#pragma unroll
            for (int h = 0; h < 2; ++h)
                __builtin_amdgcn_global_load_lds(asrc[tt][h] + (size_t)j * 2, DFK_LDS_PTR(dst + tt * 2048 + h * 1024), 16, 0, 0);
        return 2 * TT;
    }
    // W_down tiles of a 32-row block: tile h (0, 1) holds rows 4h + 8g + u for instruction u.  The
    // 8 instructions of a block are dealt out evenly: with 4 wavefronts each issues instruction
    // u = wave of both tiles, with 8 wavefronts instruction wave % 4 of tile wave / 4.
    __device__ __forceinline__ int issue_w(int s, int buf) {
        const int u = wave & 3;
        unsigned char* dst = lds + (size_t)buf * shared_step + u * 1024;
        int n = 0;
        for (int b = 0; b < kBigSB; ++b) {
            const int jb = s * kBigSB + b;
            if (jb < njb) {
#pragma unroll
                for (int hh = 0; hh < (NW == 8 ? 1 : 2); ++hh) {
                    const int h = NW == 8 ? (wave >> 2) : hh;
                    const int row = min(j0 + jb * 32 + 4 * h + 8 * g + u, d_ff - 1);   // past d_ff: masked at use
                    __builtin_amdgcn_global_load_lds(Wd + (size_t)row * row_bytes + colb + 16 * q,
                                                     DFK_LDS_PTR(dst + (b * 2 + h) * kTileBytes), 16, 0, kAuxNonTemporal);
                }
                n += NW == 8 ? 1 : 2;
            }
        }
        return n;
    }
};

// Which (d_ff split, column block) a workgroup of the down kernel takes.  Workgroups are handed to
// the 8 XCDs in turn (workgroup b runs on XCD b % 8) and each XCD has its own L2; all column blocks
// of a split read the same A_2 rows, so a split's workgroups are placed on one XCD (or, with fewer
// than 8 splits, on 8 / splits of them) and those rows are fetched into that L2 once.  Any other
// split count keeps the plain order, and so does a launch whose whole A_2 fits one L2 (the host
// decides: there the plain order measured 2 us faster, at 128 tokens of the 8B shape; beyond,
// the placement gains 1 to 4 us of 60 at 256 tokens of that shape and 13 of 200 on the 70B
// shape).  A bijection from
// [0, S * C) onto S x C in every case.
__device__ __forceinline__ void down_tile_of(int b, int S, int C, bool by_xcd, int& js, int& cb) {
    const int x = b & 7, r = b >> 3;
    if (!by_xcd) {
        js = b / C;
        cb = b - js * C;
    } else if ((S & 7) == 0) {
        js = x + 8 * (r / C);
        cb = r % C;
    } else if ((S == 1 || S == 2 || S == 4) && ((C * S) & 7) == 0) {
        js = x % S;
        cb = (x / S) * (C * S / 8) + r;
    } else {
        js = b / C;
        cb = b - js * C;
    }
}

template <int TT, typename E, int NW>
__global__ __launch_bounds__(NW * 64) void k_down_big(MlpArgs a, BigGeom geo) {
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    __shared__ int flag;
    static_assert(NW == 4 || NW == 8, "shared tiles are dealt out to 4 or 8 wavefronts");
    constexpr int NTHREADS = NW * 64;
    constexpr int SB = kBigSB;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int q = lane & 15, g = lane >> 4;
    int js, cb;   // d_ff split and 128-column block of this workgroup (one column block each: checked on the host)
    down_tile_of((int)blockIdx.x, a.k2_splits, a.k2_col_blocks, geo.by_xcd != 0, js, cb);
    int j0, j1;
    slice_rows(a.d_ff, a.k2_splits, js, j0, j1);
    const int rows = j1 - j0;
    const int njb = (rows + 31) / 32;
    const int nsteps = (njb + SB - 1) / SB;
    const size_t row_bytes = (size_t)a.d_model * 2;
    const int tile0 = wave * TT;
    const size_t colb = (size_t)cb * 256;

    BigLoads2<TT, NW> ld;
    ld.Wd = (const char*)a.Wd; ld.row_bytes = row_bytes; ld.colb = colb;
    ld.j0 = j0; ld.rows = rows; ld.njb = njb; ld.d_ff = a.d_ff; ld.wave = wave; ld.q = q; ld.g = g;
    ld.lds = lds; ld.shared_step = geo.shared_step; ld.priv_step = geo.priv_step;
    ld.lane = lane;
#pragma unroll
    for (int tt = 0; tt < TT; ++tt)
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int token = min((tile0 + tt) * 16 + 8 * h + (lane >> 3), a.m_count - 1);
            ld.asrc[tt][h] = (const char*)a.a2 + ((size_t)(a.m_base + token) * a.d_ff + j0) * 2;
        }
    unsigned char* apriv = lds + geo.priv_off + (size_t)wave * geo.pl * geo.priv_step;
    ld.apriv = apriv;

    DFK_PIPE_DECL();
    DFK_STAMP(3);
    // The workgroups of one split read the same A_2 rows: each walks the steps in its own rotation.
    const int rot = (int)((cb * 5u) % (unsigned)nsteps);
#define DFK_ST(step) (((step) + rot) < nsteps ? (step) + rot : (step) + rot - nsteps)
    {
        int as = 0, ws = 0;
        for (int s = 0; s < 3; ++s) {
            if (as < geo.pl && as < nsteps && as <= s) { issued += ld.issue_a(DFK_ST(as), as); DFK_PIPE_SET_P(as); ++as; }
            if (ws < geo.nb - 1 && ws < nsteps && ws <= s) { issued += ld.issue_w(DFK_ST(ws), ws); DFK_PIPE_SET_S(ws); ++ws; }
        }
    }

    f32x4 acc2[8][TT];
#pragma unroll
    for (int c = 0; c < 8; ++c)
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) acc2[c][tt] = f32x4{0.f, 0.f, 0.f, 0.f};

    int abuf = 0, wbuf = 0, wfree = geo.nb - 1;
    for (int s = 0; s < nsteps; ++s) {
        const int se = DFK_ST(s);   // the rows this step covers: 64 se .. 64 se + 63 of the split
        DFK_PIPE_ENTER_STEP();
        u32x4 av[SB][TT];      // A operands: A_2[token q of tile tt][rows 8g .. 8g+7 of block b]
        {
            // token q of the tile sits in instruction q / 8 at lanes 8 (q % 8) .. +7, chunk k at (k ^ (q % 8))
            const unsigned char* as = apriv + (size_t)abuf * geo.priv_step + (q >> 3) * 1024 + (q & 7) * 128;
#pragma unroll
            for (int b = 0; b < SB; ++b) {
                const int k = 4 * b + g;
#pragma unroll
                for (int tt = 0; tt < TT; ++tt) av[b][tt] = *(const u32x4*)(as + tt * 2048 + ((k ^ (q & 7)) * 16));
            }
            if ((se + 1) * SB * 32 > rows) {   // only the split's last 64 rows can reach past it
#pragma unroll
                for (int b = 0; b < SB; ++b) {
                    const bool past = (se * SB + b) * 32 + 8 * g >= rows;
#pragma unroll
                    for (int tt = 0; tt < TT; ++tt)
                        if (past) av[b][tt] = u32x4{0, 0, 0, 0};
                }
            }
        }
        DFK_WAIT_LGKM0();
        asm volatile("" ::: "memory");
        if (s + geo.pl < nsteps) { issued += ld.issue_a(DFK_ST(s + geo.pl), abuf); DFK_PIPE_SET_P(geo.pl - 1); }
        if (s + geo.nb - 1 < nsteps) { issued += ld.issue_w(DFK_ST(s + geo.nb - 1), wfree); DFK_PIPE_SET_S(geo.nb - 2); }
        // Both blocks of the step are read and multiplied unconditionally: a block past the split
        // has every row masked to zero below and its A operands zeroed above.
        const unsigned char* wt = lds + (size_t)wbuf * geo.shared_step + lane * 16;
        u32x4 w[SB][8];
#pragma unroll
        for (int b = 0; b < SB; ++b)
#pragma unroll
            for (int r = 0; r < 8; ++r) w[b][r] = *(const u32x4*)(wt + (b * 2 + (r >> 2)) * kTileBytes + (r & 3) * 1024);
#pragma unroll
        for (int b = 0; b < SB; ++b) {
            const int jb = se * SB + b;
            if (jb * 32 + 32 > rows) {   // rows past the split contribute nothing
#pragma unroll
                for (int r = 0; r < 8; ++r)
                    if (jb * 32 + 8 * g + r >= rows) w[b][r] = u32x4{0, 0, 0, 0};
            }
#pragma unroll
            for (int c = 0; c < 8; ++c) {
                const uint32_t sel = (c & 1) ? 0x07060302u : 0x05040100u;
                u32x4 bb;
#pragma unroll
                for (int p = 0; p < 4; ++p) bb[p] = __builtin_amdgcn_perm(w[b][2 * p + 1][c >> 1], w[b][2 * p][c >> 1], sel);
#pragma unroll
                for (int tt = 0; tt < TT; ++tt) acc2[c][tt] = mfma16<E>(av[b][tt], bb, acc2[c][tt]);
            }
        }
        if (++abuf == geo.pl) abuf = 0;
        if (++wbuf == geo.nb) wbuf = 0;
        if (++wfree == geo.nb) wfree = 0;
    }
#undef DFK_ST
    DFK_STAMP(4);

    // D tile (column tile c, token tile tt): lane (q, g) holds tokens 4g .. 4g+3 of the tile, column
    // 8q + c of the block: the lane's 8 column tiles are 8 consecutive columns.
    const bool atomic_mode = a.reduce_mode == DFK_REDUCE_ATOMIC;
    const int nb0 = cb * 128;
#pragma unroll
    for (int tt = 0; tt < TT; ++tt) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int m = (tile0 + tt) * 16 + 4 * g + i;
            if (m < a.m_count) {
                if (atomic_mode) {
                    float* dst = a.yacc + (size_t)m * a.d_model + nb0 + 8 * q;
#pragma unroll
                    for (int c = 0; c < 8; ++c) acc_add(dst + c, acc2[c][tt][i]);
                } else {       // partial block of the split: plain stores, summed by the launch that follows
                    float* dst = a.P + ((size_t)js * a.m_count + m) * a.d_model + nb0 + 8 * q;
                    *(f32x4*)dst = f32x4{acc2[0][tt][i], acc2[1][tt][i], acc2[2][tt][i], acc2[3][tt][i]};
                    *(f32x4*)(dst + 4) = f32x4{acc2[4][tt][i], acc2[5][tt][i], acc2[6][tt][i], acc2[7][tt][i]};
                }
            }
        }
    }
    if (atomic_mode) {
        drain_own_memory_ops();
        __syncthreads();
        if (tid == 0) flag = arrive_last(a.tickets + cb, (unsigned)a.k2_splits) ? 1 : 0;
        __syncthreads();
        if (!flag) return;
        for (int idx = tid; idx < a.m_count * 64; idx += NTHREADS) {
            const int m = idx >> 6, c2 = idx & 63;
            float* src = a.yacc + (size_t)m * a.d_model + nb0 + 2 * c2;
            float v0 = acc_take(src), v1 = acc_take(src + 1);
            const size_t o = (size_t)(a.m_base + m) * a.d_model + nb0 + 2 * c2;
            if (a.resid) {
                float r0, r1;
                E::widen2(*(const uint32_t*)((const uint16_t*)a.resid + o), r0, r1);
                v0 += r0; v1 += r1;
            }
            *(uint32_t*)((uint16_t*)a.Y + o) = E::pack2(v0, v1);
        }
    }
}

// Sum of the splits' partial blocks (counter reduction mode of the down kernel above): with
// hundreds of tokens the blocks are tens of MB, too much for the last workgroup of a column
// block to add up alone, so a launch of its own spreads the sum over the whole chip.  Fixed
// order (split 0, 1, ...): bitwise reproducible.  One thread per four consecutive outputs.
template <typename E>
__global__ __launch_bounds__(256) void k_sum_partials_big(MlpArgs a) {
    const int w4 = a.d_model >> 2;
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (size_t)a.m_count * w4) return;
    const int m = (int)(idx / w4), c4 = (int)(idx - (size_t)m * w4);
    const size_t blk = (size_t)a.m_count * a.d_model;
    const float* src = a.P + (size_t)m * a.d_model + 4 * c4;
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int js0 = 0; js0 < a.k2_splits; js0 += 8) {
        float4 t[8];
#pragma unroll
        for (int k = 0; k < 8; ++k)
            t[k] = js0 + k < a.k2_splits ? *(const float4*)(src + (size_t)(js0 + k) * blk) : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int k = 0; k < 8; ++k) { v.x += t[k].x; v.y += t[k].y; v.z += t[k].z; v.w += t[k].w; }
    }
    store4_plus<E>(a.Y, a.resid, (size_t)(a.m_base + m) * a.d_model + 4 * c4, v);
}

// Every instantiation the launcher uses, spelled out (the host pass otherwise emitted the launch
// stub of only one element type per token-tile count).
#define DFK_INST_GATEUP(NTC)                                                     \
    template __global__ void k_gateup_big<1, BF16, NTC, 8>(MlpArgs, BigGeom);    \
    template __global__ void k_gateup_big<1, FP16, NTC, 8>(MlpArgs, BigGeom);    \
    template __global__ void k_gateup_big<2, BF16, NTC, 8>(MlpArgs, BigGeom);    \
    template __global__ void k_gateup_big<2, FP16, NTC, 8>(MlpArgs, BigGeom);    \
    template __global__ void k_gateup_big<2, BF16, NTC, 4>(MlpArgs, BigGeom);    \
    template __global__ void k_gateup_big<2, FP16, NTC, 4>(MlpArgs, BigGeom);    \
    template __global__ void k_gateup_big<4, BF16, NTC, 4>(MlpArgs, BigGeom);    \
    template __global__ void k_gateup_big<4, FP16, NTC, 4>(MlpArgs, BigGeom);    \
    template __global__ void k_gateup_big<1, BF16, NTC, 4>(MlpArgs, BigGeom);    \
    template __global__ void k_gateup_big<1, FP16, NTC, 4>(MlpArgs, BigGeom);
DFK_INST_GATEUP(1) DFK_INST_GATEUP(2) DFK_INST_GATEUP(3) DFK_INST_GATEUP(4)
DFK_INST_GATEUP(5) DFK_INST_GATEUP(6) DFK_INST_GATEUP(7) DFK_INST_GATEUP(8)
#undef DFK_INST_GATEUP
template __global__ void k_sum_partials_big<BF16>(MlpArgs);
template __global__ void k_sum_partials_big<FP16>(MlpArgs);
template __global__ void k_down_big<1, BF16, kBigDownWaves>(MlpArgs, BigGeom);
template __global__ void k_down_big<1, FP16, kBigDownWaves>(MlpArgs, BigGeom);
template __global__ void k_down_big<2, BF16, kBigDownWaves>(MlpArgs, BigGeom);
template __global__ void k_down_big<2, FP16, kBigDownWaves>(MlpArgs, BigGeom);

// ---------------------------------------------------------------- host side
int big_token_tiles(int m_count) { return m_count <= 128 ? 2 : 4; }   // per wavefront

// LDS of the gate/up kernel: nb shared buffers of the slice's weight tiles, then pl X buffers per wavefront.
size_t big_lds_gateup(const dfk_config_t& c, int TT, int d_ff, BigGeom* geo) {
    const int nt_max = max_slice_rows(d_ff, c.splits) / 8;
    geo->nb = c.depth;
    geo->shared_step = nt_max * kTileBytes;
    geo->priv_off = geo->nb * geo->shared_step;
    geo->priv_step = TT * kTileBytes * kBigWaves / c.waves;   // TT counts token tiles per wavefront of the 4-wavefront form
    const size_t one = (size_t)c.waves * geo->priv_step;
    geo->pl = (size_t)geo->priv_off + 2 * one <= (size_t)kLdsLimit ? 2 : 1;
    return (size_t)geo->priv_off + geo->pl * one;
}
size_t big_lds_down(const dfk_config_t& c, BigGeom* geo) {
    geo->nb = c.depth;
    geo->shared_step = kBigSB * 2 * kTileBytes;
    geo->priv_off = geo->nb * geo->shared_step;
    geo->priv_step = 2 * 2048;                 // 2 KB per token tile of the wavefront (up to 2)
    const size_t one = (size_t)kBigDownWaves * geo->priv_step;
    geo->pl = (size_t)geo->priv_off + 2 * one <= (size_t)kLdsLimit ? 2 : 1;
    return (size_t)geo->priv_off + geo->pl * one;
}

template <int TT, typename E, int NTC>
hipError_t launch_big_gateup(const MlpArgs& a, const dfk_config_t& c, hipStream_t st) {
    static LdsAllowance allowed4, allowed8;   // of the two kernels of this instantiation, per device
    BigGeom geo{};
    const size_t lds = big_lds_gateup(c, TT, a.d_ff, &geo);
    if (c.waves == 8) {
        if (hipError_t e = allow_lds(allowed8, (const void*)k_gateup_big<TT / 2, E, NTC, 8>, lds); e != hipSuccess) return e;
        hipLaunchKernelGGL((k_gateup_big<TT / 2, E, NTC, 8>), dim3(a.splits), dim3(512), lds, st, a, geo);
    } else {
        if (hipError_t e = allow_lds(allowed4, (const void*)k_gateup_big<TT, E, NTC, 4>, lds); e != hipSuccess) return e;
        hipLaunchKernelGGL((k_gateup_big<TT, E, NTC, 4>), dim3(a.splits), dim3(256), lds, st, a, geo);
    }
    return hipGetLastError();
}

template <int TT, typename E>
hipError_t launch_big_te(const MlpArgs& a, const dfk_config_t& c, hipStream_t st) {
    static LdsAllowance allowed2;   // of the down kernel of this instantiation, per device
    if (g_stage_mask & 1) {
        hipError_t e;
        switch (max_slice_rows(a.d_ff, c.splits) / 8) {
            case 1: e = launch_big_gateup<TT, E, 1>(a, c, st); break;
            case 2: e = launch_big_gateup<TT, E, 2>(a, c, st); break;
            case 3: e = launch_big_gateup<TT, E, 3>(a, c, st); break;
            case 4: e = launch_big_gateup<TT, E, 4>(a, c, st); break;
            case 5: e = launch_big_gateup<TT, E, 5>(a, c, st); break;
            case 6: e = launch_big_gateup<TT, E, 6>(a, c, st); break;
            case 7: e = launch_big_gateup<TT, E, 7>(a, c, st); break;
            case 8: e = launch_big_gateup<TT, E, 8>(a, c, st); break;
            default: e = hipErrorInvalidValue; break;
        }
        if (e != hipSuccess) return e;
    }
    if (g_stage_mask & 2) {
        BigGeom geo{};
        const size_t lds = big_lds_down(c, &geo);
        geo.by_xcd = (size_t)a.m_count * a.d_ff * 2 > kL2BytesPerXcd;
        if (hipError_t e = allow_lds(allowed2, (const void*)k_down_big<TT / 2, E, kBigDownWaves>, lds); e != hipSuccess) return e;
        // (TT token tiles per wavefront of the 4-wavefront gate/up kernel are TT / 2 in the 8 of this one)
        hipLaunchKernelGGL((k_down_big<TT / 2, E, kBigDownWaves>), dim3(a.k2_splits * a.k2_col_blocks), dim3(kBigDownWaves * 64), lds, st, a, geo);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess || a.reduce_mode == DFK_REDUCE_ATOMIC) return e;
        const size_t n4 = (size_t)a.m_count * (a.d_model / 4);
        hipLaunchKernelGGL((k_sum_partials_big<E>), dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, st, a);
        return hipGetLastError();
    }
    return hipSuccess;
}

template <int TT>
hipError_t launch_big_t(const MlpArgs& a, const dfk_config_t& c, hipStream_t st) {
    return a.dtype == DFK_FP16 ? launch_big_te<TT, FP16>(a, c, st) : launch_big_te<TT, BF16>(a, c, st);
}

}  // namespace

int mfma_big_tokens_per_launch() { return kBigTokensPerLaunch; }

// The gate/up kernel alone with four wavefronts of one token tile each: up to 64 tokens per launch.  Paired with
// the down kernel of the 64-token pair for 33..64 tokens (config field kmajor = 3): with three or four token
// tiles the shared weight tiles (read from L2 once per workgroup instead of once per wavefront) pay, while the
// down kernel of this family does not yet.
namespace {
template <typename E, int NTC>
hipError_t launch_gateup_64_n(const MlpArgs& a, const dfk_config_t& c, hipStream_t st) {
    static LdsAllowance allowed;
    BigGeom geo{};
    const size_t lds = big_lds_gateup(c, 1, a.d_ff, &geo);
    if (hipError_t e = allow_lds(allowed, (const void*)k_gateup_big<1, E, NTC, 4>, lds); e != hipSuccess) return e;
    hipLaunchKernelGGL((k_gateup_big<1, E, NTC, 4>), dim3(a.splits), dim3(256), lds, st, a, geo);
    return hipGetLastError();
}
template <typename E>
hipError_t launch_gateup_64_e(const MlpArgs& a, const dfk_config_t& c, hipStream_t st) {
    switch (max_slice_rows(a.d_ff, c.splits) / 8) {
        case 1: return launch_gateup_64_n<E, 1>(a, c, st);
        case 2: return launch_gateup_64_n<E, 2>(a, c, st);
        case 3: return launch_gateup_64_n<E, 3>(a, c, st);
        case 4: return launch_gateup_64_n<E, 4>(a, c, st);
        case 5: return launch_gateup_64_n<E, 5>(a, c, st);
        case 6: return launch_gateup_64_n<E, 6>(a, c, st);
        case 7: return launch_gateup_64_n<E, 7>(a, c, st);
        case 8: return launch_gateup_64_n<E, 8>(a, c, st);
        default: return hipErrorInvalidValue;
    }
}
}  // namespace

// c.waves must be 4 here (the caller passes a copy of its configuration with the gate/up kernel's wavefront count)
hipError_t launch_big_gateup_64(const MlpArgs& a, const dfk_config_t& c, hipStream_t st) {
    if (a.norm_w || a.m_count > 64) return hipErrorInvalidValue;
    return a.dtype == DFK_FP16 ? launch_gateup_64_e<FP16>(a, c, st) : launch_gateup_64_e<BF16>(a, c, st);
}
bool big_gateup_64_fits(const dfk_config_t& c, int d_model, int d_ff) {
    if (d_model < 128 || d_model % kKC || d_model > kMaxDModel) return false;
    if (c.depth < 3 || c.depth > 4) return false;
    if (max_slice_rows(d_ff, c.splits) / 8 > kBigMaxRowTiles) return false;
    BigGeom geo{};
    return big_lds_gateup(c, 1, d_ff, &geo) <= (size_t)kLdsLimit;
}

bool mfma_big_config_valid(const dfk_config_t& c, int M, int d_model, int d_ff, dfk_dtype_t dtype) {
    if (c.path != DFK_PATH_MFMA || (dtype != DFK_BF16 && dtype != DFK_FP16) || c.variant != DFK_VARIANT_TWO_KERNEL) return false;
    if (c.kmajor != 2 || c.k2_rows_by_wave != 0 || c.a2_dtype != (int)dtype) return false;
    if (c.reduce != DFK_REDUCE_TICKET && c.reduce != DFK_REDUCE_ATOMIC) return false;
    if ((c.waves != 4 && c.waves != 8) || c.depth < 3 || c.depth > 4) return false;   // depth = buffers of shared tiles
    if (M < 1 || d_model < 128 || d_ff < 8 || d_ff % 8 || d_model % kKC || d_model > kMaxDModel) return false;
    const int ng = d_ff / 8;
    if (c.splits < 1 || c.splits > ng || c.splits > 65535) return false;
    if (max_slice_rows(d_ff, c.splits) / 8 > kBigMaxRowTiles) return false;
    if (c.k2_splits < 1 || c.k2_splits > ng) return false;
    if (c.k2_col_blocks != d_model / 128) return false;                        // one 128-column block per workgroup
    if ((long long)c.k2_splits * c.k2_col_blocks > 65535 || c.k2_col_blocks > kTicketLevel2) return false;
    const int tokens = std::min(M, kBigTokensPerLaunch);
    if (c.reduce == DFK_REDUCE_ATOMIC && (size_t)tokens * d_model * 4 > kYaccBytes) return false;   // fp32 accumulator of one launch
    // (this pair's counter mode keeps one partial block per split and no group sums)
    if (c.reduce == DFK_REDUCE_TICKET && (size_t)c.k2_splits * tokens * d_model * 4 > partial_bytes(M, d_model)) return false;
    BigGeom geo{};
    return big_lds_gateup(c, big_token_tiles(tokens), d_ff, &geo) <= (size_t)kLdsLimit && big_lds_down(c, &geo) <= (size_t)kLdsLimit;
}

hipError_t launch_mfma_big(const MlpArgs& a, const dfk_config_t& c, hipStream_t st) {
    if (a.norm_w) return hipErrorInvalidValue;   // the normalisation is folded into the 64-token pair only
    return big_token_tiles(a.m_count) == 2 ? launch_big_t<2>(a, c, st) : launch_big_t<4>(a, c, st);
}

}  // namespace dfk
