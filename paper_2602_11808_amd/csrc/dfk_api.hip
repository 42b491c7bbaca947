// C ABI of libdfk: argument validation, the profile-driven scheduler and its
// table, dispatch to the VALU / MFMA launchers.  Host code only.
#include <algorithm>
#include <cstdio>
#include <cstring>
#include <map>
#include <mutex>
#include <tuple>
#include <vector>

#include "dfk_internal.h"

namespace dfk {
thread_local int g_stage_mask = 3;

namespace {

thread_local int g_last_hip_error = 0;
thread_local int g_tune_skipped = 0;                  // candidates the last dfk_tune on this thread left out
thread_local dfk_status_t g_tune_skip_status = DFK_OK;  // status of the last one

dfk_status_t hip_fail(hipError_t e) {
    g_last_hip_error = (int)e;
    return DFK_ERR_HIP;
}

struct Registered {
    void* ptr = nullptr;
    size_t bytes = 0;
};
Registered g_ws;
Registered g_trace;
std::mutex g_mu;

// A consistent copy of a registered buffer: the setters write under the same lock.
Registered snapshot(const Registered& r) {
    std::lock_guard<std::mutex> lk(g_mu);
    return r;
}

// ---------------------------------------------------------------- validation
size_t elt_bytes(dfk_dtype_t d) { return d == DFK_FP32 ? 4 : 2; }

bool overlaps(const void* a, size_t na, const void* b, size_t nb) {
    const uintptr_t a0 = (uintptr_t)a, b0 = (uintptr_t)b;
    return a0 < b0 + nb && b0 < a0 + na;
}

// The shapes a call accepts: every query below and the argument check agree on it.
bool shape_supported(int M, int d_model, int d_ff) {
    return M >= 1 && M <= DFK_MAX_M && d_model >= 8 && d_model <= kMaxDModel && d_ff >= 8 && d_model % 8 == 0 && d_ff % 8 == 0;
}

bool config_valid(const dfk_config_t& c, int M, int d_model, int d_ff, dfk_dtype_t dtype) {
    if (!shape_supported(M, d_model, d_ff)) return false;
    if (c.path == DFK_PATH_VALU) return valu_config_valid(c, M, d_model, d_ff, dtype);
    if (c.path == DFK_PATH_MFMA) return mfma_config_valid(c, M, d_model, d_ff, dtype);
    return false;
}

// configurations whose down kernel takes W_down as [d_model, d_ff]
bool wdt_layout(const dfk_config_t& c) { return c.kmajor == 5; }

dfk_status_t check(const void* X, const void* Wg, const void* Wu, const void* Wd, const void* Y,
                   int M, int d_model, int d_ff, dfk_dtype_t dtype, const dfk_config_t* cfg,
                   const void* ws, size_t ws_bytes, bool need_ws, bool y_may_be_x = false, bool wd_t = false) {
    if (!X || !Wg || !Wu || !Wd || !Y) return DFK_ERR_INVALID_ARG;
    if (M < 1 || d_model < 1 || d_ff < 1) return DFK_ERR_INVALID_ARG;
    if (dtype != DFK_BF16 && dtype != DFK_FP32 && dtype != DFK_FP16) return DFK_ERR_INVALID_ARG;
    if (!shape_supported(M, d_model, d_ff)) return DFK_ERR_UNSUPPORTED_SHAPE;
    const void* ptrs[5] = {X, Wg, Wu, Wd, Y};
    for (const void* p : ptrs)
        if ((uintptr_t)p % 16) return DFK_ERR_ALIGNMENT;
    const size_t eb = elt_bytes(dtype);
    const size_t nx = (size_t)M * d_model * eb, nw = (size_t)d_ff * d_model * eb;
    if ((!(y_may_be_x && Y == X) && overlaps(Y, nx, X, nx)) || overlaps(Y, nx, Wg, nw) || overlaps(Y, nx, Wu, nw) ||
        overlaps(Y, nx, Wd, nw))
        return DFK_ERR_ALIAS;
    if (cfg) {
        if (cfg->variant != DFK_VARIANT_FUSED && cfg->variant != DFK_VARIANT_TWO_KERNEL)
            return DFK_ERR_INVALID_ARG;
        if (cfg->path != DFK_PATH_VALU && cfg->path != DFK_PATH_MFMA) return DFK_ERR_INVALID_ARG;
        if (wdt_layout(*cfg) != wd_t) return DFK_ERR_INVALID_ARG;   // the configuration is for the other layout of W_down
        if (!config_valid(*cfg, M, d_model, d_ff, dtype)) return DFK_ERR_UNSUPPORTED_SHAPE;
    }
    if (need_ws || ws || ws_bytes) {
        if (!ws) return DFK_ERR_WORKSPACE;
        if ((uintptr_t)ws % 256) return DFK_ERR_ALIGNMENT;
        if (ws_bytes < ws_layout(M, d_model, d_ff).total) return DFK_ERR_WORKSPACE;
        if (overlaps(ws, ws_bytes, Y, nx) || overlaps(ws, ws_bytes, X, nx) ||
            overlaps(ws, ws_bytes, Wg, nw) || overlaps(ws, ws_bytes, Wu, nw) ||
            overlaps(ws, ws_bytes, Wd, nw))
            return DFK_ERR_ALIAS;
    }
    return DFK_OK;
}

// ---------------------------------------------------------------- candidates and heuristic
// the single launch that holds both kernels' workgroups: variant FUSED, but partial sums and stages of the pair
bool roles_launch(const dfk_config_t& c) { return c.variant == DFK_VARIANT_FUSED && c.path == DFK_PATH_MFMA && c.kmajor == 4; }

int clamp_splits(int want, int d_ff) { return std::max(1, std::min(want, d_ff / 8)); }

dfk_config_t make_cfg(int variant, int path, int splits, int waves, int depth, int k2s, int k2c,
                      int a2dt, int reduce = DFK_REDUCE_TICKET, int rows_by_wave = 0, int kmajor = 0) {
    dfk_config_t c;
    std::memset(&c, 0, sizeof c);
    c.variant = variant; c.path = path; c.splits = splits; c.waves = waves; c.depth = depth;
    c.reduce = reduce; c.k2_splits = k2s; c.k2_col_blocks = k2c; c.a2_dtype = a2dt;
    c.k2_rows_by_wave = rows_by_wave;
    c.kmajor = kmajor;
    return c;
}

bool same_cfg(const dfk_config_t& a, const dfk_config_t& b) {
    return a.variant == b.variant && a.path == b.path && a.splits == b.splits && a.waves == b.waves &&
           a.depth == b.depth && a.reduce == b.reduce && a.k2_splits == b.k2_splits &&
           a.k2_col_blocks == b.k2_col_blocks && a.a2_dtype == b.a2_dtype &&
           a.k2_rows_by_wave == b.k2_rows_by_wave && a.kmajor == b.kmajor;
}

// The candidate set of the scheduler (Method: tiling variants x tile sizes).
std::vector<dfk_config_t> candidates(int M, int d_model, int d_ff, dfk_dtype_t dtype) {
    std::vector<dfk_config_t> out;
    auto push = [&](const dfk_config_t& c) {
        if (!config_valid(c, M, d_model, d_ff, dtype)) return;
        for (const auto& o : out)
            if (same_cfg(o, c)) return;
        out.push_back(c);
    };
    const int a2dt = dtype == DFK_BF16 ? DFK_BF16 : DFK_FP32;   // VALU pair: fp32 unless the inputs are bf16
    if (dtype == DFK_BF16 || dtype == DFK_FP16) {   // (the first-generation MFMA kernels validate for bf16 only)
        // MFMA path: d_ff slices ("column-major tiling": each workgroup owns a
        // block of weight rows and reuses it for every token).
        for (int splits : {256, 512})
            for (int waves : {4, 8})
                for (int depth : {2, 4, 6, 8})
                    for (int reduce : {DFK_REDUCE_ATOMIC, DFK_REDUCE_TICKET})
                        push(make_cfg(DFK_VARIANT_FUSED, DFK_PATH_MFMA, clamp_splits(splits, d_ff), waves,
                                      depth, 0, 0, a2dt, reduce));
        const int nblk = d_model / 128;
        // the single launch on the k-major stage one of the 64-token pair (a slice of at most 64 rows per workgroup)
        for (int splits : {256, 512, d_ff > 512 * 64 ? ((d_ff + 63) / 64 + 255) / 256 * 256 : 512})
            for (int reduce : {DFK_REDUCE_ATOMIC, DFK_REDUCE_TICKET})
                for (int wd : {83, 84, 46, 48})   // wavefronts, ring depth
                    push(make_cfg(DFK_VARIANT_FUSED, DFK_PATH_MFMA, clamp_splits(splits, d_ff), wd / 10, wd % 10, 0, 0, (int)dtype,
                                  reduce, 0, 1));
        // two-kernel: the down projection is tiled (d_ff splits) x (column blocks of
        // waves*128 or 2*waves*128 columns), about one or two workgroups per CU
        for (int splits : {256, 512})
            for (int waves : {4, 8})
                for (int per_wave : {1, 2}) {
                    const int wg_blocks = waves * per_wave;
                    if (wg_blocks > nblk || nblk % wg_blocks) continue;
                    const int k2c = nblk / wg_blocks;
                    for (int grid : {256, 512})
                        for (int reduce : {DFK_REDUCE_ATOMIC, DFK_REDUCE_TICKET})
                            push(make_cfg(DFK_VARIANT_TWO_KERNEL, DFK_PATH_MFMA, clamp_splits(splits, d_ff),
                                          waves, 4, clamp_splits(std::max(1, grid / k2c), d_ff), k2c, a2dt,
                                          reduce));
                }
        // two-kernel, down projection with the rows divided among the wavefronts: few d_ff splits
        for (int waves : {8, 4})
            for (int cbw : {1, 2, 4}) {           // 128-column blocks per workgroup
                if (nblk < cbw || nblk % cbw) continue;
                const int k2c = nblk / cbw;
                for (int grid : {256, 512})
                    for (int reduce : {DFK_REDUCE_TICKET, DFK_REDUCE_ATOMIC})
                        for (int depth : {3, 4})
                            push(make_cfg(DFK_VARIANT_TWO_KERNEL, DFK_PATH_MFMA, clamp_splits(256, d_ff), waves, depth,
                                          clamp_splits(std::max(1, grid / k2c), d_ff), k2c, DFK_BF16, reduce, 1));
            }
        // two-kernel, activations through the tile rings: up to 64 tokens per launch.  A slice of the
        // gate/up kernels of this pair and of the next holds at most 64 rows, so a d_ff beyond
        // 512 * 64 needs more slices: the next multiple of 256 that is enough.
        const int more_splits = d_ff > 512 * 64 ? ((d_ff + 63) / 64 + 255) / 256 * 256 : 512;
        for (int splits : {256, 512, more_splits})
            for (int cbw : {1, 2}) {
                if (nblk < cbw || nblk % cbw) continue;
                const int k2c = nblk / cbw;
                for (int grid : {256, 512})
                    for (int reduce : {DFK_REDUCE_TICKET, DFK_REDUCE_ATOMIC})
                        for (int wd : {83, 84, 46, 48})   // wavefronts, ring depth
                            push(make_cfg(DFK_VARIANT_TWO_KERNEL, DFK_PATH_MFMA, clamp_splits(splits, d_ff), wd / 10, wd % 10,
                                          clamp_splits(std::max(1, grid / k2c), d_ff), k2c, (int)dtype, reduce, 0, 1));
            }
        // both kernels of that pair in one launch (gate/up workgroups at the head of the grid, down workgroups
        // behind them)
        for (int splits : {256, 512})
            for (int cbw : {1, 2}) {
                if (nblk < cbw || nblk % cbw) continue;
                const int k2c = nblk / cbw;
                for (int grid : {256, 512})
                    for (int reduce : {DFK_REDUCE_TICKET, DFK_REDUCE_ATOMIC})
                        for (int depth : {3, 4})
                            push(make_cfg(DFK_VARIANT_FUSED, DFK_PATH_MFMA, clamp_splits(splits, d_ff), 8, depth,
                                          clamp_splits(std::max(1, grid / k2c), d_ff), k2c, (int)dtype, reduce, 0, 4));
            }
        // two-kernel for 33..64 tokens: gate/up kernel with workgroup-shared weight tiles and one token tile per
        // wavefront, down kernel of the pair above
        if (M > 32 && nblk >= 1)
            for (int splits : {256, 512})
                for (int grid : {256, 512})
                    for (int reduce : {DFK_REDUCE_TICKET, DFK_REDUCE_ATOMIC})
                        for (int depth : {3, 4})
                            push(make_cfg(DFK_VARIANT_TWO_KERNEL, DFK_PATH_MFMA, clamp_splits(splits, d_ff), 8, depth,
                                          clamp_splits(std::max(1, grid / nblk), d_ff), nblk, (int)dtype, reduce, 0, 3));
        // two-kernel, workgroup-shared weight tiles: up to 256 tokens per launch.  Offered beyond 64 tokens,
        // and below where d_model rules out the pair above (it needs whole 128-k chunks per wavefront,
        // this one only d_model % 128 == 0)
        bool have_km = false;
        for (const auto& o : out) have_km = have_km || o.kmajor == 1;
        if ((M > 64 || !have_km) && nblk >= 1) {
            const int k2c = nblk;
            for (int splits : {256, 512, more_splits})
                for (int grid : {256, 512})
                    for (int reduce : {DFK_REDUCE_TICKET, DFK_REDUCE_ATOMIC})
                        for (int depth : {3, 4})
                            for (int waves : {8, 4})   // of the gate/up kernel
                                push(make_cfg(DFK_VARIANT_TWO_KERNEL, DFK_PATH_MFMA, clamp_splits(splits, d_ff), waves, depth,
                                              clamp_splits(std::max(1, grid / k2c), d_ff), k2c, (int)dtype, reduce, 0, 2));
        }
    }
    for (int splits : {256, 512, 1024})
        for (int waves : {4, 8})
            push(make_cfg(DFK_VARIANT_FUSED, DFK_PATH_VALU, clamp_splits(splits, d_ff), waves, 0, 0, 0,
                          a2dt));
    const int nchunk = d_model / (dtype == DFK_FP32 ? 4 : 8);
    for (int splits : {512, 1024})
        for (int k2s : {8, 16, 32}) {
            const int k2 = clamp_splits(k2s, d_ff);
            const int cb = std::max(1, std::min(nchunk / 64 > 0 ? nchunk / 64 : 1, std::max(1, 512 / k2)));
            push(make_cfg(DFK_VARIANT_TWO_KERNEL, DFK_PATH_VALU, clamp_splits(splits, d_ff), 8, 0, k2,
                          cb, a2dt));
        }
    return out;
}

// W_down given as [d_model, d_ff]: the 64-token pair's gate/up kernel, then the down kernel whose workgroups own
// slices of d_model (no sum across workgroups).  First in the list = the untuned default.
std::vector<dfk_config_t> candidates_wdt(int M, int d_model, int d_ff, dfk_dtype_t dtype) {
    std::vector<dfk_config_t> out;
    // plain fp32-FMA kernels for every shape and type (after the MFMA pair in the list, where there is one)
    auto valu = [&]() {
        const int a2dt = dtype == DFK_BF16 ? DFK_BF16 : DFK_FP32;
        for (int splits : {512, 1024})
            for (int k2s : {256, 512}) {
                dfk_config_t c = make_cfg(DFK_VARIANT_TWO_KERNEL, DFK_PATH_VALU, clamp_splits(splits, d_ff), 8, 0,
                                          std::max(1, std::min(k2s, (d_model + 7) / 8)), 1, a2dt, DFK_REDUCE_TICKET, 0, 5);
                if (!config_valid(c, M, d_model, d_ff, dtype)) continue;
                bool dup = false;
                for (const auto& o : out) dup = dup || same_cfg(o, c);
                if (!dup) out.push_back(c);
            }
    };
    if (dtype != DFK_BF16 && dtype != DFK_FP16) {
        valu();
        return out;
    }
    const int more_splits = d_ff > 512 * 64 ? ((d_ff + 63) / 64 + 255) / 256 * 256 : 512;
    const int t16 = d_model / 16;
    for (int wd : {82, 83, 84, 46})          // wavefronts, ring depth
        for (int splits : {256, 512, more_splits})
            for (int k2s : {256, 512, 128}) {
                dfk_config_t c = make_cfg(DFK_VARIANT_TWO_KERNEL, DFK_PATH_MFMA, clamp_splits(splits, d_ff), wd / 10, wd % 10,
                                          std::max(1, std::min(k2s, t16)), 1, (int)dtype, DFK_REDUCE_TICKET, 0, 5);
                if (!config_valid(c, M, d_model, d_ff, dtype)) continue;
                bool dup = false;
                for (const auto& o : out) dup = dup || same_cfg(o, c);
                if (!dup) out.push_back(c);
            }
    valu();
    return out;
}

// Untuned default, from measurements on MI355X.  One token: the single launch that keeps A_2 in LDS, with the
// atomic reduction (no boundary between two kernels, and its 256 full-width partial sums are still cheap).  Up to
// 64 tokens: the single launch that holds both kernels' workgroups (atomic reduction), which saves the launch
// boundary at every token count.  Of the two-kernel forms: beyond 64 tokens the pair that takes up to 256 per
// launch, else the pair for up to 64 tokens, then the rows-split down kernel, then the rest.
bool heuristic(int M, int d_model, int d_ff, dfk_dtype_t dtype, int want_variant, dfk_config_t* out) {
    auto cands = candidates(M, d_model, d_ff, dtype);
    auto rank = [&](const dfk_config_t& c) {
        if (c.variant == DFK_VARIANT_TWO_KERNEL) {
            if (c.kmajor == 2) return M > 64 ? -1 : 1;     // one launch for up to 256 tokens beats several of 64
            if (c.kmajor == 3) return 1;
            return c.kmajor ? 0 : c.k2_rows_by_wave ? 1 : 2;
        }
        if (roles_launch(c)) return M <= 64 && c.reduce == DFK_REDUCE_ATOMIC && c.depth == 4 ? -2 : 3;
        if (c.path == DFK_PATH_MFMA && c.kmajor == 1)      // the single launch with A_2 in LDS
            return c.reduce == DFK_REDUCE_ATOMIC && c.waves == 8 ? (M == 1 ? -3 : 3) : 4;
        return 5;
    };
    const dfk_config_t* best = nullptr;
    for (const auto& c : cands) {
        if (want_variant != DFK_VARIANT_AUTO && c.variant != want_variant) continue;
        if (!best || rank(c) < rank(*best)) best = &c;
    }
    if (!best) return false;
    *out = *best;
    return true;
}

// ---------------------------------------------------------------- tuning table
struct Entry {
    dfk_config_t cfg;
    double usec;
};
// M, d_model, d_ff, dtype, slot.  Slot 0 holds the choice for the problem; slots DFK_VARIANT_FUSED and
// DFK_VARIANT_TWO_KERNEL the best known configuration of that variant (what a call that asks for a variant gets).
using Key = std::tuple<int, int, int, int, int>;
std::map<Key, Entry> g_table;
constexpr int kSlotWdt = 3;   // slot of the best configuration for W_down given as [d_model, d_ff]
void table_put(int M, int d_model, int d_ff, int dtype, const Entry& e, bool chosen) {   // g_mu held
    if (wdt_layout(e.cfg)) {   // the other layout of W_down has a slot of its own and never is the plain choice
        g_table[Key(M, d_model, d_ff, dtype, kSlotWdt)] = e;
        return;
    }
    g_table[Key(M, d_model, d_ff, dtype, e.cfg.variant)] = e;
    if (chosen) g_table[Key(M, d_model, d_ff, dtype, 0)] = e;
}

int m_bucket(int M) {
    int b = 1;
    while (b < M) b <<= 1;
    return b;
}

bool lookup(int M, int d_model, int d_ff, dfk_dtype_t dtype, int want_variant, dfk_config_t* out) {
    std::lock_guard<std::mutex> lk(g_mu);
    for (int m : {M, m_bucket(M)}) {
        auto it = g_table.find(Key(m, d_model, d_ff, (int)dtype, want_variant == DFK_VARIANT_AUTO ? 0 : want_variant));
        if (it == g_table.end()) continue;
        const dfk_config_t& c = it->second.cfg;
        if (!config_valid(c, M, d_model, d_ff, dtype)) continue;
        *out = c;
        return true;
    }
    return false;
}

bool choose_wdt(int M, int d_model, int d_ff, dfk_dtype_t dtype, dfk_config_t* out, int* tuned) {
    if (lookup(M, d_model, d_ff, dtype, kSlotWdt, out)) {
        if (tuned) *tuned = 1;
        return true;
    }
    if (tuned) *tuned = 0;
    auto cands = candidates_wdt(M, d_model, d_ff, dtype);
    if (cands.empty()) return false;
    *out = cands[0];
    return true;
}

bool choose(int M, int d_model, int d_ff, dfk_dtype_t dtype, int want_variant, dfk_config_t* out,
            int* tuned) {
    if (lookup(M, d_model, d_ff, dtype, want_variant, out)) {
        if (tuned) *tuned = 1;
        return true;
    }
    if (tuned) *tuned = 0;
    return heuristic(M, d_model, d_ff, dtype, want_variant, out);
}

// ---------------------------------------------------------------- dispatch
// norm_w / eps / resid: the pre-norm residual form (kernel pair for up to 64 tokens only,
// checked by the caller); NULL / 0 / NULL for the plain block.
dfk_status_t run_in(const WsLayout& l, const void* X, const void* Wg, const void* Wu, const void* Wd, void* Y, int M,
                    int d_model, int d_ff, dfk_dtype_t dtype, const dfk_config_t& c, void* ws,
                    hipStream_t st, const void* norm_w = nullptr, float eps = 0.f, const void* resid = nullptr) {
    MlpArgs a;
    std::memset(&a, 0, sizeof a);
    a.X = X; a.Wg = Wg; a.Wu = Wu; a.Wd = Wd; a.Y = Y;
    a.M = M; a.d_model = d_model; a.d_ff = d_ff;
    a.splits = c.splits; a.k2_splits = c.k2_splits; a.k2_col_blocks = c.k2_col_blocks;
    a.dtype = (int)dtype;
    a.a2_is_fp32 = c.a2_dtype == DFK_FP32;
    a.tickets = (unsigned*)((char*)ws + l.tickets_off);
    a.reduce_mode = c.reduce;
    a.yacc = (float*)((char*)ws + l.yacc_off);
    a.P = (float*)((char*)ws + l.p_off);
    a.Q = (float*)((char*)ws + l.q_off);
    a.a2 = (char*)ws + l.a2_off;
    a.norm_w = norm_w; a.eps = eps; a.resid = resid;
    if (norm_w && (c.kmajor == 2 || !mfma_km_block_config_valid(c, M, d_model, d_ff, dtype))) {   // (kmajor 1 and 5 fold it)
        // The 256-token pair is paced by its MFMA and LDS work, so scaling X inside every workgroup
        // costs more there than one small launch that writes the normalised input once.  The
        // 64-token pair folds the normalisation into its gate/up kernel unless the slices of the
        // normalisation weight do not fit its LDS beside the rings (very wide d_model): then it
        // takes the same small launch.
        void* xn = (char*)ws + l.xn_off;
        hipError_t e = launch_rmsnorm_weighted(X, norm_w, xn, M, d_model, eps, dtype, st);
        if (e != hipSuccess) return hip_fail(e);
        a.X = xn;
        a.norm_w = nullptr;
    }
    a.trace = nullptr;
    {
        const size_t grid = (size_t)c.splits + (size_t)c.k2_splits * std::max(1, c.k2_col_blocks);   // covers every kernel's grid
        const Registered tr = snapshot(g_trace);
        if (tr.ptr && tr.bytes >= grid * 8 * sizeof(unsigned long long))
            a.trace = (unsigned long long*)tr.ptr;
    }
    // Token chunking on the host: a launch handles at most `per` tokens; further
    // chunks are further launches on the same stream (they re-stream the weights).
    const int per = c.path == DFK_PATH_MFMA ? mfma_max_tokens_per_launch(c, d_model) : valu_max_tokens_per_launch();
    for (int m0 = 0; m0 < M; m0 += per) {
        a.m_base = m0;
        a.m_count = std::min(per, M - m0);
        hipError_t e = c.path == DFK_PATH_MFMA ? launch_mfma(a, c, st) : launch_valu(a, c, dtype, st);
        if (e != hipSuccess) return hip_fail(e);
    }
    return DFK_OK;
}

dfk_status_t run(const void* X, const void* Wg, const void* Wu, const void* Wd, void* Y, int M,
                 int d_model, int d_ff, dfk_dtype_t dtype, const dfk_config_t& c, void* ws,
                 hipStream_t st, const void* norm_w = nullptr, float eps = 0.f, const void* resid = nullptr) {
    return run_in(ws_layout(M, d_model, d_ff), X, Wg, Wu, Wd, Y, M, d_model, d_ff, dtype, c, ws, st, norm_w, eps, resid);
}

dfk_status_t call(const void* X, const void* Wg, const void* Wu, const void* Wd, void* Y, int M,
                  int d_model, int d_ff, dfk_dtype_t dtype, const dfk_config_t* cfg, int want_variant,
                  void* ws, size_t ws_bytes, void* stream, bool wd_t = false) {
    dfk_status_t s = check(X, Wg, Wu, Wd, Y, M, d_model, d_ff, dtype, cfg, ws, ws_bytes, true, false, wd_t);
    if (s != DFK_OK) return s;
    dfk_config_t c;
    if (cfg) c = *cfg;
    else if (wd_t ? !choose_wdt(M, d_model, d_ff, dtype, &c, nullptr)
                  : !choose(M, d_model, d_ff, dtype, want_variant, &c, nullptr)) return DFK_ERR_UNSUPPORTED_SHAPE;
    return run(X, Wg, Wu, Wd, Y, M, d_model, d_ff, dtype, c, ws, (hipStream_t)stream);
}

// ---------------------------------------------------------------- library-owned scratch (dfk_swiglu_mlp_static)
// One array per device, part of the code object, held until the process ends.  In host code its
// name is only a stand-in: the device address comes from hipGetSymbolAddress, once per device, and
// everything below uses that pointer.
constexpr size_t kStaticScratchBytes = (size_t)48 << 20;
constexpr size_t kStaticA2MaxBytes = (size_t)16 << 20;
}  // namespace
}  // namespace dfk

static __device__ __align__(256) unsigned char scratch[dfk::kStaticScratchBytes];

namespace dfk {
namespace {

constexpr int kStaticDevices = 32;
void* g_static_ptr[kStaticDevices];        // device address of `scratch` on each device, NULL until resolved
bool g_static_cleared[kStaticDevices];     // its counter / accumulator part has been zeroed once on that device

// The array's address on the current device (resolved at the first call on that device, with
// that device current), or an error.  *first is set where the caller must enqueue the one-time
// clearing of the part that has to be zero between calls.
hipError_t static_scratch(void** ptr, bool* first) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kStaticDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lk(g_mu);
    if (!g_static_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress((void**)&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p || (uintptr_t)p % 256) return hipErrorInvalidSymbol;
        g_static_ptr[dev] = p;
    }
    *ptr = g_static_ptr[dev];
    *first = !g_static_cleared[dev];
    g_static_cleared[dev] = true;
    return hipSuccess;
}

// Layout inside the array: counters and accumulator first, as in a caller's workspace; then A_2
// at its exact size; what is left is divided 8 : 1 between the partial sums and the group sums.
bool static_layout(int M, int d_ff, WsLayout* l, size_t* p_bytes, size_t* q_bytes) {
    const size_t a2 = align_up((size_t)M * d_ff * 4, 256);
    if (a2 > kStaticA2MaxBytes) return false;
    l->tickets_off = 0;
    l->yacc_off = kWsHeaderBytes;
    l->a2_off = l->yacc_off + kYaccBytes;
    l->p_off = l->a2_off + a2;
    const size_t rest = kStaticScratchBytes - l->p_off;
    *q_bytes = rest / 9 / 256 * 256;
    *p_bytes = (rest - *q_bytes) / 256 * 256;
    l->q_off = l->p_off + *p_bytes;
    l->xn_off = l->total = kStaticScratchBytes;   // no normalised input: this entry point is the plain block
    return true;
}

// The partial-sum blocks a configuration writes in one launch fit p_bytes / q_bytes.
bool partials_fit_static(const dfk_config_t& c, int M, int d_model, size_t p_bytes, size_t q_bytes) {
    if (c.reduce == DFK_REDUCE_ATOMIC) return true;   // accumulator only, already checked against its fixed size
    const int per = c.path == DFK_PATH_MFMA ? mfma_max_tokens_per_launch(c, d_model) : valu_max_tokens_per_launch();
    const size_t tokens = (size_t)std::min(M, per);
    const bool fused = c.variant == DFK_VARIANT_FUSED && !roles_launch(c);
    const size_t blocks = fused ? (size_t)c.splits : (size_t)c.k2_splits;
    const size_t groups = fused ? (blocks + kGroupSize - 1) / kGroupSize : 0;
    return blocks * tokens * d_model * 4 <= p_bytes && groups * tokens * d_model * 4 <= q_bytes;
}

// ---------------------------------------------------------------- tuning scratch
struct Scratch {
    size_t w_bytes, x_bytes, ws_bytes, set_bytes, total;
};
Scratch scratch_layout(int M, int d_model, int d_ff, dfk_dtype_t dtype, int sets) {
    Scratch s;
    s.w_bytes = align_up((size_t)d_ff * d_model * elt_bytes(dtype), 256);
    s.x_bytes = align_up((size_t)M * d_model * elt_bytes(dtype), 256);
    s.ws_bytes = align_up(ws_layout(M, d_model, d_ff).total, 256);
    s.set_bytes = 3 * s.w_bytes;
    s.total = (size_t)sets * s.set_bytes + 2 * s.x_bytes + s.ws_bytes;
    return s;
}

dfk_status_t time_config(const dfk_config_t& c, int M, int d_model, int d_ff, dfk_dtype_t dtype,
                         void* scratch, int sets, int iters, hipStream_t st, bool fill, double* usec) {
    const Scratch s = scratch_layout(M, d_model, d_ff, dtype, sets);
    char* base = (char*)scratch;
    char* X = base + (size_t)sets * s.set_bytes;
    char* Y = X + s.x_bytes;
    char* ws = Y + s.x_bytes;
    hipError_t e;
    if (fill) {
        const float sg = sqrtf(3.0f / (float)d_model), sd = sqrtf(3.0f / (float)d_ff);
        for (int i = 0; i < sets; ++i) {
            char* w = base + (size_t)i * s.set_bytes;
            const size_t n = (size_t)d_ff * d_model;
            if ((e = launch_fill(w, n, dtype, sg, 11u + 3u * i, st)) != hipSuccess) return hip_fail(e);
            if ((e = launch_fill(w + s.w_bytes, n, dtype, sg, 12u + 3u * i, st)) != hipSuccess) return hip_fail(e);
            if ((e = launch_fill(w + 2 * s.w_bytes, n, dtype, sd, 13u + 3u * i, st)) != hipSuccess) return hip_fail(e);
        }
        if ((e = launch_fill(X, (size_t)M * d_model, dtype, 1.7320508f, 7u, st)) != hipSuccess) return hip_fail(e);
        if ((e = launch_zero(ws, s.ws_bytes, st)) != hipSuccess) return hip_fail(e);
    }
    hipEvent_t t0, t1;
    if ((e = hipEventCreate(&t0)) != hipSuccess) return hip_fail(e);
    if ((e = hipEventCreate(&t1)) != hipSuccess) { (void)hipEventDestroy(t0); return hip_fail(e); }
    dfk_status_t rc = DFK_OK;
    for (int it = -2; it < iters && rc == DFK_OK; ++it) {
        if (it == 0 && (e = hipEventRecord(t0, st)) != hipSuccess) { rc = hip_fail(e); break; }
        char* w = base + (size_t)((it + 2) % sets) * s.set_bytes;
        rc = run(X, w, w + s.w_bytes, w + 2 * s.w_bytes, Y, M, d_model, d_ff, dtype, c, ws, st);
    }
    if (rc == DFK_OK) {
        if ((e = hipEventRecord(t1, st)) != hipSuccess) rc = hip_fail(e);
        else if ((e = hipEventSynchronize(t1)) != hipSuccess) rc = hip_fail(e);
        else {
            float ms = 0.f;
            if ((e = hipEventElapsedTime(&ms, t0, t1)) != hipSuccess) rc = hip_fail(e);
            else *usec = (double)ms * 1000.0 / iters;
        }
    }
    (void)hipEventDestroy(t0);
    (void)hipEventDestroy(t1);
    return rc;
}

// Same protocol as time_config, for each launch of the call on its own: `iters` gate/up
// launches back to back between two events, then `iters` down launches (they read the A_2
// the last gate/up launch left; every launch leaves the workspace clean).
dfk_status_t time_kernels(const dfk_config_t& c, int M, int d_model, int d_ff, dfk_dtype_t dtype,
                          void* scratch, int sets, int iters, hipStream_t st, double* usec2) {
    double whole = 0.0;
    dfk_status_t rc = time_config(c, M, d_model, d_ff, dtype, scratch, sets, 1, st, true, &whole);   // fill + warm-up
    if (rc != DFK_OK) return rc;
    const Scratch s = scratch_layout(M, d_model, d_ff, dtype, sets);
    char* base = (char*)scratch;
    char* X = base + (size_t)sets * s.set_bytes;
    char* Y = X + s.x_bytes;
    char* ws = Y + s.x_bytes;
    hipEvent_t t0, t1;
    hipError_t e;
    if ((e = hipEventCreate(&t0)) != hipSuccess) return hip_fail(e);
    if ((e = hipEventCreate(&t1)) != hipSuccess) { (void)hipEventDestroy(t0); return hip_fail(e); }
    usec2[0] = usec2[1] = 0.0;
    const int stages = c.variant == DFK_VARIANT_FUSED && !roles_launch(c) ? 1 : 2;   // (head and tail of the launch with both roles)
    for (int k = 0; k < stages && rc == DFK_OK; ++k) {
        g_stage_mask = 1 << k;
        for (int it = -2; it < iters && rc == DFK_OK; ++it) {
            if (it == 0 && (e = hipEventRecord(t0, st)) != hipSuccess) { rc = hip_fail(e); break; }
            char* w = base + (size_t)((it + 2) % sets) * s.set_bytes;
            rc = run(X, w, w + s.w_bytes, w + 2 * s.w_bytes, Y, M, d_model, d_ff, dtype, c, ws, st);
        }
        g_stage_mask = 3;
        if (rc != DFK_OK) break;
        float ms = 0.f;
        if ((e = hipEventRecord(t1, st)) != hipSuccess || (e = hipEventSynchronize(t1)) != hipSuccess ||
            (e = hipEventElapsedTime(&ms, t0, t1)) != hipSuccess) { rc = hip_fail(e); break; }
        usec2[k] = (double)ms * 1000.0 / iters;
    }
    g_stage_mask = 3;
    (void)hipEventDestroy(t0);
    (void)hipEventDestroy(t1);
    return rc;
}

}  // namespace
}  // namespace dfk

using namespace dfk;

extern "C" {

dfk_status_t dfk_swiglu_mlp(const void* X, const void* Wg, const void* Wu, const void* Wd, void* Y,
                            int M, int d_model, int d_ff, void* stream) {
    const Registered ws = snapshot(g_ws);
    return call(X, Wg, Wu, Wd, Y, M, d_model, d_ff, DFK_BF16, nullptr, DFK_VARIANT_AUTO, ws.ptr, ws.bytes, stream);
}

dfk_status_t dfk_swiglu_mlp_fused(const void* X, const void* Wg, const void* Wu, const void* Wd,
                                  void* Y, int M, int d_model, int d_ff, void* stream) {
    const Registered ws = snapshot(g_ws);
    return call(X, Wg, Wu, Wd, Y, M, d_model, d_ff, DFK_BF16, nullptr, DFK_VARIANT_FUSED, ws.ptr, ws.bytes, stream);
}

dfk_status_t dfk_swiglu_mlp_unfused(const void* X, const void* Wg, const void* Wu, const void* Wd,
                                    void* Y, int M, int d_model, int d_ff, void* stream) {
    const Registered ws = snapshot(g_ws);
    return call(X, Wg, Wu, Wd, Y, M, d_model, d_ff, DFK_BF16, nullptr, DFK_VARIANT_TWO_KERNEL, ws.ptr, ws.bytes, stream);
}

dfk_status_t dfk_swiglu_mlp_ex(const void* X, const void* Wg, const void* Wu, const void* Wd, void* Y,
                               int M, int d_model, int d_ff, dfk_dtype_t dtype,
                               const dfk_config_t* cfg, void* workspace, size_t workspace_bytes,
                               void* stream) {
    return call(X, Wg, Wu, Wd, Y, M, d_model, d_ff, dtype, cfg, DFK_VARIANT_AUTO, workspace,
                workspace_bytes, stream);
}

dfk_status_t dfk_swiglu_mlp_wdt(const void* X, const void* Wg, const void* Wu, const void* Wd_t, void* Y,
                                int M, int d_model, int d_ff, dfk_dtype_t dtype,
                                const dfk_config_t* cfg, void* workspace, size_t workspace_bytes,
                                void* stream) {
    return call(X, Wg, Wu, Wd_t, Y, M, d_model, d_ff, dtype, cfg, DFK_VARIANT_AUTO, workspace,
                workspace_bytes, stream, true);
}

dfk_status_t dfk_swiglu_mlp_static(const void* X, const void* Wg, const void* Wu, const void* Wd, void* Y,
                                   int M, int d_model, int d_ff, dfk_dtype_t dtype, const dfk_config_t* cfg,
                                   void* stream) {
    dfk_status_t s = check(X, Wg, Wu, Wd, Y, M, d_model, d_ff, dtype, cfg, nullptr, 0, false);
    if (s != DFK_OK) return s;
    WsLayout l;
    size_t p_bytes = 0, q_bytes = 0;
    if (!static_layout(M, d_ff, &l, &p_bytes, &q_bytes)) return DFK_ERR_WORKSPACE;   // A_2 beyond the array's share
    dfk_config_t c;
    if (cfg) {
        c = *cfg;
        if (!partials_fit_static(c, M, d_model, p_bytes, q_bytes)) return DFK_ERR_WORKSPACE;
    } else {
        if (!choose(M, d_model, d_ff, dtype, DFK_VARIANT_AUTO, &c, nullptr)) return DFK_ERR_UNSUPPORTED_SHAPE;
        if (!partials_fit_static(c, M, d_model, p_bytes, q_bytes)) {   // the first candidate that fits instead
            bool found = false;
            for (const auto& k : candidates(M, d_model, d_ff, dtype))
                if (partials_fit_static(k, M, d_model, p_bytes, q_bytes)) { c = k; found = true; break; }
            if (!found) return DFK_ERR_WORKSPACE;
        }
    }
    void* ws = nullptr;
    bool first = false;
    if (hipError_t e = static_scratch(&ws, &first); e != hipSuccess) return hip_fail(e);
    const size_t nx = (size_t)M * d_model * elt_bytes(dtype), nw = (size_t)d_ff * d_model * elt_bytes(dtype);
    if (overlaps(ws, kStaticScratchBytes, Y, nx) || overlaps(ws, kStaticScratchBytes, X, nx) ||
        overlaps(ws, kStaticScratchBytes, Wg, nw) || overlaps(ws, kStaticScratchBytes, Wu, nw) ||
        overlaps(ws, kStaticScratchBytes, Wd, nw))
        return DFK_ERR_ALIAS;
    if (first) {   // counters and accumulator start from zero (a fill kernel on the caller's stream); calls keep them zero
        if (hipError_t e = launch_zero(ws, kWsHeaderBytes + kYaccBytes, (hipStream_t)stream); e != hipSuccess) return hip_fail(e);
    }
    return run_in(l, X, Wg, Wu, Wd, Y, M, d_model, d_ff, dtype, c, ws, (hipStream_t)stream);
}

namespace {
dfk_status_t mlp_block(const void* H, const void* norm_weight, float eps, const void* Wg,
                       const void* Wu, const void* Wd, void* H_out, int M, int d_model, int d_ff,
                       dfk_dtype_t dtype, const dfk_config_t* cfg, void* workspace,
                       size_t workspace_bytes, void* stream, bool wd_t) {
    if (!H || !norm_weight || !H_out) return DFK_ERR_INVALID_ARG;
    if (!(eps >= 0.f) || !(eps < 1e30f)) return DFK_ERR_INVALID_ARG;
    if (dtype != DFK_BF16 && dtype != DFK_FP16)
        return dtype == DFK_FP32 ? DFK_ERR_UNSUPPORTED_SHAPE : DFK_ERR_INVALID_ARG;
    if ((uintptr_t)norm_weight % 16) return DFK_ERR_ALIGNMENT;
    // The output may be the input itself (the residual stream updated in place); any other
    // overlap is refused.
    dfk_status_t s = check(H, Wg, Wu, Wd, H_out, M, d_model, d_ff, dtype, cfg, workspace, workspace_bytes, true, true, wd_t);
    if (s != DFK_OK) return s;
    {
        const size_t nx = (size_t)M * d_model * 2, nv = (size_t)d_model * 2;
        if (overlaps(H_out, nx, norm_weight, nv) || overlaps(workspace, workspace_bytes, norm_weight, nv))
            return DFK_ERR_ALIAS;
    }
    auto carries = [&](const dfk_config_t& k) {
        if (wd_t) return k.path == DFK_PATH_MFMA && k.kmajor == 5 && mfma_km_t_config_valid(k, M, d_model, d_ff, dtype);
        return k.path == DFK_PATH_MFMA &&
               ((k.kmajor == 1 && mfma_km_config_valid(k, M, d_model, d_ff, dtype)) ||
                (k.kmajor == 2 && mfma_big_config_valid(k, M, d_model, d_ff, dtype)));
    };
    dfk_config_t c;
    if (cfg) c = *cfg;
    else {
        if (wd_t ? !choose_wdt(M, d_model, d_ff, dtype, &c, nullptr)
                 : !choose(M, d_model, d_ff, dtype, DFK_VARIANT_TWO_KERNEL, &c, nullptr)) return DFK_ERR_UNSUPPORTED_SHAPE;
        if (!carries(c)) {   // the scheduler's pick is another kernel family: first candidate that carries this form
            bool found = false;
            for (const auto& k : wd_t ? candidates_wdt(M, d_model, d_ff, dtype) : candidates(M, d_model, d_ff, dtype))
                if (k.variant == DFK_VARIANT_TWO_KERNEL && carries(k)) { c = k; found = true; break; }
            if (!found) return DFK_ERR_UNSUPPORTED_SHAPE;
        }
    }
    if (!carries(c)) return DFK_ERR_UNSUPPORTED_SHAPE;
    return run(H, Wg, Wu, Wd, H_out, M, d_model, d_ff, dtype, c, workspace, (hipStream_t)stream, norm_weight, eps, H);
}
}  // namespace

dfk_status_t dfk_mlp_block(const void* H, const void* norm_weight, float eps, const void* Wg,
                           const void* Wu, const void* Wd, void* H_out, int M, int d_model, int d_ff,
                           dfk_dtype_t dtype, const dfk_config_t* cfg, void* workspace,
                           size_t workspace_bytes, void* stream) {
    return mlp_block(H, norm_weight, eps, Wg, Wu, Wd, H_out, M, d_model, d_ff, dtype, cfg, workspace, workspace_bytes, stream, false);
}

dfk_status_t dfk_mlp_block_wdt(const void* H, const void* norm_weight, float eps, const void* Wg,
                               const void* Wu, const void* Wd_t, void* H_out, int M, int d_model, int d_ff,
                               dfk_dtype_t dtype, const dfk_config_t* cfg, void* workspace,
                               size_t workspace_bytes, void* stream) {
    return mlp_block(H, norm_weight, eps, Wg, Wu, Wd_t, H_out, M, d_model, d_ff, dtype, cfg, workspace, workspace_bytes, stream, true);
}

dfk_status_t dfk_check_args(const void* X, const void* Wg, const void* Wu, const void* Wd,
                            const void* Y, int M, int d_model, int d_ff, dfk_dtype_t dtype,
                            const dfk_config_t* cfg, const void* workspace, size_t workspace_bytes) {
    return check(X, Wg, Wu, Wd, Y, M, d_model, d_ff, dtype, cfg, workspace, workspace_bytes, false);
}

size_t dfk_workspace_bytes(int M_max, int d_model, int d_ff) {
    if (!shape_supported(M_max, d_model, d_ff)) return 0;
    return ws_layout(M_max, d_model, d_ff).total;
}

dfk_status_t dfk_workspace_init(void* workspace, size_t workspace_bytes, void* stream) {
    if (!workspace || workspace_bytes == 0) return DFK_ERR_INVALID_ARG;
    if ((uintptr_t)workspace % 256) return DFK_ERR_ALIGNMENT;
    hipError_t e = launch_zero(workspace, workspace_bytes, (hipStream_t)stream);
    return e == hipSuccess ? DFK_OK : hip_fail(e);
}

dfk_status_t dfk_set_workspace(void* workspace, size_t workspace_bytes) {
    if (workspace && (uintptr_t)workspace % 256) return DFK_ERR_ALIGNMENT;
    if (workspace && workspace_bytes == 0) return DFK_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> lk(g_mu);
    g_ws.ptr = workspace;
    g_ws.bytes = workspace ? workspace_bytes : 0;
    return DFK_OK;
}

dfk_status_t dfk_set_trace_buffer(void* buffer, size_t bytes) {
    if (buffer && (uintptr_t)buffer % 8) return DFK_ERR_ALIGNMENT;
    std::lock_guard<std::mutex> lk(g_mu);
    g_trace.ptr = buffer;
    g_trace.bytes = buffer ? bytes : 0;
    return DFK_OK;
}

int dfk_num_candidates_wdt(int M, int d_model, int d_ff, dfk_dtype_t dtype) {
    if (!shape_supported(M, d_model, d_ff)) return 0;
    return (int)candidates_wdt(M, d_model, d_ff, dtype).size();
}

dfk_status_t dfk_get_candidate_wdt(int M, int d_model, int d_ff, dfk_dtype_t dtype, int i, dfk_config_t* out) {
    if (!out) return DFK_ERR_INVALID_ARG;
    if (!shape_supported(M, d_model, d_ff)) return DFK_ERR_UNSUPPORTED_SHAPE;
    auto c = candidates_wdt(M, d_model, d_ff, dtype);
    if (i < 0 || i >= (int)c.size()) return DFK_ERR_NOT_FOUND;
    *out = c[i];
    return DFK_OK;
}

dfk_status_t dfk_get_choice_wdt(int M, int d_model, int d_ff, dfk_dtype_t dtype, dfk_config_t* out, int* tuned_out) {
    if (!out) return DFK_ERR_INVALID_ARG;
    if (M < 1 || d_model < 1 || d_ff < 1) return DFK_ERR_INVALID_ARG;
    if (!shape_supported(M, d_model, d_ff)) return DFK_ERR_UNSUPPORTED_SHAPE;
    return choose_wdt(M, d_model, d_ff, dtype, out, tuned_out) ? DFK_OK : DFK_ERR_UNSUPPORTED_SHAPE;
}

int dfk_num_candidates(int M, int d_model, int d_ff, dfk_dtype_t dtype) {
    if (!shape_supported(M, d_model, d_ff)) return 0;
    return (int)candidates(M, d_model, d_ff, dtype).size();
}

dfk_status_t dfk_get_candidate(int M, int d_model, int d_ff, dfk_dtype_t dtype, int i,
                               dfk_config_t* out) {
    if (!out) return DFK_ERR_INVALID_ARG;
    if (!shape_supported(M, d_model, d_ff)) return DFK_ERR_UNSUPPORTED_SHAPE;
    auto c = candidates(M, d_model, d_ff, dtype);
    if (i < 0 || i >= (int)c.size()) return DFK_ERR_NOT_FOUND;
    *out = c[i];
    return DFK_OK;
}

int dfk_config_valid(const dfk_config_t* cfg, int M, int d_model, int d_ff, dfk_dtype_t dtype) {
    if (!cfg) return 0;
    return config_valid(*cfg, M, d_model, d_ff, dtype) ? 1 : 0;
}

size_t dfk_tune_scratch_bytes(int M_max, int d_model, int d_ff, dfk_dtype_t dtype, int sets) {
    if (!shape_supported(M_max, d_model, d_ff) || sets < 1) return 0;
    return scratch_layout(M_max, d_model, d_ff, dtype, sets).total;
}

dfk_status_t dfk_time_config(const dfk_config_t* cfg, int M, int d_model, int d_ff, dfk_dtype_t dtype,
                             void* scratch, size_t scratch_bytes, int sets, int iters, void* stream,
                             double* usec_out) {
    if (!cfg || !scratch || !usec_out || sets < 1 || iters < 1) return DFK_ERR_INVALID_ARG;
    if (M < 1 || d_model < 1 || d_ff < 1) return DFK_ERR_INVALID_ARG;
    if (!shape_supported(M, d_model, d_ff)) return DFK_ERR_UNSUPPORTED_SHAPE;
    if (!config_valid(*cfg, M, d_model, d_ff, dtype)) return DFK_ERR_UNSUPPORTED_SHAPE;
    if ((uintptr_t)scratch % 256) return DFK_ERR_ALIGNMENT;
    if (scratch_bytes < scratch_layout(M, d_model, d_ff, dtype, sets).total) return DFK_ERR_WORKSPACE;
    return time_config(*cfg, M, d_model, d_ff, dtype, scratch, sets, iters, (hipStream_t)stream, true,
                       usec_out);
}

dfk_status_t dfk_time_kernels(const dfk_config_t* cfg, int M, int d_model, int d_ff, dfk_dtype_t dtype,
                              void* scratch, size_t scratch_bytes, int sets, int iters, void* stream,
                              double* usec_out) {
    if (!cfg || !scratch || !usec_out || sets < 1 || iters < 1 || iters > 1024) return DFK_ERR_INVALID_ARG;
    if (M < 1 || d_model < 1 || d_ff < 1) return DFK_ERR_INVALID_ARG;
    if (!shape_supported(M, d_model, d_ff)) return DFK_ERR_UNSUPPORTED_SHAPE;
    if (!config_valid(*cfg, M, d_model, d_ff, dtype)) return DFK_ERR_UNSUPPORTED_SHAPE;
    const int per = cfg->path == DFK_PATH_MFMA ? mfma_max_tokens_per_launch(*cfg, d_model) : valu_max_tokens_per_launch();
    if (M > per) return DFK_ERR_UNSUPPORTED_SHAPE;   // one set of launches per call only
    if ((uintptr_t)scratch % 256) return DFK_ERR_ALIGNMENT;
    if (scratch_bytes < scratch_layout(M, d_model, d_ff, dtype, sets).total) return DFK_ERR_WORKSPACE;
    return time_kernels(*cfg, M, d_model, d_ff, dtype, scratch, sets, iters, (hipStream_t)stream, usec_out);
}

dfk_status_t dfk_tune(const int* M_list, int nM, int d_model, int d_ff, dfk_dtype_t dtype,
                      void* scratch, size_t scratch_bytes, int sets, int iters, void* stream) {
    if (!M_list || nM < 1 || !scratch || sets < 1 || iters < 1) return DFK_ERR_INVALID_ARG;
    if (d_model < 1 || d_ff < 1) return DFK_ERR_INVALID_ARG;
    if (!shape_supported(1, d_model, d_ff)) return DFK_ERR_UNSUPPORTED_SHAPE;
    if ((uintptr_t)scratch % 256) return DFK_ERR_ALIGNMENT;
    for (int i = 0; i < nM; ++i) {
        if (M_list[i] < 1) return DFK_ERR_INVALID_ARG;
        if (M_list[i] > DFK_MAX_M) return DFK_ERR_UNSUPPORTED_SHAPE;
        if (scratch_bytes < scratch_layout(M_list[i], d_model, d_ff, dtype, sets).total)
            return DFK_ERR_WORKSPACE;
    }
    g_tune_skipped = 0;
    g_tune_skip_status = DFK_OK;
    for (int i = 0; i < nM; ++i) {
        const int M = M_list[i];
        auto cands = candidates(M, d_model, d_ff, dtype);
        if (cands.empty()) return DFK_ERR_UNSUPPORTED_SHAPE;
        Entry best, best_of[3];
        best.usec = best_of[1].usec = best_of[2].usec = -1.0;
        bool fill = true;  // scratch layout depends on M: refill once per M (until a candidate has run)
        for (const auto& c : cands) {
            double us = 0.0;
            dfk_status_t s = time_config(c, M, d_model, d_ff, dtype, scratch, sets, iters,
                                         (hipStream_t)stream, fill, &us);
            if (s != DFK_OK) {   // a candidate that cannot be timed is left out, not the whole tune
                ++g_tune_skipped;
                g_tune_skip_status = s;
                continue;
            }
            fill = false;
            if (best.usec < 0.0 || us < best.usec) { best.cfg = c; best.usec = us; }
            Entry& bv = best_of[c.variant == DFK_VARIANT_FUSED ? 1 : 2];
            if (bv.usec < 0.0 || us < bv.usec) { bv.cfg = c; bv.usec = us; }
        }
        if (best.usec < 0.0) return g_tune_skip_status;   // every candidate of this M failed
        // the candidates for W_down as [d_model, d_ff] (timing does not depend on what the synthetic weights mean)
        Entry best_t;
        best_t.usec = -1.0;
        for (const auto& c : candidates_wdt(M, d_model, d_ff, dtype)) {
            double us = 0.0;
            dfk_status_t s = time_config(c, M, d_model, d_ff, dtype, scratch, sets, iters, (hipStream_t)stream, false, &us);
            if (s != DFK_OK) {
                ++g_tune_skipped;
                g_tune_skip_status = s;
                continue;
            }
            if (best_t.usec < 0.0 || us < best_t.usec) { best_t.cfg = c; best_t.usec = us; }
        }
        std::lock_guard<std::mutex> lk(g_mu);
        for (int v = 1; v <= 2; ++v)
            if (best_of[v].usec >= 0.0) table_put(M, d_model, d_ff, (int)dtype, best_of[v], false);
        if (best_t.usec >= 0.0) table_put(M, d_model, d_ff, (int)dtype, best_t, false);
        table_put(M, d_model, d_ff, (int)dtype, best, true);
    }
    return DFK_OK;
}

int dfk_tune_skipped(dfk_status_t* last_status_out) {
    if (last_status_out) *last_status_out = g_tune_skip_status;
    return g_tune_skipped;
}

dfk_status_t dfk_get_choice(int M, int d_model, int d_ff, dfk_dtype_t dtype, dfk_config_t* out,
                            int* tuned_out) {
    if (!out) return DFK_ERR_INVALID_ARG;
    if (M < 1 || d_model < 1 || d_ff < 1) return DFK_ERR_INVALID_ARG;
    if (!shape_supported(M, d_model, d_ff)) return DFK_ERR_UNSUPPORTED_SHAPE;
    return choose(M, d_model, d_ff, dtype, DFK_VARIANT_AUTO, out, tuned_out) ? DFK_OK
                                                                             : DFK_ERR_UNSUPPORTED_SHAPE;
}

dfk_status_t dfk_set_choice(int M, int d_model, int d_ff, dfk_dtype_t dtype, const dfk_config_t* cfg,
                            double usec) {
    if (!cfg || M < 1 || d_model < 1 || d_ff < 1) return DFK_ERR_INVALID_ARG;
    if (!shape_supported(M, d_model, d_ff)) return DFK_ERR_UNSUPPORTED_SHAPE;
    if (!config_valid(*cfg, M, d_model, d_ff, dtype)) return DFK_ERR_UNSUPPORTED_SHAPE;
    std::lock_guard<std::mutex> lk(g_mu);
    Entry e;
    e.cfg = *cfg;
    e.usec = usec;
    table_put(M, d_model, d_ff, (int)dtype, e, true);
    return DFK_OK;
}

void dfk_clear_tuning(void) {
    std::lock_guard<std::mutex> lk(g_mu);
    g_table.clear();
}

dfk_status_t dfk_save_tuning(const char* path) {
    if (!path) return DFK_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> lk(g_mu);
    FILE* f = std::fopen(path, "w");
    if (!f) return DFK_ERR_IO;
    std::fprintf(f, "# dfk tuning table v2: M d_model d_ff dtype variant path splits waves depth reduce "
                    "k2_splits k2_col_blocks a2_dtype k2_rows_by_wave kmajor usec\n");
    // One line per entry; a problem's chosen configuration comes after its other variant's line, and the loader
    // takes the last line of a problem as the choice.
    for (int pass = 0; pass < 2; ++pass)
        for (const auto& kv : g_table) {
            const int slot = std::get<4>(kv.first);
            const dfk_config_t& c = kv.second.cfg;
            if (pass == 0) {
                if (slot == 0) continue;
                auto chosen = g_table.find(Key(std::get<0>(kv.first), std::get<1>(kv.first), std::get<2>(kv.first),
                                               std::get<3>(kv.first), 0));
                if (chosen != g_table.end() && same_cfg(chosen->second.cfg, c)) continue;   // written in the second pass
            } else if (slot != 0) {
                continue;
            }
            std::fprintf(f, "%d %d %d %d %d %d %d %d %d %d %d %d %d %d %d %.3f\n", std::get<0>(kv.first),
                         std::get<1>(kv.first), std::get<2>(kv.first), std::get<3>(kv.first), c.variant,
                         c.path, c.splits, c.waves, c.depth, c.reduce, c.k2_splits, c.k2_col_blocks,
                         c.a2_dtype, c.k2_rows_by_wave, c.kmajor, kv.second.usec);
        }
    const bool ok = std::fclose(f) == 0;
    return ok ? DFK_OK : DFK_ERR_IO;
}

dfk_status_t dfk_load_tuning(const char* path) {
    if (!path) return DFK_ERR_INVALID_ARG;
    FILE* f = std::fopen(path, "r");
    if (!f) return DFK_ERR_IO;
    std::vector<std::pair<Key, Entry>> fresh;   // in file order
    char line[512];
    dfk_status_t rc = DFK_OK;
    while (std::fgets(line, sizeof line, f)) {
        const char* p = line;
        while (*p == ' ' || *p == '\t') ++p;
        if (*p == '#' || *p == '\n' || *p == '\r' || *p == 0) continue;
        int M, dm, df, dt;
        Entry e;
        std::memset(&e, 0, sizeof e);
        const int n = std::sscanf(p, "%d %d %d %d %d %d %d %d %d %d %d %d %d %d %d %lf", &M, &dm, &df, &dt,
                                  &e.cfg.variant, &e.cfg.path, &e.cfg.splits, &e.cfg.waves, &e.cfg.depth,
                                  &e.cfg.reduce, &e.cfg.k2_splits, &e.cfg.k2_col_blocks, &e.cfg.a2_dtype,
                                  &e.cfg.k2_rows_by_wave, &e.cfg.kmajor, &e.usec);
        if (n != 16 || M < 1 || M > DFK_MAX_M || (dt != DFK_BF16 && dt != DFK_FP32 && dt != DFK_FP16) || dm < 8 ||
            df < 8 || dm % 8 || df % 8 || !config_valid(e.cfg, M, dm, df, (dfk_dtype_t)dt)) {
            rc = DFK_ERR_IO;
            break;
        }
        fresh.emplace_back(Key(M, dm, df, dt, 0), e);
    }
    std::fclose(f);
    if (rc != DFK_OK) return rc;  // table left untouched on a malformed file
    std::lock_guard<std::mutex> lk(g_mu);
    for (const auto& kv : fresh)
        table_put(std::get<0>(kv.first), std::get<1>(kv.first), std::get<2>(kv.first), std::get<3>(kv.first), kv.second, true);
    return DFK_OK;
}

dfk_status_t dfk_transpose_w_down(const void* Wd, void* Wd_t, int d_model, int d_ff, dfk_dtype_t dtype, void* stream) {
    if (!Wd || !Wd_t || d_model < 1 || d_ff < 1) return DFK_ERR_INVALID_ARG;
    if (dtype != DFK_BF16 && dtype != DFK_FP32 && dtype != DFK_FP16) return DFK_ERR_INVALID_ARG;
    if ((uintptr_t)Wd % 16 || (uintptr_t)Wd_t % 16) return DFK_ERR_ALIGNMENT;
    if ((d_ff + 31) / 32 > 65535) return DFK_ERR_UNSUPPORTED_SHAPE;
    const size_t nw = (size_t)d_ff * d_model * elt_bytes(dtype);
    if (overlaps(Wd, nw, Wd_t, nw)) return DFK_ERR_ALIAS;
    hipError_t e = launch_transpose(Wd, Wd_t, d_ff, d_model, dtype, (hipStream_t)stream);
    return e == hipSuccess ? DFK_OK : hip_fail(e);
}

dfk_status_t dfk_rms_normalize(const void* in, void* out, int M, int d_model, void* stream) {
    if (!in || !out || M < 1 || d_model < 1) return DFK_ERR_INVALID_ARG;
    if (M > 65535) return DFK_ERR_UNSUPPORTED_SHAPE;
    hipError_t e = launch_rms_normalize(in, out, M, d_model, (hipStream_t)stream);
    return e == hipSuccess ? DFK_OK : hip_fail(e);
}

dfk_status_t dfk_stream_read(const void* src, size_t bytes, void* sink, void* stream) {
    if (!src || !sink || bytes == 0) return DFK_ERR_INVALID_ARG;
    if (bytes % 16) return DFK_ERR_UNSUPPORTED_SHAPE;
    if ((uintptr_t)src % 16 || (uintptr_t)sink % 8) return DFK_ERR_ALIGNMENT;
    hipError_t e = launch_stream_read(src, bytes, sink, (hipStream_t)stream);
    return e == hipSuccess ? DFK_OK : hip_fail(e);
}

dfk_status_t dfk_read_gateup_pattern(const void* Wg, const void* Wu, int d_model, int d_ff, int splits, int waves,
                                     void* sink, void* stream) {
    if (!Wg || !Wu || !sink || d_model < 1 || d_ff < 1 || splits < 1) return DFK_ERR_INVALID_ARG;
    if (waves != 4 && waves != 8) return DFK_ERR_INVALID_ARG;
    if (d_ff % 8 || d_model % (128 * waves) || d_model > kMaxDModel || splits > d_ff / 8 || splits > 65535)
        return DFK_ERR_UNSUPPORTED_SHAPE;
    if ((uintptr_t)Wg % 16 || (uintptr_t)Wu % 16 || (uintptr_t)sink % 8) return DFK_ERR_ALIGNMENT;
    hipError_t e = launch_read_gateup_pattern(Wg, Wu, d_model, d_ff, splits, waves, sink, (hipStream_t)stream);
    return e == hipSuccess ? DFK_OK : hip_fail(e);
}

dfk_status_t dfk_fill_synthetic(void* dst, size_t elems, dfk_dtype_t dtype, float scale, unsigned seed,
                                void* stream) {
    if (!dst || elems == 0) return DFK_ERR_INVALID_ARG;
    if (dtype != DFK_BF16 && dtype != DFK_FP32 && dtype != DFK_FP16) return DFK_ERR_INVALID_ARG;
    if ((uintptr_t)dst % 4) return DFK_ERR_ALIGNMENT;
    hipError_t e = launch_fill(dst, elems, dtype, scale, seed, (hipStream_t)stream);
    return e == hipSuccess ? DFK_OK : hip_fail(e);
}

const char* dfk_status_string(dfk_status_t s) {
    switch (s) {
        case DFK_OK: return "ok";
        case DFK_ERR_INVALID_ARG: return "invalid argument";
        case DFK_ERR_UNSUPPORTED_SHAPE: return "unsupported shape or configuration";
        case DFK_ERR_ALIGNMENT: return "pointer not sufficiently aligned";
        case DFK_ERR_ALIAS: return "output or workspace overlaps an input";
        case DFK_ERR_WORKSPACE: return "workspace missing or too small";
        case DFK_ERR_HIP: return "HIP call failed";
        case DFK_ERR_IO: return "tuning file could not be read, written or parsed";
        case DFK_ERR_NOT_FOUND: return "not found";
    }
    return "unknown status";
}

int dfk_last_hip_error(void) { return g_last_hip_error; }

const char* dfk_version(void) { return "dfk 0.2 (gfx950)"; }

}  // extern "C"
