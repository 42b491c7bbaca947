// Internal declarations shared by the translation units of libdfk (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <atomic>
#include <stddef.h>
#include <stdint.h>

#include "dfk.h"

namespace dfk {

// ---------------------------------------------------------------- workspace layout
// [0, 4096)        arrival counters (unsigned), zero between calls
// [4096, +8 MiB)   fp32 accumulator of Y for one launch ([tokens of the launch][d_model], at most 8 MiB),
//                  zero between calls (atomic reduction)
// [.., +P)         fp32 partial sums of Y, one [tokens, d_model] block per workgroup slice
//                  (counter reduction)
// [.., +Q)         fp32 group sums (second level of the counter reduction)
// [.., +M*d_ff*4)  A_2 between the two launches of the two-kernel variant
// [.., +M*d_model*2) the normalised input of dfk_mlp_block where the normalisation is a launch of its own
// The part that has to be zero between calls comes first and has a fixed size, so
// calls of different shapes on one workspace never put scratch where another call
// expects zeros.
constexpr size_t kWsHeaderBytes = 4096;
constexpr int kMaxTickets = 1024;
constexpr int kTicketLevel2 = 512;          // counters [0,512): level 1 / column blocks, [512,1024): level 2
constexpr int kYaccTokens = 64;             // rows of the fp32 accumulator at the widest d_model (its size is fixed, see above)
constexpr int kMaxDModel = 32768;
constexpr size_t kYaccBytes = (size_t)kYaccTokens * kMaxDModel * 4;
constexpr size_t kPartialCapBytes = (size_t)128 << 20;
constexpr int kGroupSize = 16;              // workgroup partials summed per first-level group

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

inline size_t partial_bytes(int M, int d_model) {
    const size_t want = (size_t)1024 * (M < kYaccTokens ? M : kYaccTokens) * d_model * 4;
    return want < kPartialCapBytes ? want : kPartialCapBytes;
}

struct WsLayout {
    size_t tickets_off, yacc_off, p_off, q_off, a2_off, xn_off, total;
};

inline WsLayout ws_layout(int M, int d_model, int d_ff) {
    WsLayout l;
    l.tickets_off = 0;
    l.yacc_off = kWsHeaderBytes;
    l.p_off = l.yacc_off + kYaccBytes;
    l.q_off = l.p_off + align_up(partial_bytes(M, d_model), 256);
    l.a2_off = l.q_off + align_up(partial_bytes(M, d_model) / 8, 256);
    l.xn_off = l.a2_off + align_up((size_t)M * d_ff * 4, 256);
    l.total = l.xn_off + align_up((size_t)M * d_model * 2, 256);
    return l;
}

// true if `splits` partial blocks of `tokens` x d_model fp32 fit the partial area sized for M
inline bool partials_fit(int splits, int tokens, int M, int d_model) {
    const size_t need = (size_t)splits * tokens * d_model * 4;
    const size_t groups = (size_t)(splits + kGroupSize - 1) / kGroupSize;
    return need <= partial_bytes(M, d_model) && groups * tokens * d_model * 4 <= partial_bytes(M, d_model) / 8;
}

// ---------------------------------------------------------------- kernel arguments
struct MlpArgs {
    const void* X;
    const void* Wg;
    const void* Wu;
    const void* Wd;
    void* Y;
    int M, d_model, d_ff;
    int m_base;        // first token this launch handles (host-side token chunking)
    int m_count;       // tokens this launch handles (at most what the kernels of the configuration take)
    int splits;        // d_ff slices (grid of the fused kernel / first kernel)
    int k2_splits, k2_col_blocks;
    int dtype;         // dfk_dtype_t of X, the weights and Y
    int a2_is_fp32;    // storage type of A_2 in the workspace (two-kernel variant): fp32, else the 16-bit input type
    int reduce_mode;   // dfk_reduce_t
    float* yacc;       // [m_count, d_model] fp32 accumulator, zero on entry and on exit (atomic reduction)
    float* P;          // partial sums [slice][m_count][d_model]
    float* Q;          // group sums   [group][m_count][d_model]
    unsigned* tickets; // zero on entry and on exit
    void* a2;          // [M, d_ff] in the workspace
    unsigned long long* trace;  // optional [workgroup][8] wall-clock stamps (NULL = off)
    // Pre-norm residual form (kernel pair for up to 64 tokens only; all NULL / 0 otherwise):
    const void* norm_w;  // [d_model] weight of the RMS normalisation applied to X on the way in
    float eps;           // added to the mean square under the root
    const void* resid;   // [M, d_model] added to the result at the final store (may be Y itself)
};

// d_ff is cut into slices at multiples of 8 rows: slice s of S covers the
// 8-row groups [s*NG/S, (s+1)*NG/S), NG = d_ff/8.
__host__ __device__ inline void slice_rows(int d_ff, int S, int s, int& j0, int& j1) {
    const long long ng = d_ff / 8;
    j0 = (int)(ng * s / S) * 8;
    j1 = (int)(ng * (s + 1) / S) * 8;
}

inline int max_slice_rows(int d_ff, int S) {
    const long long ng = d_ff / 8;
    return (int)((ng + S - 1) / S) * 8;
}

// ---------------------------------------------------------------- per-launch timing
// Which launches of a call the launchers issue on the calling thread: bit 0 the first
// (fused kernel, or gate/up kernel), bit 1 the second (down kernel).  3 except inside
// dfk_time_kernels, which times each launch on its own, back to back.
extern thread_local int g_stage_mask;

// ---------------------------------------------------------------- dynamic-LDS allowance of a kernel
// hipFuncSetAttribute(MaxDynamicSharedMemorySize) applies to a function on one device.  Each launcher
// keeps one of these per kernel instantiation (a function-local static, so zero to begin with) and
// remembers, per device, the largest size it has set; callers may be concurrent.
struct LdsAllowance {
    static constexpr int kDevices = 32;
    std::atomic<size_t> set_[kDevices];
    // true if `bytes` are already allowed on the current device; *dev is that device, or -1 if it
    // cannot be tracked (then the attribute is simply set again on every launch)
    bool covers(size_t bytes, int* dev) const {
        if (hipGetDevice(dev) != hipSuccess || *dev < 0 || *dev >= kDevices) {
            *dev = -1;
            return false;
        }
        return bytes <= set_[*dev].load(std::memory_order_relaxed);
    }
    void record(int dev, size_t bytes) {
        if (dev < 0) return;
        size_t cur = set_[dev].load(std::memory_order_relaxed);
        while (cur < bytes && !set_[dev].compare_exchange_weak(cur, bytes, std::memory_order_relaxed)) {}
    }
};

// Raises the allowance of `fn` on the current device to `bytes` if it is lower.
inline hipError_t allow_lds(LdsAllowance& known, const void* fn, size_t bytes) {
    int dev;
    if (known.covers(bytes, &dev)) return hipSuccess;
    const hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e == hipSuccess) known.record(dev, bytes);
    return e;
}

// ---------------------------------------------------------------- launchers (defined per path)
// Each returns hipSuccess or the launch error.  No allocation, no sync.
hipError_t launch_valu(const MlpArgs& a, const dfk_config_t& c, dfk_dtype_t dtype, hipStream_t st);
hipError_t launch_mfma(const MlpArgs& a, const dfk_config_t& c, hipStream_t st);

// Host-only validity of a configuration for a problem.
bool valu_config_valid(const dfk_config_t& c, int M, int d_model, int d_ff, dfk_dtype_t dtype);
bool mfma_config_valid(const dfk_config_t& c, int M, int d_model, int d_ff, dfk_dtype_t dtype);
int mfma_max_tokens_per_launch(const dfk_config_t& c, int d_model);
// the pair of kernels for up to 64 tokens per launch (dfk_mfma_km.hip; config field kmajor)
hipError_t launch_mfma_km(const MlpArgs& a, const dfk_config_t& c, hipStream_t st);
bool mfma_km_config_valid(const dfk_config_t& c, int M, int d_model, int d_ff, dfk_dtype_t dtype);
bool mfma_km_block_config_valid(const dfk_config_t& c, int M, int d_model, int d_ff, dfk_dtype_t dtype);
int mfma_km_tokens_per_launch();
// the pair whose down kernel takes W_down as [d_model, d_ff] (kmajor = 5)
bool mfma_km_t_config_valid(const dfk_config_t& c, int M, int d_model, int d_ff, dfk_dtype_t dtype);
// both kernels' workgroups in one launch (variant FUSED, kmajor = 4)
hipError_t launch_mfma_km_roles(const MlpArgs& a, const dfk_config_t& c, hipStream_t st);
bool mfma_km_roles_config_valid(const dfk_config_t& c, int M, int d_model, int d_ff, dfk_dtype_t dtype);
// the single launch built on that pair (dfk_mfma_fused.hip; variant FUSED with kmajor = 1)
hipError_t launch_mfma_fused_km(const MlpArgs& a, const dfk_config_t& c, hipStream_t st);
bool mfma_fused_km_config_valid(const dfk_config_t& c, int M, int d_model, int d_ff, dfk_dtype_t dtype);
int mfma_fused_km_tokens_per_launch();
// the pair of kernels for 65..256 tokens per launch (dfk_mfma_big.hip; config field kmajor = 2)
hipError_t launch_mfma_big(const MlpArgs& a, const dfk_config_t& c, hipStream_t st);
bool mfma_big_config_valid(const dfk_config_t& c, int M, int d_model, int d_ff, dfk_dtype_t dtype);
int mfma_big_tokens_per_launch();
// its gate/up kernel with four wavefronts of one token tile each (up to 64 tokens), for the mixed pair (kmajor = 3)
hipError_t launch_big_gateup_64(const MlpArgs& a, const dfk_config_t& c, hipStream_t st);
bool big_gateup_64_fits(const dfk_config_t& c, int d_model, int d_ff);
int valu_max_tokens_per_launch();

// utility kernels
hipError_t launch_zero(void* p, size_t bytes, hipStream_t st);
hipError_t launch_transpose(const void* in, void* out, int rows, int cols, dfk_dtype_t dtype, hipStream_t st);
hipError_t launch_stream_read(const void* src, size_t bytes, void* sink, hipStream_t st);
hipError_t launch_read_gateup_pattern(const void* Wg, const void* Wu, int d_model, int d_ff, int splits, int waves,
                                      void* sink, hipStream_t st);
hipError_t launch_rms_normalize(const void* in, void* out, int M, int d_model, hipStream_t st);
hipError_t launch_rmsnorm_weighted(const void* in, const void* w, void* out, int M, int d_model, float eps, dfk_dtype_t dtype,
                                   hipStream_t st);
hipError_t launch_fill(void* dst, size_t elems, dfk_dtype_t dtype, float scale, unsigned seed,
                       hipStream_t st);

}  // namespace dfk
