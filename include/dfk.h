/*
 * dfk.h - C ABI of the deeply fused SwiGLU MLP library for AMD MI355X (gfx950).
 *
 * The operation (Background section, SwiGLU equations; Method section,
 * two-stage split):
 *
 *     A_2 = (X W_up) (x) SiLU(X W_gate),      Y = A_2 W_down,
 *     SiLU(g) = Sigmoid(g) * g,               (x) = elementwise product,
 *
 * with W_gate, W_up in R^{d_model x d_ff} and W_down in R^{d_ff x d_model}.
 *
 * Storage layouts (fixed by this ABI; the paper gives mathematical shapes only).
 * All tensors are dense, row-major, in DEVICE memory, 16-byte aligned:
 *     X      [M,    d_model]   activations, read-only
 *     W_gate [d_ff, d_model]   transposed mathematical shape (row j = column j of W_gate)
 *     W_up   [d_ff, d_model]   transposed mathematical shape
 *     W_down [d_ff, d_model]   the mathematical shape
 *     Y      [M,    d_model]   output, fully overwritten (never accumulated into)
 * so that every d_ff slice of each weight matrix is one contiguous block.  The entry points with the
 * suffix _wdt take the down projection's weights the other way round instead:
 *     W_down_t [d_model, d_ff]  transposed mathematical shape (row n = column n of W_down)
 * which is how a linear layer stores them ([out, in]), and how W_gate and W_up are stored here.
 * Element type: bfloat16 or IEEE half (inputs and Y; fp32 accumulation; A_2 is
 * rounded to the same 16-bit type on the MFMA path) or, in the fp32 test mode,
 * IEEE fp32 for inputs and Y.  Y must not overlap any input.
 *
 * Ownership and execution: the caller owns every buffer, including the
 * workspace.  No entry point on the call path allocates or frees device
 * memory or synchronises the host; work is enqueued on `stream` (a
 * hipStream_t passed as void*, NULL = the default stream) and the call
 * returns at once.  The workspace holds arrival counters and the fp32
 * accumulator of the atomic reduction (its first 8 MiB + 4 KiB), the fp32
 * partial sums of Y and A_2 (two-kernel variant, and the single launch that holds both
 * kernels' workgroups).  Counters and accumulator
 * must be zero before the first call (dfk_workspace_init) and every call leaves
 * them zero again, so a workspace may be reused by successive calls, of any
 * shape that fits, on ONE stream.  Calls that share a workspace and overlap in
 * time race.
 *
 * Errors: every function returns a dfk_status_t (or a plain value where
 * noted) and never throws or aborts.  All argument errors are detected on the
 * host before any HIP call is made.
 */
#ifndef DFK_H
#define DFK_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    DFK_OK = 0,
    DFK_ERR_INVALID_ARG = -1,        /* null pointer, M < 1, d_model < 1, d_ff < 1, bad enum */
    DFK_ERR_UNSUPPORTED_SHAPE = -2,  /* d_model % 8, d_ff % 8, M > DFK_MAX_M, d_model > 32768, or config not valid for shape */
    DFK_ERR_ALIGNMENT = -3,          /* a device pointer is not 16-byte aligned */
    DFK_ERR_ALIAS = -4,              /* Y overlaps X, W_gate, W_up or W_down */
    DFK_ERR_WORKSPACE = -5,          /* workspace missing or smaller than dfk_workspace_bytes() */
    DFK_ERR_HIP = -6,                /* a HIP call failed; see dfk_last_hip_error() */
    DFK_ERR_IO = -7,                 /* tuning file could not be read / written / parsed */
    DFK_ERR_NOT_FOUND = -8           /* no tuned entry / no such candidate */
} dfk_status_t;

typedef enum { DFK_BF16 = 0, DFK_FP32 = 1, DFK_FP16 = 2 } dfk_dtype_t;   /* FP16 = IEEE binary16 */

/* Fusion depth (Method section; Figure 1 b/c): one launch for the whole block,
 * or two launches cut after A_2. */
typedef enum { DFK_VARIANT_AUTO = 0, DFK_VARIANT_FUSED = 1, DFK_VARIANT_TWO_KERNEL = 2 } dfk_variant_t;

/* How the contractions are computed. */
typedef enum { DFK_PATH_VALU = 0, DFK_PATH_MFMA = 1 } dfk_path_t;

/* How the split-d_ff partial sums of the down projection are combined.
 * DFK_REDUCE_TICKET: partial blocks in the workspace, summed in a fixed order by
 * the last workgroup to arrive at each of two levels of arrival counters;
 * run-to-run bitwise deterministic.
 * DFK_REDUCE_ATOMIC: device-wide fp32 atomic adds into an accumulator in the
 * workspace, drained per 128-column block by the last wavefront to arrive;
 * shorter tail, summation order (hence the last bits) varies from run to run.
 * MFMA path only. */
typedef enum { DFK_REDUCE_TICKET = 0, DFK_REDUCE_ATOMIC = 1 } dfk_reduce_t;

#define DFK_MAX_M 256            /* largest token count one call accepts */

/*
 * One candidate kernel configuration (Method section: tiling / loop-order
 * variants and tile sizes; the scheduler chooses among these).
 *   variant        DFK_VARIANT_FUSED or DFK_VARIANT_TWO_KERNEL
 *   path           DFK_PATH_VALU (any supported shape, all three element types) or
 *                  DFK_PATH_MFMA (bf16, and IEEE half with the kernel families kmajor >= 1;
 *                  shape constraints, see dfk_config_valid)
 *   splits         number of d_ff slices = workgroups of the fused kernel, or of
 *                  the first kernel of the two-kernel variant
 *   waves          wavefronts (64 lanes) per workgroup
 *   depth          software pipeline depth of the weight stream (tiles or loads in flight)
 *   reduce         dfk_reduce_t
 *   k2_splits      two-kernel variant: d_ff splits of the down projection
 *   k2_col_blocks  two-kernel variant: column blocks of the down projection
 *                  (grid of the second kernel = k2_splits * k2_col_blocks)
 *   a2_dtype       two-kernel variant: type A_2 is stored in between the
 *                  kernels: DFK_FP32, or the 16-bit type of the inputs (DFK_BF16 with
 *                  bf16 inputs; with half inputs DFK_FP16, kmajor pair only)
 *   k2_rows_by_wave  two-kernel variant, MFMA path: 0 = in the down projection each
 *                  wavefront owns 128-column blocks of the workgroup's columns;
 *                  1 = the wavefronts share the workgroup's (at most 4) column blocks
 *                  and divide its d_ff rows (meant for few d_ff splits: a short
 *                  cross-workgroup sum whatever the token count)
 *   kmajor         MFMA path, kernel family.
 *                  two-kernel variant:
 *                  1 = the pair of kernels that take up to 64 tokens per launch (the activations
 *                  travel through the same LDS rings as the weight tiles instead of sitting in
 *                  registers; gate/up kernel k-major with all its row tiles accumulating in
 *                  registers); needs k2_rows_by_wave = 0 and d_model a multiple of 128 with at
 *                  least `waves` 128-k chunks (512 and up);
 *                  0 = the first pair (activations in registers, row-tile-major);
 *                  2 = the pair that takes up to 256 tokens per launch (offered beyond 64
 *                  tokens, and at any token count where d_model rules out pair 1): the wavefronts
 *                  share every weight tile through LDS and own a share of the tokens each;
 *                  waves = 4 or 8 (wavefronts of the gate/up kernel; the down kernel always runs
 *                  8), depth = 3 or 4 (buffers of shared tiles), k2_col_blocks = d_model / 128;
 *                  with DFK_REDUCE_TICKET the splits' partial sums are added by a third, small
 *                  launch;
 *                  5 = gate/up kernel of pair 1, then a down kernel that takes W_down as
 *                  [d_model, d_ff] (dfk_swiglu_mlp_wdt only): k2_splits workgroups own a slice of
 *                  d_model each (whole 16-row tiles, at most 8 per workgroup), k2_col_blocks = 1,
 *                  reduce = DFK_REDUCE_TICKET (nothing is reduced across workgroups; the result
 *                  is deterministic), up to 64 tokens per launch.  With path = DFK_PATH_VALU the
 *                  same pair in plain fp32 FMAs (any shape and type; k2_splits = workgroups of
 *                  the down kernel, whose wavefronts own output columns whole);
 *                  3 = gate/up kernel of pair 2 with four wavefronts of one token tile each,
 *                  down kernel of pair 1 (offered for 33..64 tokens; waves = 8, depth = 3 or 4,
 *                  the constraints of both pairs).
 *                  fused variant:
 *                  1 = the single launch built on pair 1's k-major stage one: each workgroup
 *                  keeps A_2 of its d_ff slice in LDS and runs both stages over one tile stream
 *                  (up to 16 tokens per launch, slices of at most 64 rows, waves = 4 or 8,
 *                  d_model a multiple of 128 with at least `waves` 128-k chunks; bf16 and half);
 *                  4 = both kernels of pair 1 in one launch: the grid holds the gate/up kernel's
 *                  `splits` workgroups followed by the down kernel's k2_splits * k2_col_blocks;
 *                  a down workgroup requests its first W_down tiles, then waits (a bounded
 *                  number of polls) until the gate/up workgroups of its d_ff rows have
 *                  published A_2, which crosses through device memory as between two kernels.
 *                  Up to 64 tokens per launch; waves = 8; otherwise the constraints of pair 1,
 *                  whose k2_splits, k2_col_blocks and reduce fields it uses.  The bound of the wait is
 *                  about two million polls (seconds); a workgroup whose wait runs out turns its
 *                  share of Y into NaN.  (Tests force that path from the host with the environment
 *                  variable DFK_DEBUG_SPIN_LIMIT = number of polls; leave it unset otherwise.);
 *                  0 = the first single-launch kernel (bf16 only).
 */
typedef struct dfk_config_t {
    int variant;
    int path;
    int splits;
    int waves;
    int depth;
    int reduce;
    int k2_splits;
    int k2_col_blocks;
    int a2_dtype;
    int k2_rows_by_wave;
    int kmajor;
} dfk_config_t;

/* ---------------------------------------------------------------- the block */

/*
 * Y = (SiLU(X W_gate) (x) (X W_up)) W_down in bfloat16 with fp32 accumulation;
 * the scheduler picks variant and tile configuration for (M, d_model, d_ff)
 * (tuned entry if dfk_tune / dfk_load_tuning / dfk_set_choice provided one,
 * else a built-in heuristic).  Uses the workspace registered with
 * dfk_set_workspace (DFK_ERR_WORKSPACE if none or too small).
 * All pointers are device pointers.
 */
dfk_status_t dfk_swiglu_mlp(const void* X, const void* W_gate, const void* W_up,
                            const void* W_down, void* Y,
                            int M, int d_model, int d_ff, void* stream);

/* Same, forcing the single-launch deeply fused kernel (Figure 1c). */
dfk_status_t dfk_swiglu_mlp_fused(const void* X, const void* W_gate, const void* W_up,
                                  const void* W_down, void* Y,
                                  int M, int d_model, int d_ff, void* stream);

/* Same, forcing the two-kernel layout cut after A_2 (Figure 1b; Method, the
 * two-stage split). A_2 lives in the workspace between the two launches. */
dfk_status_t dfk_swiglu_mlp_unfused(const void* X, const void* W_gate, const void* W_up,
                                    const void* W_down, void* Y,
                                    int M, int d_model, int d_ff, void* stream);

/*
 * Fully explicit form.  dtype selects bf16, IEEE half (the precision of the paper's
 * Experiments section) or the fp32 test mode (all five tensors in that type).  cfg == NULL means "scheduler's choice"; otherwise
 * cfg must satisfy dfk_config_valid for the shape.  workspace is a device
 * buffer of at least dfk_workspace_bytes(M, d_model, d_ff) bytes, 256-byte
 * aligned, initialised once with dfk_workspace_init.
 */
dfk_status_t dfk_swiglu_mlp_ex(const void* X, const void* W_gate, const void* W_up,
                               const void* W_down, void* Y,
                               int M, int d_model, int d_ff, dfk_dtype_t dtype,
                               const dfk_config_t* cfg,
                               void* workspace, size_t workspace_bytes, void* stream);

/*
 * dfk_swiglu_mlp_ex with the down projection's weights given as W_down_t [d_model, d_ff], row n = column n of
 * the paper's W_down (Background, SwiGLU equations: Y = A_2 W_down): the [out, in] layout a linear layer's
 * weights are stored in, and the layout W_gate and W_up already have here.  Same result.  In this layout a
 * workgroup of the down kernel owns a slice of d_model over all of d_ff, so nothing is summed across workgroups
 * (config field kmajor = 5: on the MFMA path for the 16-bit types with d_model a multiple of 128 and d_ff a
 * multiple of 128 with at least `waves` 128-k chunks each; on the VALU path for every supported shape and type).
 * cfg == NULL: the scheduler's choice for this layout (dfk_get_choice_wdt); else cfg must be a kmajor = 5
 * configuration (the other entry points reject those, and this one rejects the others, with
 * DFK_ERR_INVALID_ARG: a configuration belongs to one layout).
 */
dfk_status_t dfk_swiglu_mlp_wdt(const void* X, const void* W_gate, const void* W_up,
                                const void* W_down_t, void* Y,
                                int M, int d_model, int d_ff, dfk_dtype_t dtype,
                                const dfk_config_t* cfg,
                                void* workspace, size_t workspace_bytes, void* stream);

/* W_down_t [d_model, d_ff] from W_down [d_ff, d_model] (device buffers that do not overlap, 16-byte aligned;
 * any of the three element types), for callers that hold the other layout.  Asynchronous on `stream`. */
dfk_status_t dfk_transpose_w_down(const void* W_down, void* W_down_t, int d_model, int d_ff,
                                  dfk_dtype_t dtype, void* stream);

/*
 * dfk_swiglu_mlp_ex for callers that cannot allocate device memory and therefore have no workspace
 * to pass: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * The same kernels run with their scratch (arrival counters, fp32 accumulator, partial sums, A_2)
 * in an array that is part of the library's code object: 48 MiB per device, held from the moment
 * the library is loaded on that device until the process ends.  No call allocates or frees anything.
 * Arguments as dfk_swiglu_mlp_ex without the workspace; cfg == NULL takes the scheduler's choice, or,
 * if its partial sums do not fit the array, the first candidate that fits.
 * Limits: M * d_ff * 4 (A_2) at most 16 MiB, and the partial-sum blocks of the configuration within
 * what is left (about 21 MiB; the atomic reduction needs none).  Beyond them: DFK_ERR_WORKSPACE,
 * before any launch.  The first call on a device resolves the array's address and enqueues a fill
 * kernel that zeroes its counters; make that call outside a graph capture.  All calls on one device
 * share the array: calls that overlap in time on one device race (one stream, or ordered streams).
 */
dfk_status_t dfk_swiglu_mlp_static(const void* X, const void* W_gate, const void* W_up,
                                   const void* W_down, void* Y,
                                   int M, int d_model, int d_ff, dfk_dtype_t dtype,
                                   const dfk_config_t* cfg, void* stream);

/*
 * The block together with its two neighbours in a pre-norm decoder layer.  This goes one
 * step beyond the paper's operator, which starts at X and ends at Y (Method); in the
 * Llama-style models of the Experiments section an RMS normalisation produces X and a
 * residual add consumes Y, each a separate pass over [M, d_model] otherwise:
 *
 *     H_out = H + SwiGLU_MLP( RMSNorm(H; norm_weight, eps) )
 *     RMSNorm(H; w, eps)[m,k] = H[m,k] * w[k] / sqrt( mean_k H[m,k]^2 + eps )
 *
 * in the same two launches as the plain block: the gate/up kernel scales its X operand by
 * norm_weight, sums the squares of the H values it streams anyway and applies the
 * per-token factor to its fp32 sums; the down kernel adds H at its final store.
 *
 * H, H_out [M, d_model], norm_weight [d_model], weights as above; dtype DFK_BF16 or
 * DFK_FP16 (DFK_FP32: DFK_ERR_UNSUPPORTED_SHAPE).  H_out may be H itself (in place); any
 * other overlap is DFK_ERR_ALIAS.  eps >= 0; a row of zeros with eps == 0 yields NaN, as
 * the definition does.  The product H[m,k] * w[k] is rounded once to dtype before the
 * contraction (with half inputs it must stay finite in half precision).
 * Runs on the kernel pairs that take the activations through LDS: cfg->kmajor == 1 (up to 64
 * tokens per launch, everything folded into the two launches as described; where d_model is
 * so wide that the normalisation weight does not fit that kernel's LDS beside its rings, the
 * normalisation becomes one small launch of its own, as below), or
 * cfg->kmajor == 2 (up to 256 tokens; there the normalisation is one small launch of its own
 * ahead of the pair, into the workspace: that pair is paced by its arithmetic, and scaling X
 * inside every workgroup measured slower; the residual add stays in the final store).
 * cfg == NULL picks the scheduler's choice among those.  Any other configuration, and shapes
 * those pairs do not cover, give DFK_ERR_UNSUPPORTED_SHAPE.  Workspace as for dfk_swiglu_mlp_ex.
 */
dfk_status_t dfk_mlp_block(const void* H, const void* norm_weight, float eps,
                           const void* W_gate, const void* W_up, const void* W_down,
                           void* H_out, int M, int d_model, int d_ff, dfk_dtype_t dtype,
                           const dfk_config_t* cfg,
                           void* workspace, size_t workspace_bytes, void* stream);

/* The same with the down projection's weights given as W_down_t [d_model, d_ff] (see dfk_swiglu_mlp_wdt):
 * cfg == NULL or a kmajor = 5 configuration; the normalisation is folded into the gate/up kernel as with
 * kmajor = 1, the residual is added where the down kernel stores Y. */
dfk_status_t dfk_mlp_block_wdt(const void* H, const void* norm_weight, float eps,
                               const void* W_gate, const void* W_up, const void* W_down_t,
                               void* H_out, int M, int d_model, int d_ff, dfk_dtype_t dtype,
                               const dfk_config_t* cfg,
                               void* workspace, size_t workspace_bytes, void* stream);

/* Host-only argument check: exactly the validation the calls above perform,
 * with no HIP call.  cfg may be NULL.  workspace may be NULL only if
 * workspace_bytes is 0, in which case the workspace checks are skipped. */
dfk_status_t dfk_check_args(const void* X, const void* W_gate, const void* W_up,
                            const void* W_down, const void* Y,
                            int M, int d_model, int d_ff, dfk_dtype_t dtype,
                            const dfk_config_t* cfg,
                            const void* workspace, size_t workspace_bytes);

/* ---------------------------------------------------------------- workspace */

/* Upper bound, over every configuration the library can pick, of the workspace
 * a call with M <= M_max needs.  Returns 0 for invalid arguments and for shapes no
 * call accepts (the conditions of DFK_ERR_UNSUPPORTED_SHAPE). */
size_t dfk_workspace_bytes(int M_max, int d_model, int d_ff);

/* Enqueue the zero-initialisation of a workspace (a fill kernel; capturable). */
dfk_status_t dfk_workspace_init(void* workspace, size_t workspace_bytes, void* stream);

/* Register the workspace the non-_ex calls use (per process; the pointer is
 * kept, not copied).  The caller must have initialised it. NULL unregisters. */
dfk_status_t dfk_set_workspace(void* workspace, size_t workspace_bytes);

/* ---------------------------------------------------------------- scheduler
 * Profile-driven kernel scheduler (Method, last paragraph; Experiments: the
 * scheduler benchmarks the candidate kernels before inference on the target
 * hardware and selects the fastest for the model shape and batch).  After
 * tuning, a call costs one table lookup. */

/* Number of candidate configurations for this problem, and the i-th one. */
int dfk_num_candidates(int M, int d_model, int d_ff, dfk_dtype_t dtype);
dfk_status_t dfk_get_candidate(int M, int d_model, int d_ff, dfk_dtype_t dtype, int i,
                               dfk_config_t* out);

/* 1 if cfg can run this problem, else 0. Host-only. */
int dfk_config_valid(const dfk_config_t* cfg, int M, int d_model, int d_ff, dfk_dtype_t dtype);

/* Bytes of device scratch dfk_tune needs: `sets` rotating copies of the three
 * weight matrices (so timed launches stream from HBM, not from cache) plus X,
 * Y and a workspace for the largest M in the list.  0 for invalid arguments and
 * unsupported shapes. */
size_t dfk_tune_scratch_bytes(int M_max, int d_model, int d_ff, dfk_dtype_t dtype, int sets);

/*
 * Time every candidate for each M in M_list on the current device and record
 * the fastest, and beside it the fastest of each variant (what dfk_swiglu_mlp_fused
 * and dfk_swiglu_mlp_unfused, which ask for a variant, then use).  scratch is caller-owned device memory of at least
 * dfk_tune_scratch_bytes(max M, ...) bytes; its previous contents are
 * overwritten with synthetic values.  iters timed launches per candidate
 * (after 2 warm-ups), rotating over `sets` weight copies.  Synchronises
 * the stream (this is the pre-inference step, not the call path).
 */
dfk_status_t dfk_tune(const int* M_list, int nM, int d_model, int d_ff, dfk_dtype_t dtype,
                      void* scratch, size_t scratch_bytes, int sets, int iters, void* stream);

/* dfk_tune leaves out a candidate whose timing fails (a launch error, say) and goes on with the
 * others; it fails only where every candidate of a token count failed, with that status.  This
 * returns how many candidates the last dfk_tune call on the calling thread left out, and the status
 * of the last one in *last_status_out (may be NULL; DFK_OK if none).  Host-only. */
int dfk_tune_skipped(dfk_status_t* last_status_out);

/* Time one configuration the same way; writes mean microseconds per call. */
dfk_status_t dfk_time_config(const dfk_config_t* cfg, int M, int d_model, int d_ff,
                             dfk_dtype_t dtype, void* scratch, size_t scratch_bytes,
                             int sets, int iters, void* stream, double* usec_out);

/* Time the launches of one configuration separately, same protocol: `iters` launches
 * of the first kernel back to back between two HIP events on `stream`, then the same
 * for the second.  usec_out[0] = the fused kernel, or the gate/up kernel of the
 * two-kernel variant; usec_out[1] = its down-projection kernel (0 for the fused
 * variant; with kmajor = 2 and DFK_REDUCE_TICKET it includes the small launch that adds the
 * partial sums).  M must fit one launch of the configuration (16, 32, 64 or 256 tokens on the
 * MFMA path, 8 on the VALU path), else DFK_ERR_UNSUPPORTED_SHAPE; iters <= 1024. */
dfk_status_t dfk_time_kernels(const dfk_config_t* cfg, int M, int d_model, int d_ff,
                              dfk_dtype_t dtype, void* scratch, size_t scratch_bytes,
                              int sets, int iters, void* stream, double* usec_out);

/* The configuration a call would use now (tuned entry, else heuristic).
 * *tuned_out (may be NULL) is set to 1 if it came from the table. */
dfk_status_t dfk_get_choice(int M, int d_model, int d_ff, dfk_dtype_t dtype,
                            dfk_config_t* out, int* tuned_out);

/* The same three queries for W_down given as [d_model, d_ff] (dfk_swiglu_mlp_wdt): its candidates, and the
 * configuration a call would use now.  dfk_tune times these
 * candidates too and keeps the fastest beside the others. */
int dfk_num_candidates_wdt(int M, int d_model, int d_ff, dfk_dtype_t dtype);
dfk_status_t dfk_get_candidate_wdt(int M, int d_model, int d_ff, dfk_dtype_t dtype, int i, dfk_config_t* out);
dfk_status_t dfk_get_choice_wdt(int M, int d_model, int d_ff, dfk_dtype_t dtype,
                                dfk_config_t* out, int* tuned_out);

/* Enter / overwrite a table entry by hand (usec <= 0 means unknown): cfg becomes the choice for the
 * problem and the entry of its variant. */
dfk_status_t dfk_set_choice(int M, int d_model, int d_ff, dfk_dtype_t dtype,
                            const dfk_config_t* cfg, double usec);

/* Forget all tuned entries. */
void dfk_clear_tuning(void);

/* Persist / reload the table (plain text, one entry per line; where a problem has entries of both
 * variants the chosen one is written last, and a loader takes a problem's last line as its choice). */
dfk_status_t dfk_save_tuning(const char* path);
dfk_status_t dfk_load_tuning(const char* path);

/* ---------------------------------------------------------------- measurement */

/* Read-only streaming kernel over `bytes` of device memory (128-bit loads whose
 * XOR fold is compared with a magic value; sink, 8 bytes, is written only on a
 * match, i.e. practically never): measures the achievable HBM read ceiling that
 * the block's bandwidth is compared with.  bytes must be a multiple of 16. */
dfk_status_t dfk_stream_read(const void* src, size_t bytes, void* sink, void* stream);

/* Read-only kernel that fetches W_gate and W_up [d_ff, d_model] (16-bit elements) exactly as the
 * gate/up kernel of the two-kernel variant for up to 64 tokens does (Method: the first stage is
 * where the weights dominate): `splits` workgroups, one d_ff slice each, `waves` (4 or 8)
 * wavefronts that divide every row's k range, 4 rows x 256 bytes per load instruction, the same
 * tile order, 16 instructions in flight per wavefront; and nothing else (no X, no MFMA, no LDS,
 * no stores).  Its duration is what that kernel's memory pattern costs on its own.
 * d_model must be a multiple of 128 * waves, d_ff of 8, 1 <= splits <= min(d_ff / 8, 65535);
 * sink as for dfk_stream_read.  Errors as for the other calls (arguments are checked on the host). */
dfk_status_t dfk_read_gateup_pattern(const void* W_gate, const void* W_up, int d_model, int d_ff,
                                     int splits, int waves, void* sink, void* stream);

/* Fill a device buffer with synthetic bf16 (or fp32) values in (-scale, scale),
 * a cheap hash of the element index and seed.  Used by dfk_tune and by benchmarks. */
dfk_status_t dfk_fill_synthetic(void* dst, size_t elems, dfk_dtype_t dtype, float scale,
                                unsigned seed, void* stream);

/* out[m, :] = in[m, :] / rms(in[m, :]) for bf16 [M, d_model] (fp32 arithmetic, no weight; in == out
 * allowed).  Not part of the block: benchmarks and tests chain random layers with it, which would
 * otherwise shrink the activations to zero within a few layers.  M <= 65535. */
dfk_status_t dfk_rms_normalize(const void* in, void* out, int M, int d_model, void* stream);

/* Optional in-kernel timeline for profiling the MFMA kernels: while a device buffer
 * of at least 64 bytes per workgroup of the launch is registered, each workgroup
 * writes up to 8 wall-clock stamps (100 MHz counter): [0] start, [1] first tile
 * landed, [2] stage one streamed, [3] A_2 ready, [4] stage two streamed,
 * [5] partial published, [6] end of first reduction level (or exit), [7] Y written by the last group.  NULL unregisters.  Off by default. */
dfk_status_t dfk_set_trace_buffer(void* buffer, size_t bytes);

/* ---------------------------------------------------------------- misc */

const char* dfk_status_string(dfk_status_t s);
int dfk_last_hip_error(void);          /* hipError_t of the last DFK_ERR_HIP on this thread */
const char* dfk_version(void);

#ifdef __cplusplus
}
#endif
#endif /* DFK_H */
