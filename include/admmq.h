/*
 * admmq.h - C ABI of the MI355X (gfx950) ADMM-Q layer solver.
 *
 * One linear layer Y = X W with X [N][n] calibration activations and dense weights W0 [n][p]
 * (n input channels, p output channels; paper Sec. 3.1).  The library accumulates the Hessian
 * H = X^T X, runs the diagonally scaled ADMM loop of Alg. 1 (eqs. 7-10) under the geometric
 * penalty schedule rho_t = rho0 * gamma^t (Sec. 3.6), and refines the result with the pair-swap
 * local search of Sec. 3.5.  Results are integer codes with per-group scales and real-valued
 * zero offsets:  Wq[i][j] = zeros[i/g][j] + codes[i][j] * scales[i/g][j].
 *
 * Conventions
 *   - Every array argument marked "device" is a pointer to GPU memory owned by the caller, on the
 *     context's device; "host" marks ordinary host memory.  All matrices are row-major.
 *   - The library never hands out memory of its own.  Scratch comes from an arena the context grows
 *     with hipMalloc on demand, or from caller memory given to admmq_set_workspace.
 *   - Work is enqueued on the context's stream; calls that return host values (stats, objectives)
 *     synchronise that stream before returning, the others return after enqueueing.
 *   - Errors are return codes only.  Arguments are validated on the host before any device work,
 *     so a failed validation leaves all outputs untouched and needs no GPU.
 *   - One context may be used by one host thread at a time.
 */
#ifndef ADMMQ_H
#define ADMMQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct admmq_ctx admmq_ctx;

typedef enum {
    ADMMQ_OK = 0,
    ADMMQ_ERR_NULL = 1,        /* a required pointer is NULL */
    ADMMQ_ERR_SHAPE = 2,       /* n, p, rows, leading dimension or group size do not fit */
    ADMMQ_ERR_PARAM = 3,       /* bits, T, rho0, gamma, damp ... out of range */
    ADMMQ_ERR_NOT_FINITE = 4,  /* H or W0 holds a NaN or an infinity */
    ADMMQ_ERR_ZERO_DIAG = 5,   /* a diagonal entry of the damped Hessian is <= 0 (dead channel) */
    ADMMQ_ERR_WORKSPACE = 6,   /* caller workspace too small / allocation failed */
    ADMMQ_ERR_STATE = 7,       /* step call without the factorisation it needs */
    ADMMQ_ERR_DEVICE = 8       /* a HIP call failed */
} admmq_status;

typedef enum { ADMMQ_F32 = 0, ADMMQ_BF16 = 1 } admmq_dtype;

/* ---- context ------------------------------------------------------------------------------ */

/* Creates a context on `device`.  `hip_stream` is a borrowed hipStream_t (NULL = the default
 * stream); the caller keeps it alive for the context's lifetime.  device = -1 gives a context
 * without a GPU: every call still validates its arguments and then returns ADMMQ_ERR_DEVICE. */
admmq_status admmq_create(admmq_ctx **out, int device, void *hip_stream);
void admmq_destroy(admmq_ctx *ctx);
const char *admmq_status_string(admmq_status s);

/* Bytes of scratch admmq_quantize_layer and admmq_quantize_layer_format need for an n x p layer, for any
 * group size of 3 rows or more, up to 5 local-search rounds of (n+1)/2 batches of 64 pairs (pure host function). */
size_t admmq_workspace_bytes(int64_t n, int64_t p, int32_t T);
/* Optional: use caller memory (device, 256-byte aligned) as the scratch arena from now on. */
admmq_status admmq_set_workspace(admmq_ctx *ctx, void *dev_ptr, size_t bytes);

/* Opt-in, per context, off by default (on = 1 / 0): the two products of every W-update (eq. 7) whose output is whole
 * 256 x 256 tiles (n and the column count multiples of 256; at least 200 tiles, or 25 and more with the contraction
 * cut into up to eight slices of 512 rows or more) run on the fp16 matrix cores.
 * Each fp32 operand is scaled by a power of two and split into an fp16 pair hi + lo (22 bits); the product is
 * hiA hiB + hiA loB + loA hiB, every term exact, accumulated in fp32.  Against the fp32 product this drops the
 * operands' last two bits and the lo-lo term (about 3e-7 of a term, an order of magnitude below the fp32
 * accumulation error both share): the W-update stays within the 1e-5 relative Frobenius bar, but results are not
 * bit-identical to the default.  Applies to admmq_quantize_layer, admmq_quantize_layer_format,
 * admmq_quantize_layers and admmq_w_update; other shapes keep the fp32 products.  Needs
 * admmq_fast_products_bytes(n, p) more scratch than admmq_workspace_bytes (0 when the shape does not qualify). */
admmq_status admmq_set_fast_products(admmq_ctx *ctx, int32_t on);
size_t admmq_fast_products_bytes(int64_t n, int64_t p);

/* Measurement aid (no counterpart in the paper): copies `bytes` (a multiple of 16; both pointers device, 16-byte
 * aligned, not overlapping) with a plain streaming kernel on the context's stream.  bench.py times it on 1 GiB as
 * the bandwidth a kernel of this library reaches on the box at hand, beside the published HBM peak, and the
 * hardware-counter runs use it to calibrate FETCH_SIZE / WRITE_SIZE. */
admmq_status admmq_stream_copy(admmq_ctx *ctx, void *dst, const void *src, size_t bytes);

/* ---- Hessian accumulation (Sec. 3.1: H = X^T X) ------------------------------------------- */

/* H [n][n] (device fp32, caller zero-initialises before the first chunk) += X^T X for a chunk
 * X [rows][ldx] (device; fp32 or bf16 bit patterns), ldx >= n.  Both triangles of H are kept
 * up to date.  *n_samples (host, may be NULL) += rows.  Every product is exact and is added in
 * fp32: bf16 inputs with n a multiple of 256 and 16-byte aligned rows are contracted on the bf16 matrix
 * cores (fp32 accumulation), any other input on the fp32 ones (bf16 widened on the way in).  Scratch: one
 * [n][n] fp32 partial sum per token slice (the library picks the number of slices; in a caller's workspace
 * as many as fit, at least one, else ADMMQ_ERR_WORKSPACE with H untouched). */
admmq_status admmq_accumulate_hessian(admmq_ctx *ctx, float *H, int64_t n, const void *X,
                                      admmq_dtype xdt, int64_t rows, int64_t ldx, uint64_t *n_samples);

/* ---- whole layer (Alg. 1) ----------------------------------------------------------------- */

typedef struct {
    int32_t T;             /* ADMM iterations, run exactly unless quiet_stop is set (paper: 300) */
    double rho0;           /* initial penalty (paper: 0.1)                                   */
    double gamma;          /* growth factor > 1, or exactly 1 for a fixed penalty (paper: 1.1).  The penalties reach
                              the kernels in fp32: rho0 >= 1e-30 and rho0 * gamma^T <= 1e30, else ADMMQ_ERR_PARAM
                              (the paper's schedule ends at 0.1 * 1.1^300 = 2.6e11) */
    double damp;           /* lambda = damp * Tr(H)/n added to the diagonal (paper App. D: 0.01) */
    int32_t precondition;  /* 1 = diagonal scaling Sigma = Diag(H')^{-1/2} (Sec. 3.2); 0 = Sigma = I */
    int32_t ls_rounds;     /* local-search rounds, 0 = none (paper: at most 5)                */
    int32_t ls_batches;    /* batches per round, 0 = ceil(n/2)                                */
    int32_t ls_pairs;      /* row pairs per batch, 0 = 64                                     */
    int32_t refresh_iter;  /* iteration at which one grid refresh is tried (App. B), -1 = never */
    int32_t symmetric;     /* 1 = symmetric grid: range [-a, a], a = max|w| of the group (Table 1 setting) */
    int32_t clip_points;   /* MSE clipping search (Sec. 3.4, App. D: 100), 0 = plain min/max fit       */
    double clip_shrink;    /* largest shrink of the range searched (App. D: 0.8)                       */
    int32_t reuse_factor;  /* 1 = H, damp and precondition are those of the factorisation the context
                              already holds (admmq_factorize or an earlier layer): skip Alg. 1 lines 1-3.
                              Matrices that see the same activations (q/k/v, gate/up) share one Hessian.
                              The library checks the address of H, n, damp and precondition, not the contents
                              of H: a Hessian accumulated further in place since it was factorised must be
                              passed with reuse_factor = 0. */
    uint64_t seed;         /* seed of the pair sampler                                        */
    int32_t quiet_stop;    /* 0 = run exactly T iterations (Alg. 1).  K > 0 (not in the paper's listing): stop
                              after the first iteration at which the codes have been unchanged for K iterations
                              in a row - Thm. 1 (Sec. 3.6) has the discrete iterates converge, so on the finite
                              grid they are constant from some iteration on.  Costs one scalar read-back (a
                              stream synchronisation) per iteration; uniform grids only.                   */
} admmq_schedule;

typedef struct {            /* host struct, filled when the pointer is not NULL */
    float ms_total, ms_setup, ms_factor, ms_admm, ms_local_search;
    double j_damp;          /* Tr(E^T H' E), E = Wq - W0, after ADMM + local search (eq. 2 x 2) */
    double j_damp_admm;     /* same, before local search */
    double j_damp_rtn;      /* same, for round-to-nearest on the same grid */
    double lambda;          /* the damping added to the diagonal */
    int32_t iters_done;     /* iterations run: T, or fewer when quiet_stop ended the loop */
    int32_t ls_moves;       /* applied row pairs */
    float *primal_res;      /* optional host array [T]: ||W - D||_F per iteration, or NULL */
    int64_t *code_flips;    /* optional host array [T]: codes changed per iteration, or NULL */
    /* in: non-zero = bracket every launch of the kernels below with HIP events on the context's
     * stream; out: summed device time (ms) and launch counts inside the ADMM loop / local search */
    int32_t profile;
    int32_t n_gemm, n_tridiag, n_project, n_ls_apply;
    float ms_gemm;          /* the two n x n x p products of each W-update (eq. 7)            */
    float ms_tridiag;       /* the solve with the middle factor between them (either form)    */
    float ms_project;       /* fused projection + dual + residual pass (eqs. 8-10, 9)         */
    float ms_ls_apply;      /* rank-2 gradient correction passes of the local search          */
    int32_t refresh_accepted;          /* 1 if the grid refresh was tried and accepted (eq. 12)  */
    double refresh_err_old, refresh_err_new;   /* the two sides of eq. 12 at the attempt        */
    double j_recon;         /* Tr(E^T H E) = ||X (Wq - W0)||_F^2 of the final result: j_damp without the damping term */
    /* second products of eq. 7 that carried eqs. 8-10 as their epilogue (the iterate W stays in registers; taken
     * where the product's tiles are whole and no codes are wanted from the iteration); not part of n_gemm / ms_gemm,
     * and such iterations launch no projection pass */
    int32_t n_gemm_project;
    float ms_gemm_project;
    /* in: non-zero = do not evaluate the objectives (j_damp, j_damp_admm, j_damp_rtn, j_recon are left 0).  They are
     * not part of Alg. 1: each costs one n x n x p product, inside ms_total (j_damp_rtn also inside ms_setup) */
    int32_t skip_objectives;
} admmq_stats;

/* H: raw X^T X (device fp32 [n][n], undamped, read only).  W0: device fp32 [n][ldw], ldw >= p.
 * bits in [2,8].  group_size = 0 means one grid per output column, otherwise it must divide n and
 * a group is group_size consecutive input channels inside one column.
 * Outputs (device): codes u8 [n][p]; scales, zeros fp32 [n/g][p].  The grid is the min/max grid
 * of W0 (Sec. 3.4, no clipping) with zeros = group minimum (the real offset z0 of eq. 10). */
admmq_status admmq_quantize_layer(admmq_ctx *ctx, const float *H, const float *W0, int64_t n,
                                  int64_t p, int64_t ldw, int32_t bits, int32_t group_size,
                                  const admmq_schedule *sched, uint8_t *codes, float *scales,
                                  float *zeros, admmq_stats *stats);

/* ---- several matrices on one Hessian (Sec. 3.5: the objective separates over output columns) -- */

/* One matrix of a group that sees the same activations (q/k/v, gate/up): its own width, bit width,
 * group size and outputs.  All pointers are device memory; layouts as in admmq_quantize_layer. */
typedef struct {
    const float *W0;        /* [n][ldw], read only                                             */
    int64_t p, ldw;         /* ldw >= p                                                        */
    int32_t bits;           /* [2,8]                                                           */
    int32_t group_size;     /* 0 = one grid per column, else divides n                         */
    uint8_t *codes;         /* out [n][p]                                                      */
    float *scales, *zeros;  /* out [n/g][p]                                                    */
} admmq_layer;

/* Runs Alg. 1 once for `count` matrices (1..64) that share the Hessian H [n][n]: one damping, one scaling and one
 * factorisation (lines 1-3), then every W-update (eq. 7) as one pair of products over the concatenated columns
 * [W0_1 | W0_2 | ...], and projection, dual update and local search matrix by matrix on each one's own grid.
 * Columns never interact in eqs. 7-11, so every matrix receives exactly what admmq_quantize_layer would give it
 * alone with the same schedule (the same codes when the local search is off or the seeds agree).
 * `layers` is a host array; outputs of different matrices must not overlap.  sched->quiet_stop ends the loop once
 * no matrix has changed a code for that many iterations.  sched->refresh_iter must be -1
 * (the refresh decision of eq. 12 is taken per matrix, which a shared iteration cannot follow) ->
 * ADMMQ_ERR_PARAM otherwise.  The scratch needed is admmq_workspace_bytes(n, sum of p, T).
 * The local searches of up to four matrices run side by side on streams of the library's own (default priority,
 * created on first use, ordered after the context's stream) driven by short-lived host threads; the call returns
 * after all of them have finished.
 * stats: NULL or a host array [count]; objectives, moves and residual arrays are per matrix, the timing and
 * profile fields describe the whole call and are repeated in every entry (profile is read from stats[0];
 * ms_ls_apply / n_ls_apply are collected only when count is 1; code_flips, when given, is filled with -1). */
admmq_status admmq_quantize_layers(admmq_ctx *ctx, const float *H, int64_t n, const admmq_layer *layers,
                                   int32_t count, const admmq_schedule *sched, admmq_stats *stats);

/* ---- local search alone (Sec. 3.5, eq. 11) ------------------------------------------------ */

typedef struct {
    int32_t rounds, batches_per_round, pairs_per_batch;   /* 0 = defaults 5, ceil(n/2), 64 */
    double damp;
    uint64_t seed;
} admmq_ls_params;

/* Refines `codes` in place on the fixed grid (scales, zeros) against the damped Hessian
 * H' = H + damp*Tr(H)/n I.  Usable on any codes (ADMM output or round-to-nearest).
 * explicit_pairs (host int32 [rounds*batches*pairs][2], may be NULL) replaces the sampler.
 * moves_out / drop_out (host, may be NULL): applied pairs and the summed objective decrease. */
admmq_status admmq_local_search(admmq_ctx *ctx, const float *H, const float *W0, int64_t n, int64_t p,
                                int64_t ldw, int32_t bits, int32_t group_size, const float *scales,
                                const float *zeros, uint8_t *codes, const admmq_ls_params *prm,
                                const int32_t *explicit_pairs, int32_t *moves_out, double *drop_out);

/* Diagnostic.  The search runs each group of 16 batches as one launch whose blocks hand their partial sums to one
 * another through memory, with every wait bounded; a group that gives up a wait is left unapplied, and it and
 * everything after it is redone with one launch per batch (same result, bit for bit).  Returns how many groups of
 * the last local search on this context (stand-alone or inside a layer call) went that way; 0 is the normal case.
 * Environment: ADMMQ_LS_PERSISTENT=0 turns the grouped form off; ADMMQ_LS_SPIN_TICKS sets the bound of a wait in
 * ticks of the device's wall clock (default 20 ms; a negative value makes every block give up at once). */
int32_t admmq_ls_fallback_count(const admmq_ctx *ctx);

/* The pair sampler of the local search, on the host: SplitMix64 (Steele, Lea, Flood 2014) keyed by
 * (seed, round, batch, slot); writes i1 != i2 in [0, n). */
void admmq_sample_pair(uint64_t seed, int32_t round, int32_t batch, int32_t slot, int64_t n,
                       int32_t *i1, int32_t *i2);

/* ---- single steps, exposed so that each can be checked on identical inputs ---------------- */

/* Grid fit (Sec. 3.4): per column and group, scales = (max-min)/(2^bits-1), zeros = min.
 * A group with max == min gets scale 0 by that formula: all its codes stay 0. */
admmq_status admmq_grid_init(admmq_ctx *ctx, const float *W0, int64_t n, int64_t p, int64_t ldw,
                             int32_t bits, int32_t group_size, float *scales, float *zeros);

/* Grid fit with the options of Sec. 3.4 / App. D.  symmetric: the range of a group becomes [-a, a] with
 * a = max|w|.  clip_points > 0: MSE search over the ranges r_i*(min, max), r_i = 1 - i/clip_points for
 * i < floor(clip_shrink*clip_points); the candidate with the smallest squared error on the group's weights
 * wins (the widest on ties).  With symmetric = 0 and clip_points = 0 this is admmq_grid_init. */
admmq_status admmq_grid_fit(admmq_ctx *ctx, const float *W0, int64_t n, int64_t p, int64_t ldw, int32_t bits,
                            int32_t group_size, int32_t symmetric, int32_t clip_points, double clip_shrink,
                            float *scales, float *zeros);

/* Alg. 1 lines 1-3: damp, scale and factorise H once; the result stays in the context and serves
 * every rho.  d_out (device fp32 [n], may be NULL) receives d_i = sqrt(H'_ii) = 1/Sigma_ii.
 * The factorisation is an orthogonal similarity Hs = Q M Q^T in fp64 (Householder reflectors) with M tridiagonal for
 * n < 4096 and a band matrix of half-bandwidth 16 from there on: (Hs + rho I)^{-1} = Q (M + rho I)^{-1} Q^T for any
 * rho, which plays the part of the eigendecomposition of Sec. 3.3.  The environment variable ADMMQ_FACTOR
 * (tridiag / band, read at every call) forces one form. */
admmq_status admmq_factorize(admmq_ctx *ctx, const float *H, int64_t n, double damp,
                             int32_t precondition, float *d_out, double *lambda_out);

/* Eq. 7 with the kept factorisation: W = (Hs + rho I)^{-1}(Hs Ws + rho D - V).
 * Ws, D, V, W_out: device fp32 [n][p] contiguous, in the scaled space. */
admmq_status admmq_w_update(admmq_ctx *ctx, const float *Ws, const float *D, const float *V,
                            int64_t n, int64_t p, double rho, float *W_out);

/* Eqs. 8-10 and 9 fused, one streaming pass: target W + V/rho, project Sigma(.) on the grid,
 * D = Sigma^{-1}(z0 + k*delta), V += rho (W - D), B_out = D - V_new / rho_next.
 * V is updated in place.  codes (u8, may be NULL) receives k.  res_sq (host, may be NULL) gets
 * ||W - D||_F^2.  d: device fp32 [n]. */
admmq_status admmq_project_dual(admmq_ctx *ctx, const float *W, float *V, int64_t n, int64_t p,
                                const float *d, int32_t bits, int32_t group_size, const float *scales,
                                const float *zeros, double rho, double rho_next, uint8_t *codes,
                                float *B_out, double *res_sq);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc): admmq_project_dual without the context's arena.  Its scratch (the fp32 reciprocals of d and of
 * scales: 4*(n + (n/g)*p) bytes, each rounded up to 256) lives in a fixed array inside the library's device image,
 * ADMMQ_NOALLOC_SCRATCH_BYTES per GPU, held until the process ends; a shape that needs more returns
 * ADMMQ_ERR_WORKSPACE before any device work.  The call allocates and frees nothing, clears with a kernel rather
 * than a memset, and never synchronises: res_sq is a DEVICE pointer here (8-byte aligned double, may be NULL)
 * that receives ||W - D||_F^2 when the enqueued work completes.  All other arguments, the arithmetic and the
 * results (codes, V, B_out bit for bit) are those of admmq_project_dual.  Every call on one GPU uses that GPU's
 * one array, whatever the context or stream: calls that overlap in time on one GPU race - keep them in stream
 * order. */
#define ADMMQ_NOALLOC_SCRATCH_BYTES (8u << 20)
admmq_status admmq_project_dual_noalloc(admmq_ctx *ctx, const float *W, float *V, int64_t n, int64_t p,
                                        const float *d, int32_t bits, int32_t group_size, const float *scales,
                                        const float *zeros, double rho, double rho_next, uint8_t *codes,
                                        float *B_out, double *res_sq);

/* Grid refresh (Sec. 3.3, App. B) on the state of one iteration: refits (scales, zeros) by min/max of
 * the projection target Sigma (W + V/rho) per group, projects the target on the old and on the refitted
 * grid, and accepts the refit iff ||D_new - Wt||_F^2 <= ||D_old - Wt||_F^2 (eq. 12, scaled variables).
 * On acceptance scales/zeros (device, [n/g][p]) are overwritten.  W, V: device fp32 [n][p]; d: [n].
 * accepted, err_old, err_new: host outputs (err_* may be NULL). */
admmq_status admmq_grid_refresh(admmq_ctx *ctx, const float *W, const float *V, int64_t n, int64_t p,
                                const float *d, int32_t bits, int32_t group_size, double rho, float *scales,
                                float *zeros, int32_t *accepted, double *err_old, double *err_new);

/* Tr(E^T (H + lambda I) E) with E = dequant(codes) - W0, lambda = damp * Tr(H)/n (eq. 2 x 2). */
admmq_status admmq_objective(admmq_ctx *ctx, const float *H, const float *W0, int64_t n, int64_t p,
                             int64_t ldw, int32_t group_size, const float *scales, const float *zeros,
                             const uint8_t *codes, double damp, double *j_out);

/* One batch of eq. 11: for `npairs` row pairs (device int32 [npairs][2]) the summed gain over the
 * columns, each column taking its best feasible sign combination if that lowers the loss.
 * G: device fp32 [n][p] = H'(W0 - Wq).  totals: device fp32 [npairs]. */
admmq_status admmq_ls_evaluate(admmq_ctx *ctx, const float *H, double lambda, const float *G,
                               const uint8_t *codes, int64_t n, int64_t p, int32_t bits,
                               int32_t group_size, const float *scales, const int32_t *pairs,
                               int32_t npairs, float *totals);

/* ---- other quantization formats (Sec. 4.3) ------------------------------------------------------------
 * Only the projection of the D-update changes; the W- and V-updates, the schedule and the factorisation
 * are those of admmq_quantize_layer.  The paper names the two formats and prints no formulas; the
 * conventions below are this library's.
 *
 * ADMMQ_FORMAT_DUAL_GRID: flags[i][j] != 0 marks an outlier.  Within each group of each output channel
 *   the inliers share one uniform grid and the outliers another (same bits); scales / zeros are
 *   [2][n/g][p] (inlier grid first), fitted by min/max over each subset of W0 (an empty subset gets
 *   scale 0: its codes stay 0).
 * ADMMQ_FORMAT_CODEBOOK: codebook[l][j], l < 2^bits, strictly ascending in l, holds the levels of output
 *   channel j (bits 1..4, group_size must be 0).  An entry goes to the nearest level, the lower one when
 *   two are equally near.  flags (may be NULL) marks entries kept dense: they are unconstrained, their
 *   projection is the target itself, their dual is 0 and their code is 0.
 * All pointers are device pointers; flags is u8 [n][p] contiguous. */
typedef enum admmq_format_kind { ADMMQ_FORMAT_DUAL_GRID = 1, ADMMQ_FORMAT_CODEBOOK = 2 } admmq_format_kind;

typedef struct admmq_format {
    int32_t kind;            /* admmq_format_kind */
    int32_t bits;
    int32_t group_size;      /* dual grid: 0 = one group per column; codebook: 0 */
    const uint8_t *flags;    /* [n][p]; dual grid: required; codebook: optional */
    const float *codebook;   /* codebook only: [2^bits][p] */
    float *scales;           /* dual grid only: [2][n/g][p]; written by admmq_quantize_layer_format and */
    float *zeros;            /*   admmq_grid_init_dual, read by admmq_project_dual_format             */
} admmq_format;

/* Dual-grid fit on W0 (see above); fmt->scales / fmt->zeros receive the two grids. */
admmq_status admmq_grid_init_dual(admmq_ctx *ctx, const float *W0, int64_t n, int64_t p, int64_t ldw,
                                  const admmq_format *fmt);

/* The fused projection + dual pass of admmq_project_dual with the projection of `fmt` (eqs. 8 and 9 with
 * the format's own admissible set in place of eq. 10).  Xq_out (device fp32 [n][p], may be NULL) receives the
 * projected values in the unscaled space, Sigma D.  ADMMQ_ERR_PARAM for a codebook that is not finite and
 * strictly ascending. */
admmq_status admmq_project_dual_format(admmq_ctx *ctx, const float *W, float *V, int64_t n, int64_t p,
                                       const float *d, const admmq_format *fmt, double rho, double rho_next,
                                       uint8_t *codes, float *B_out, float *Xq_out, double *res_sq);

/* Alg. 1 lines 1-10 with the projection of `fmt`.  codes: device u8 [n][p]; Wq: device fp32 [n][p], the
 * quantized weights Sigma D^(T) in the unscaled space (kept entries hold their dense values).  No local
 * search (its moves of one grid step are defined for uniform grids): sched->ls_rounds, refresh_iter (other
 * than -1), symmetric and clip_points must be 0, else ADMMQ_ERR_PARAM; stats->code_flips must be NULL.
 * stats->j_damp_rtn is the objective of the plain projection of W0. */
admmq_status admmq_quantize_layer_format(admmq_ctx *ctx, const float *H, const float *W0, int64_t n, int64_t p,
                                         int64_t ldw, const admmq_format *fmt, const admmq_schedule *sched,
                                         uint8_t *codes, float *Wq, admmq_stats *stats);

#ifdef __cplusplus
}
#endif
#endif /* ADMMQ_H */
