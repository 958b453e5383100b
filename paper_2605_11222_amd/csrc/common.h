// Shared host-side declarations of the ADMM-Q library: context, scratch arena, launch wrappers.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/admmq.h"

#define ADMMQ_HIP(call)                                  \
    do {                                                 \
        hipError_t e_ = (call);                          \
        if (e_ != hipSuccess) return ADMMQ_ERR_DEVICE;   \
    } while (0)

#define ADMMQ_TRY(call)                     \
    do {                                    \
        admmq_status s_ = (call);           \
        if (s_ != ADMMQ_OK) return s_;      \
    } while (0)

// Factorisation of the scaled, damped Hessian kept between calls:  Hs = Q M Q^T with M a band matrix of
// half-bandwidth 16 (`band`: large n) or tridiagonal (`ta`, `tb`: small n); see admmq_factor_is_band.
struct admmq_factor {
    int64_t n = 0;
    double lambda = 0.0;
    float *d = nullptr;       // [n] d_i = sqrt(H'_ii)
    float *inv_d = nullptr;   // [n] fp32 reciprocal of d_i
    float *Q = nullptr;       // [n][n] fp32, row-major Q
    float *Qt = nullptr;      // [n][n] fp32, row-major Q^T
    double *ta = nullptr;     // [n]   diagonal of T
    double *tb = nullptr;     // [n]   sub-diagonal of T (tb[n-1] = 0)
    double *band = nullptr;   // [17][npad] band[t][j] = M[j + t][j], npad = n rounded up to 16; NULL for the tridiagonal form
    bool valid = false;
    const float *H_src = nullptr;   // the raw Hessian it was made from (identity check for reuse)
    double damp = 0.0;
    int precondition = 1;
};

// Optional per-launch timing: pairs of HIP events on the context's stream, summed per tag at the end.
struct admmq_profiler {
    struct span { hipEvent_t a, b; int tag; };
    span *spans = nullptr;
    int count = 0, cap = 0;
    bool on = false;
};
enum { ADMMQ_TAG_GEMM = 0, ADMMQ_TAG_TRIDIAG = 1, ADMMQ_TAG_PROJECT = 2, ADMMQ_TAG_LS_APPLY = 3, ADMMQ_TAG_GEMM_PROJECT = 4,
       ADMMQ_TAGS = 5 };

struct admmq_ctx {
    int device = 0;
    admmq_profiler prof;
    hipStream_t stream = nullptr;
    // bump arena: [0, persist_top) holds the factorisation, [persist_top, top) transient scratch
    char *arena = nullptr;
    size_t arena_bytes = 0;
    bool arena_owned = true;
    size_t persist_top = 0;
    size_t top = 0;
    admmq_factor fac;
    // small pinned host buffer for scalar read-backs
    double *host_scalars = nullptr;   // 64 doubles
    // streams (default priority) on which independent local searches of one batched call run side by side
    hipStream_t side[3] = {nullptr, nullptr, nullptr};
    hipEvent_t side_ready = nullptr;
    // events that order the accumulation of Q (on side[0]) after the panels of the factorisation: created on
    // first use, kept for the context's lifetime
    hipEvent_t *panel_events = nullptr;
    int panel_event_count = 0;
    // opt-in: W-update products of whole 256 x 256 tiles as three fp16 matrix-core products of split operands
    bool fast_on = false;
    // groups of the last local search on this context that gave up a bounded wait and were redone batch by batch
    int ls_fallback_groups = 0;
    // how many local searches run side by side on the device (the batched call's helper contexts): a search whose
    // blocks wait for one another may only launch what fits beside the others
    int ls_side_by_side = 1;
    // this device's copy of the library's fixed scratch array (the entry point that allocates nothing)
    void *fixed_scratch = nullptr;
};

// Returns a span index (or -1 when profiling is off); call admmq_prof_end with it after the launch.
int admmq_prof_begin(admmq_ctx *ctx, int tag);
void admmq_prof_end(admmq_ctx *ctx, int span);

static inline size_t admmq_align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }

// Kernels with more than 64 KB of dynamic LDS need the attribute raised once per kernel and device; `done` is the
// call site's own bit mask of the devices already served (a relaxed race between two threads sets it twice at worst).
static inline hipError_t admmq_allow_lds(const void *kernel, int bytes, int device, unsigned long long *done) {
    const unsigned long long bit = 1ull << (device & 63);
    if (*done & bit) return hipSuccess;
    const hipError_t e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess) *done |= bit;
    return e;
}

// Makes sure the arena can hold `bytes` above the persistent region; keeps the persistent region.
admmq_status admmq_arena_reserve(admmq_ctx *ctx, size_t bytes);
// Bump allocation inside the reserved arena (never fails after a sufficient reserve).
void *admmq_arena_alloc(admmq_ctx *ctx, size_t bytes);
static inline void admmq_arena_reset_transient(admmq_ctx *ctx) { ctx->top = ctx->persist_top; }

// ---- GEMM family (gemm_tn.hip) -------------------------------------------------------------
// out[m][n] = alpha * sum_{k in [0,K)} A[k][m] * B[k][n] + beta * Z[m][n]
// A is [K][lda] (fp32, or bf16 bit patterns when a_bf16), B is [K][ldb] likewise; both operands are
// "k-major": consecutive m (or n) are contiguous.  Z may be NULL (beta ignored) and may alias out.
struct gemm_tn_args {
    const void *A;
    const void *B;
    int64_t lda, ldb;
    int a_bf16, b_bf16;
    int64_t M, N, K;
    float alpha, beta;
    const float *Z;
    int64_t ldz;
    float *out;
    int64_t ldo;
    int lower_only;      // 1: only tiles that touch the lower triangle (m >= n) are computed
    int split_k;         // >1: slice s handles k in [s*Kc,(s+1)*Kc) and writes out + s*slice_stride
    int64_t slice_stride;
    const struct gemm_proj_args *proj;    // not NULL: eqs. 8-10 applied to the result while it is in registers
};
// Projection, dual update and residual (eqs. 8-10) as the epilogue of the second product of eq. 7: the product's
// result W = A^T B + Z never goes to memory; with t = W + V/rho the epilogue forms D = P_Q(t) on the grid, V += rho
// (W - D) in place, writes B' = D - V/rho_next to `out` (which may be Z itself) and adds |W - D|_F^2 to res_sq.
// The arithmetic per element is that of the stand-alone pass (admmq_k_project_dual), operation for operation.
// Needs alpha = beta = 1, Z given, whole aligned tiles (admmq_gemm_tn_can_project) and a group size that is a power
// of two or the whole column (g_shift = log2 g, or 62 for one group).
struct gemm_proj_args {
    float *V;
    int64_t ldv;
    const float *d, *inv_d;               // [M]
    const float *scales, *inv_scales, *zeros;   // [M / g][ld_grid], indexed by the product's column
    int64_t ld_grid;
    int g_shift;
    float levels, rho, inv_rho, inv_rho_next;
    double *res_sq;
};
admmq_status admmq_gemm_tn(admmq_ctx *ctx, const gemm_tn_args &a);
bool admmq_gemm_tn_can_project(const gemm_tn_args &a);
// bf16 matrix-core path of the Hessian (hessian_bf16.hip): usable when n is a multiple of 256, rows of X are 16-byte
// aligned and there is at least one 32-token stage; handles the first main_rows(rows) tokens.
bool admmq_hessian_bf16_ok(const void *X, int64_t n, int64_t ldx, int64_t rows);
int64_t admmq_hessian_bf16_main_rows(int64_t rows);
admmq_status admmq_hessian_bf16(admmq_ctx *ctx, const void *X, int64_t ldx, int64_t k_main, int64_t n, float *P,
                                int split, int64_t slice_stride);
// Split-fp16 products (gemm_f16x3.hip).  split: hi = fp16(s x), lo = fp16(s x - hi), s the power of two that brings
// the largest |x| into [2^14, 2^15); slots: 8 bytes of device scratch per matrix (largest |x| as bits, zero on
// entry, then s); next_slots (may be NULL): another matrix's slots, whose first word is zeroed for the split after;
// have_max: the kernel that wrote src has already left the largest |x| in the slot.
// product: out = alpha * A^T B + beta * Z with A, B given by their fp16 pairs, k-major [K][M] and [K][N] with dense
// rows; M, N multiples of 256, K a multiple of 32 (admmq_gemm_f16x3_ok).
// With fewer than 200 tiles the k axis is cut into 2, 4 or 8 slices whose partial sums (partial_bytes of scratch,
// passed as `partial`) a second kernel adds up.
bool admmq_gemm_f16x3_ok(int64_t M, int64_t N, int64_t K);
int admmq_gemm_f16x3_split(int64_t M, int64_t N, int64_t K);
size_t admmq_gemm_f16x3_partial_bytes(int64_t M, int64_t N, int64_t K);
admmq_status admmq_k_split_f16(admmq_ctx *ctx, const float *src, int64_t rows, int64_t cols, int64_t ld, void *hi,
                               void *lo, void *slots, void *next_slots, bool have_max = false);
admmq_status admmq_gemm_f16x3(admmq_ctx *ctx, const void *A1, const void *A2, const void *slotsA, const void *B1,
                              const void *B2, const void *slotsB, int64_t M, int64_t N, int64_t K, float alpha,
                              float beta, const float *Z, int64_t ldz, float *out, int64_t ldo,
                              float *partial = nullptr);
// H[i][j] (+)= sum_s P[s][i][j] for i >= j and mirrors the result into the upper triangle.
admmq_status admmq_sym_reduce(admmq_ctx *ctx, float *H, int64_t n, const float *P, int slices,
                              int64_t slice_stride, int accumulate);

// ---- streaming kernels (stream.hip) --------------------------------------------------------
admmq_status admmq_k_grid_init(admmq_ctx *ctx, const float *W0, int64_t n, int64_t p, int64_t ldw, int bits,
                               int64_t g, float *scales, float *zeros);
// min/max fit with the options of Sec. 3.4: symmetric range and MSE clipping search (clip_points = 0: off)
admmq_status admmq_k_grid_fit(admmq_ctx *ctx, const float *W0, int64_t n, int64_t p, int64_t ldw, int bits,
                              int64_t g, int symmetric, int clip_points, double clip_shrink, float *scales,
                              float *zeros);
admmq_status admmq_k_project_dual(admmq_ctx *ctx, const float *W, float *V, int64_t n, int64_t p, const float *d,
                                  const float *inv_d, int bits, int64_t g, const float *scales,
                                  const float *inv_scales, const float *zeros, float rho, float inv_rho,
                                  float inv_rho_next, uint8_t *codes, int count_flips, float *B_out,
                                  double *dev_res_sq, unsigned long long *dev_flips, int64_t ldw,
                                  unsigned *amax_out = nullptr);   // amax_out: atomic max of |B| as float bits
// grid refresh (App. B): refit by min/max of the projection target; both sides of eq. 12 as per-block partials
admmq_status admmq_k_refit_grid(admmq_ctx *ctx, const float *W, const float *V, int64_t n, int64_t p,
                                const float *inv_d, float inv_rho, int bits, int64_t g, float *scales, float *zeros);
int admmq_refresh_error_blocks();
admmq_status admmq_k_refresh_error(admmq_ctx *ctx, const float *W, const float *V, int64_t n, int64_t p,
                                   const float *d, const float *inv_d, float inv_rho, int bits, int64_t g,
                                   const float *sc_old, const float *zr_old, const float *sc_new,
                                   const float *zr_new, double *part);
// inv[i] = 1/x[i] in fp32 with IEEE division, 0 where x[i] == 0
admmq_status admmq_k_recip(admmq_ctx *ctx, const float *x, float *inv, int64_t n);
admmq_status admmq_k_scale_rows(admmq_ctx *ctx, const float *W0, int64_t ldw, const float *d, int64_t n, int64_t p,
                                float *out, int64_t ldo);
// B = D - V * inv_rho
admmq_status admmq_k_form_b(admmq_ctx *ctx, const float *D, const float *V, float inv_rho, int64_t count,
                            float *B);
// dst[0, bytes) = src[0, bytes), bytes a multiple of 16, both 16-byte aligned
admmq_status admmq_k_stream_copy(admmq_ctx *ctx, void *dst, const void *src, size_t bytes);
admmq_status admmq_k_fill_f32(admmq_ctx *ctx, float *x, float v, int64_t count);
admmq_status admmq_k_fill_bytes(admmq_ctx *ctx, void *x, int v, size_t bytes);
// mode 0: E = dequant(codes) - W0; mode 1: E = W0 - dequant(codes); mode 2: codes := round-to-nearest
// of W0 on the grid first, then E = dequant(codes) - W0
admmq_status admmq_k_quant_error(admmq_ctx *ctx, const float *W0, int64_t ldw, uint8_t *codes, int64_t n,
                                 int64_t p, int64_t g, const float *scales, const float *zeros, int bits, int mode,
                                 float *E);
// *dev_out = sum_{i,j} A[i][j] * B[i][j]  (double accumulation)
admmq_status admmq_k_dot(admmq_ctx *ctx, const float *A, const float *B, int64_t count, double *dev_out);
// trace and finiteness of a square fp32 matrix; dev_out[0] = trace, dev_out[1] = #non-finite entries,
// dev_out[2] = #diagonal entries <= 0 after adding nothing (raw diagonal)
admmq_status admmq_k_matrix_check(admmq_ctx *ctx, const float *H, int64_t n, double *dev_out);
admmq_status admmq_k_count_nonfinite(admmq_ctx *ctx, const float *A, int64_t rows, int64_t cols, int64_t ld,
                                     double *dev_out);

// ---- factorisation (factor.hip) ------------------------------------------------------------
// LDL^T factors of T + rho_t I for `count` values of rho: dinv[t][i], l[t][i] (fp64).
admmq_status admmq_k_tridiag_factor(admmq_ctx *ctx, const double *ta, const double *tb, int64_t n,
                                    const double *rhos_dev, int count, double *dinv, double *lfac);
// S = (T + rho I)^{-1} T Y, column by column (Y, S fp32 [n][p]; may alias), F fp64 scratch [n][p]
// The same two steps for the band form (band.hip): block-elimination factors of M + rho_t I, and the solve.
size_t admmq_band_factor_doubles(int64_t n, int count);
admmq_status admmq_k_band_factor(admmq_ctx *ctx, const double *bd, int64_t n, const double *rhos_dev, int count,
                                 double *fac);
admmq_status admmq_k_band_apply(admmq_ctx *ctx, const double *fac, int64_t n, int64_t p, const float *Y, float *S,
                                unsigned *amax_out = nullptr);
// which form the factorisation of an n x n Hessian takes (band from n = 8192 on; ADMMQ_FACTOR=band / tridiag forces one)
bool admmq_factor_is_band(int64_t n);
admmq_status admmq_k_tridiag_apply(admmq_ctx *ctx, const double *ta, const double *tb, const double *dinv,
                                   const double *lfac, int64_t n, int64_t p, const float *Y, double *carries,
                                   float *S, unsigned *amax_out = nullptr);   // atomic max of |S| as float bits
