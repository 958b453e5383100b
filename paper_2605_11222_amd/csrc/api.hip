// C ABI of the ADMM-Q library: argument validation, scratch arena, and the orchestration of Alg. 1.
#include <math.h>
#include <stdlib.h>
#include <string.h>

#include <mutex>
#include <new>
#include <thread>
#include <vector>

#include "common.h"

// No C++ exception may cross the C boundary (or leave a helper thread): host allocations that fail become an error code.
template <class F>
static admmq_status admmq_guarded(F &&body) {
    try {
        return body();
    } catch (const std::bad_alloc &) {
        return ADMMQ_ERR_WORKSPACE;
    } catch (...) {
        return ADMMQ_ERR_DEVICE;
    }
}

// ---- declarations of launchers defined in the other translation units -----------------------
admmq_status admmq_k_scaling(admmq_ctx *ctx, const float *H, int64_t n, double lambda, int precondition, float *d,
                             float *inv_d, double *dev_flags);
admmq_status admmq_k_factorize(admmq_ctx *ctx, const float *H, int64_t n, double lambda, const float *d,
                               double *A64, double *R64, double *vecs, float *Q, float *Qt, double *ta,
                               double *tb, double *band);
size_t admmq_band_scratch_doubles(int64_t n);
size_t admmq_householder_scratch_doubles(int64_t n);
int admmq_ls_chunks(int64_t p);
int admmq_ls_defer();
admmq_status admmq_k_ls_step(admmq_ctx *ctx, const float *H, float lambda, const float *G, const uint8_t *codes,
                             int64_t n, int64_t p, int bits, int64_t g, const float *scales,
                             const int32_t *pairs_prev, int npairs_prev, const float *partial_prev,
                             const uint8_t *mv_prev, int slot_prev, const int32_t *pairs_cur, int npairs_cur,
                             int npend, int32_t *pend_idx, float *pend_d, float *hcol, float *partial_cur,
                             uint8_t *mv_cur, int32_t *choice, int *dev_moves, double *dev_drop,
                             const int32_t *pairs_next, int npairs_next, const float *exs_cur, float *exs_next);
int admmq_ls_fast_pairs();
admmq_status admmq_k_ls_flush(admmq_ctx *ctx, const float *H, float lambda, float *G, uint8_t *codes, int64_t n,
                              int64_t p, const int32_t *pend_idx, const float *pend_d, int count,
                              const int *commit = nullptr, int commit_needed = 0);
int admmq_ls_group_pairs_per_thread(admmq_ctx *ctx, int64_t p, int npairs);
size_t admmq_ls_group_xch_words(int64_t p);
int admmq_ls_group_max_blocks(int64_t p);
admmq_status admmq_k_ls_group(admmq_ctx *ctx, int pairs_per_thread, const float *H, float lambda, const float *G,
                              const uint8_t *codes, int64_t n, int64_t p, int bits, int64_t g, const float *scales,
                              const int32_t *pairs, int npairs, int cnt, unsigned seq0, int group_seq,
                              unsigned long long *xch, unsigned *fin, int *commit, int *abort_word,
                              long long spin_ticks, int32_t *pend_idx, float *pend_d, int *dev_moves,
                              double *dev_drop, const float *couple);
admmq_status admmq_k_ls_couple(admmq_ctx *ctx, const float *H, float lambda, int64_t n, const int32_t *pairs,
                               int npairs, int batches, float *X);
size_t admmq_ls_couple_floats(int batches);
admmq_status admmq_k_ls_totals(admmq_ctx *ctx, const float *partial, int chunks, int npairs, float *totals);
admmq_status admmq_k_dual_grid_init(admmq_ctx *ctx, const float *W0, int64_t n, int64_t p, int64_t ldw, int bits,
                                    int64_t g, const uint8_t *flags, float *scales, float *zeros);
admmq_status admmq_k_codebook_check(admmq_ctx *ctx, const float *codebook, int L, int64_t p, double *dev_bad);
admmq_status admmq_k_project_format(admmq_ctx *ctx, int kind, const float *W, float *V, int64_t n, int64_t p,
                                    const float *d, const float *inv_d, int bits, int64_t g,
                                    const uint8_t *flags, const float *scales, const float *inv_scales,
                                    const float *zeros, const float *codebook, float rho, float inv_rho,
                                    float inv_rho_next, int last, uint8_t *codes, float *B_out, float *Xq,
                                    double *dev_res_sq, unsigned *amax_out = nullptr);
admmq_status admmq_k_nearest_error(admmq_ctx *ctx, int kind, const float *W0, int64_t ldw, int64_t n, int64_t p,
                                   int bits, int64_t g, const uint8_t *flags, const float *scales,
                                   const float *zeros, const float *codebook, uint8_t *codes, float *E);
admmq_status admmq_k_diff(admmq_ctx *ctx, const float *A, const float *W0, int64_t ldw, int64_t n, int64_t p,
                          float *E);

// ---- per-launch profiler ---------------------------------------------------------------------
int admmq_prof_begin(admmq_ctx *ctx, int tag) {
    admmq_profiler &pf = ctx->prof;
    if (!pf.on) return -1;
    if (pf.count == pf.cap) {
        const int ncap = pf.cap ? pf.cap * 2 : 1024;
        admmq_profiler::span *ns = (admmq_profiler::span *)realloc(pf.spans, (size_t)ncap * sizeof(*ns));
        if (!ns) return -1;
        pf.spans = ns;
        pf.cap = ncap;
    }
    admmq_profiler::span &sp = pf.spans[pf.count];
    if (hipEventCreate(&sp.a) != hipSuccess) return -1;
    if (hipEventCreate(&sp.b) != hipSuccess) {
        (void)hipEventDestroy(sp.a);
        return -1;
    }
    sp.tag = tag;
    (void)hipEventRecord(sp.a, ctx->stream);
    return pf.count++;
}

void admmq_prof_end(admmq_ctx *ctx, int span) {
    if (span >= 0) (void)hipEventRecord(ctx->prof.spans[span].b, ctx->stream);
}

// sums and releases the recorded spans (synchronises the stream)
static void prof_collect(admmq_ctx *ctx, float ms[ADMMQ_TAGS], int cnt[ADMMQ_TAGS]) {
    admmq_profiler &pf = ctx->prof;
    for (int t = 0; t < ADMMQ_TAGS; ++t) { ms[t] = 0.f; cnt[t] = 0; }
    if (pf.count > 0) (void)hipStreamSynchronize(ctx->stream);
    for (int i = 0; i < pf.count; ++i) {
        float e = 0.f;
        if (hipEventElapsedTime(&e, pf.spans[i].a, pf.spans[i].b) == hipSuccess) {
            ms[pf.spans[i].tag] += e;
            cnt[pf.spans[i].tag] += 1;
        }
        (void)hipEventDestroy(pf.spans[i].a);
        (void)hipEventDestroy(pf.spans[i].b);
    }
    pf.count = 0;
    pf.on = false;
}

// ---- arena -------------------------------------------------------------------------------------
admmq_status admmq_arena_reserve(admmq_ctx *ctx, size_t bytes) {
    const size_t need = ctx->persist_top + admmq_align_up(bytes) + 4096;
    if (need <= ctx->arena_bytes) return ADMMQ_OK;
    if (!ctx->arena_owned) return ADMMQ_ERR_WORKSPACE;
    char *fresh = nullptr;
    if (hipMalloc((void **)&fresh, need) != hipSuccess) {
        (void)hipGetLastError();
        return ADMMQ_ERR_WORKSPACE;
    }
    if (ctx->arena) {
        if (ctx->persist_top > 0) {
            ADMMQ_HIP(hipMemcpyAsync(fresh, ctx->arena, ctx->persist_top, hipMemcpyDeviceToDevice, ctx->stream));
            // persistent pointers move with the arena
            const ptrdiff_t shift = fresh - ctx->arena;
            admmq_factor &f = ctx->fac;
            auto mvf = [shift](float *&ptr) { if (ptr) ptr = (float *)((char *)ptr + shift); };
            auto mvd = [shift](double *&ptr) { if (ptr) ptr = (double *)((char *)ptr + shift); };
            mvf(f.d); mvf(f.inv_d); mvf(f.Q); mvf(f.Qt); mvd(f.ta); mvd(f.tb); mvd(f.band);
        }
        ADMMQ_HIP(hipStreamSynchronize(ctx->stream));
        ADMMQ_HIP(hipFree(ctx->arena));
    }
    ctx->arena = fresh;
    ctx->arena_bytes = need;
    return ADMMQ_OK;
}

void *admmq_arena_alloc(admmq_ctx *ctx, size_t bytes) {
    const size_t off = admmq_align_up(ctx->top);
    if (off + bytes > ctx->arena_bytes) return nullptr;
    ctx->top = off + bytes;
    return ctx->arena + off;
}

namespace {

template <typename T>
admmq_status take(admmq_ctx *ctx, T *&ptr, size_t count) {
    ptr = (T *)admmq_arena_alloc(ctx, count * sizeof(T));
    return ptr ? ADMMQ_OK : ADMMQ_ERR_WORKSPACE;
}

size_t band_doubles(int64_t n) { return 17 * (((size_t)n + 15) / 16 * 16); }
size_t factor_persist_bytes(int64_t n) {
    const size_t N = (size_t)n;
    return 2 * admmq_align_up(N * 4) + 2 * admmq_align_up(N * N * 4) + 2 * admmq_align_up(N * 8) +
           admmq_align_up(band_doubles(n) * 8) + 4096;
}
size_t factor_scratch_doubles(int64_t n) {
    const size_t a = admmq_householder_scratch_doubles(n), b = admmq_band_scratch_doubles(n);
    return a > b ? a : b;
}
size_t factor_transient_bytes(int64_t n) {
    const size_t N = (size_t)n;
    return 2 * admmq_align_up(N * N * 8) + admmq_align_up(factor_scratch_doubles(n) * 8) + 4096;
}
// The factors of the middle matrix plus rho_t I for a whole schedule: two n-vectors per penalty for the tridiagonal
// form (LDL^T), three 16 x 16 matrices per block row and penalty for the band form.
struct MidFactors {
    double *a = nullptr, *b = nullptr;
    size_t stride = 0;          // doubles per penalty
};
size_t mid_factor_bytes(int64_t n, int32_t T) {
    // (room for either form: the choice can be forced through the environment between two calls)
    const size_t a = admmq_align_up(admmq_band_factor_doubles(n, T) * 8), b = 2 * admmq_align_up((size_t)T * n * 8);
    return admmq_factor_is_band(n) ? (a > b ? a : b) : b;
}
size_t admm_transient_bytes(int64_t n, int64_t p, int32_t T) {
    const size_t np = (size_t)n * (size_t)p;
    return 6 * admmq_align_up(np * 4) + admmq_align_up((np + (size_t)p) * 8) + mid_factor_bytes(n, T) +
           4 * admmq_align_up((size_t)T * 8) + 65536;
}
// batches whose coupling table (H' between the candidates of consecutive batches) is formed in one launch
constexpr int LS_COUPLE_SPAN = 1024;
size_t ls_transient_bytes(int64_t n, int64_t p, int64_t total_pairs, int pairs_per_batch) {
    const size_t np = (size_t)n * (size_t)p;
    const int64_t nb = pairs_per_batch > 0 ? total_pairs / pairs_per_batch : 0;
    return admmq_align_up(admmq_ls_couple_floats((int)(nb < LS_COUPLE_SPAN ? nb : LS_COUPLE_SPAN)) * 4) +
           2 * admmq_align_up(np * 4) + admmq_align_up((size_t)total_pairs * 8) +
           2 * admmq_align_up((size_t)pairs_per_batch * admmq_ls_chunks(p) * 4) +
           admmq_align_up((size_t)2 * admmq_ls_defer() * p * 4) + admmq_align_up((size_t)pairs_per_batch * 4) +
           2 * admmq_align_up((size_t)pairs_per_batch * p) + admmq_align_up((size_t)2 * admmq_ls_defer() * n * 4) +
           2 * admmq_align_up((size_t)admmq_ls_fast_pairs() * admmq_ls_fast_pairs() * 16) +
           admmq_align_up(admmq_ls_group_xch_words(p) * 8) + admmq_align_up((size_t)admmq_ls_group_max_blocks(p) * 4) + 65536;
}

admmq_status read_back(admmq_ctx *ctx, void *host, const void *dev, size_t bytes) {
    ADMMQ_HIP(hipMemcpyAsync(host, dev, bytes, hipMemcpyDeviceToHost, ctx->stream));
    ADMMQ_HIP(hipStreamSynchronize(ctx->stream));
    return ADMMQ_OK;
}

inline uint64_t mix64(uint64_t x) {
    x += 0x9E3779B97F4A7C15ull;
    uint64_t z = x;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

admmq_status check_layer_args(const void *H, const void *W0, int64_t n, int64_t p, int64_t ldw, int32_t bits,
                              int32_t group_size) {
    if (!H || !W0) return ADMMQ_ERR_NULL;
    if (n < 1 || p < 1 || ldw < p || n > (1 << 20) || p > (1 << 24)) return ADMMQ_ERR_SHAPE;
    if (group_size < 0 || (group_size > 0 && n % group_size != 0)) return ADMMQ_ERR_SHAPE;
    if (bits < 2 || bits > 8) return ADMMQ_ERR_PARAM;
    return ADMMQ_OK;
}

struct Timer {
    hipEvent_t a = nullptr, b = nullptr;
    hipStream_t st;
    bool on;
    Timer(hipStream_t s, bool enable) : st(s), on(enable) {
        if (on) {
            if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) on = false;
        }
    }
    ~Timer() {
        if (a) (void)hipEventDestroy(a);
        if (b) (void)hipEventDestroy(b);
    }
    void start() { if (on) (void)hipEventRecord(a, st); }
    float stop() {
        if (!on) return 0.f;
        (void)hipEventRecord(b, st);
        (void)hipEventSynchronize(b);
        float ms = 0.f;
        (void)hipEventElapsedTime(&ms, a, b);
        return ms;
    }
};

// trace, finiteness and lambda of a raw Hessian (synchronises)
admmq_status hessian_scalars(admmq_ctx *ctx, const float *H, int64_t n, double damp, double *lambda) {
    double *dev = nullptr;
    ADMMQ_TRY(take(ctx, dev, 4));
    ADMMQ_TRY(admmq_k_fill_bytes(ctx, dev, 0, 32));
    ADMMQ_TRY(admmq_k_matrix_check(ctx, H, n, dev));
    double host[4];
    ADMMQ_TRY(read_back(ctx, host, dev, 32));
    if (host[1] > 0.0 || !isfinite(host[0])) return ADMMQ_ERR_NOT_FINITE;
    *lambda = damp * host[0] / (double)n;
    return ADMMQ_OK;
}

// Alg. 1 lines 1-3 into the persistent region; leaves the transient region reset.
admmq_status do_factorize(admmq_ctx *ctx, const float *H, int64_t n, double damp, int precondition,
                          double *lambda_out) {
    ctx->fac.valid = false;
    ctx->persist_top = 0;
    ctx->top = 0;
    ADMMQ_TRY(admmq_arena_reserve(ctx, factor_persist_bytes(n) + factor_transient_bytes(n)));
    admmq_factor &f = ctx->fac;
    f = admmq_factor();
    ADMMQ_TRY(take(ctx, f.d, (size_t)n));
    ADMMQ_TRY(take(ctx, f.inv_d, (size_t)n));
    ADMMQ_TRY(take(ctx, f.Q, (size_t)n * n));
    ADMMQ_TRY(take(ctx, f.Qt, (size_t)n * n));
    ADMMQ_TRY(take(ctx, f.ta, (size_t)n));
    ADMMQ_TRY(take(ctx, f.tb, (size_t)n));
    if (admmq_factor_is_band(n)) ADMMQ_TRY(take(ctx, f.band, band_doubles(n)));
    ctx->persist_top = admmq_align_up(ctx->top);
    ctx->top = ctx->persist_top;

    double lambda = 0.0;
    ADMMQ_TRY(hessian_scalars(ctx, H, n, damp, &lambda));
    double *flags = nullptr;
    ADMMQ_TRY(take(ctx, flags, 4));
    ADMMQ_TRY(admmq_k_fill_bytes(ctx, flags, 0, 32));
    ADMMQ_TRY(admmq_k_scaling(ctx, H, n, lambda, precondition, f.d, f.inv_d, flags));
    double hflag[4];
    ADMMQ_TRY(read_back(ctx, hflag, flags, 32));
    if (hflag[0] > 0.0) {
        ctx->persist_top = 0;
        ctx->top = 0;
        return ADMMQ_ERR_ZERO_DIAG;
    }
    double *A64 = nullptr, *R64 = nullptr, *vecs = nullptr;
    ADMMQ_TRY(take(ctx, A64, (size_t)n * n));
    ADMMQ_TRY(take(ctx, R64, (size_t)n * n));
    ADMMQ_TRY(take(ctx, vecs, factor_scratch_doubles(n)));
    ADMMQ_TRY(admmq_k_factorize(ctx, H, n, lambda, f.d, A64, R64, vecs, f.Q, f.Qt, f.ta, f.tb, f.band));
    f.n = n;
    f.lambda = lambda;
    f.H_src = H;
    f.damp = damp;
    f.precondition = precondition;
    f.valid = true;
    if (lambda_out) *lambda_out = lambda;
    admmq_arena_reset_transient(ctx);
    return ADMMQ_OK;
}

// Opt-in fast products (admmq_set_fast_products): Q and Q^T split into fp16 pairs once per call, the state operand
// before each product; all of it in the call's transient arena.
struct FastBufs {
    void *Q1 = nullptr, *Q2 = nullptr, *Qt1 = nullptr, *Qt2 = nullptr, *O1 = nullptr, *O2 = nullptr;
    float *partial = nullptr;                  // partial sums of a product whose k axis is cut into slices
    void *slotsQ = nullptr, *slotsQt = nullptr;
    void *slotsO[2] = {nullptr, nullptr};      // the state operand's two splits per W-update: each zeroes the other's
    mutable bool b_max_ready = false;          // the projection pass has left the largest |B| in slotsO[0]
};
size_t fast_products_bytes(int64_t n, int64_t p) {
    return 4 * admmq_align_up((size_t)n * n * 2) + 2 * admmq_align_up((size_t)n * p * 2) +
           admmq_align_up(admmq_gemm_f16x3_partial_bytes(n, p, n)) + 4 * 256 + 4096;
}
// true when this context asks for the fast products and the shape suits them (whole 256 x 256 tiles, enough of them)
bool fast_wanted(const admmq_ctx *ctx, int64_t n, int64_t p) { return ctx->fast_on && admmq_gemm_f16x3_ok(n, p, n); }
admmq_status fast_setup(admmq_ctx *ctx, int64_t n, int64_t p, FastBufs &fb) {
    const admmq_factor &f = ctx->fac;
    char *q = nullptr, *o = nullptr, *sl = nullptr;
    ADMMQ_TRY(take(ctx, q, 4 * admmq_align_up((size_t)n * n * 2)));
    ADMMQ_TRY(take(ctx, o, 2 * admmq_align_up((size_t)n * p * 2)));
    if (admmq_gemm_f16x3_partial_bytes(n, p, n) > 0)
        ADMMQ_TRY(take(ctx, fb.partial, admmq_gemm_f16x3_partial_bytes(n, p, n) / 4));
    ADMMQ_TRY(take(ctx, sl, 4 * 256));
    ADMMQ_TRY(admmq_k_fill_bytes(ctx, sl, 0, 4 * 256));
    const size_t qs = admmq_align_up((size_t)n * n * 2), os = admmq_align_up((size_t)n * p * 2);
    fb.Q1 = q; fb.Q2 = q + qs; fb.Qt1 = q + 2 * qs; fb.Qt2 = q + 3 * qs;
    fb.O1 = o; fb.O2 = o + os;
    fb.slotsQ = sl; fb.slotsQt = sl + 256; fb.slotsO[0] = sl + 512; fb.slotsO[1] = sl + 768;
    ADMMQ_TRY(admmq_k_split_f16(ctx, f.Q, n, n, n, fb.Q1, fb.Q2, fb.slotsQ, nullptr));
    ADMMQ_TRY(admmq_k_split_f16(ctx, f.Qt, n, n, n, fb.Qt1, fb.Qt2, fb.slotsQt, nullptr));
    return ADMMQ_OK;
}

admmq_status mid_factors_take(admmq_ctx *ctx, int64_t n, int32_t T, MidFactors &mf) {
    if (ctx->fac.band) {
        mf.stride = admmq_band_factor_doubles(n, 1);
        ADMMQ_TRY(take(ctx, mf.a, mf.stride * (size_t)T));
        return ADMMQ_OK;
    }
    mf.stride = (size_t)n;
    ADMMQ_TRY(take(ctx, mf.a, (size_t)T * n));
    ADMMQ_TRY(take(ctx, mf.b, (size_t)T * n));
    return ADMMQ_OK;
}
admmq_status mid_factors_compute(admmq_ctx *ctx, int64_t n, const double *rhos_dev, int32_t T, const MidFactors &mf) {
    const admmq_factor &f = ctx->fac;
    if (f.band) return admmq_k_band_factor(ctx, f.band, n, rhos_dev, T, mf.a);
    return admmq_k_tridiag_factor(ctx, f.ta, f.tb, n, rhos_dev, T, mf.a, mf.b);
}
// ADMMQ_FUSE_PROJECTION=0 keeps the projection pass a launch of its own in every iteration (read at every call)
bool fuse_projection_enabled() {
    const char *e = getenv("ADMMQ_FUSE_PROJECTION");
    return !(e && atoi(e) == 0);
}

// S = (M + rho_t I)^-1 M Y; carries: the tridiagonal solve's per-tile checkpoints
admmq_status mid_apply(admmq_ctx *ctx, const MidFactors &mf, int t, int64_t n, int64_t p, const float *Y, double *carries,
                       float *S, unsigned *amax_out) {
    const admmq_factor &f = ctx->fac;
    if (f.band) return admmq_k_band_apply(ctx, mf.a + (size_t)t * mf.stride, n, p, Y, S, amax_out);
    return admmq_k_tridiag_apply(ctx, f.ta, f.tb, mf.a + (size_t)t * mf.stride, mf.b + (size_t)t * mf.stride, n, p, Y,
                                 carries, S, amax_out);
}

// W = B + Q (M + rho I)^{-1} M (C0 - Q^T B)   (eq. 7 rewritten around B = D - V/rho; Hs = Q M Q^T)
// F: n p + p doubles of scratch: the solve's fp32 result [n][p] in front, its per-tile checkpoints behind
// With `proj` (fp32 products only) the second product applies eqs. 8-10 to its result in registers and writes
// B^(t+1) to W, which may then be B itself; proj->V is updated in place.
admmq_status w_update_core(admmq_ctx *ctx, const float *C0, const float *B, int64_t n, int64_t p, const MidFactors &mf,
                           int t, float *Y, double *F, float *W, const FastBufs *fb = nullptr,
                           const gemm_proj_args *proj = nullptr) {
    const admmq_factor &f = ctx->fac;
    if (fb && proj) return ADMMQ_ERR_PARAM;
    if (fb) {
        // the time of splitting the state operand is booked with its product
        int sp = admmq_prof_begin(ctx, ADMMQ_TAG_GEMM);
        void *sb = fb->slotsO[0], *ss = fb->slotsO[1];
        ADMMQ_TRY(admmq_k_split_f16(ctx, B, n, p, p, fb->O1, fb->O2, sb, ss, fb->b_max_ready));
        fb->b_max_ready = false;
        ADMMQ_TRY(admmq_gemm_f16x3(ctx, fb->Q1, fb->Q2, fb->slotsQ, fb->O1, fb->O2, sb, n, p, n, -1.f, 1.f, C0, p, Y, p,
                                   fb->partial));
        admmq_prof_end(ctx, sp);
        float *S = (float *)F;
        double *carries = F + ((size_t)n * p + 1) / 2;
        sp = admmq_prof_begin(ctx, ADMMQ_TAG_TRIDIAG);
        ADMMQ_TRY(mid_apply(ctx, mf, t, n, p, Y, carries, S, (unsigned *)ss));
        admmq_prof_end(ctx, sp);
        sp = admmq_prof_begin(ctx, ADMMQ_TAG_GEMM);
        // (the solve has left the largest |S| in its slot; the second split zeroes the first one's slot again: the
        // next W-update, or the projection pass before it, starts where this one did)
        ADMMQ_TRY(admmq_k_split_f16(ctx, S, n, p, p, fb->O1, fb->O2, ss, sb, true));
        ADMMQ_TRY(admmq_gemm_f16x3(ctx, fb->Qt1, fb->Qt2, fb->slotsQt, fb->O1, fb->O2, ss, n, p, n, 1.f, 1.f, B, p, W, p,
                                   fb->partial));
        admmq_prof_end(ctx, sp);
        return ADMMQ_OK;
    }
    gemm_tn_args g1 = {};
    g1.A = f.Q; g1.lda = n; g1.B = B; g1.ldb = p; g1.M = n; g1.N = p; g1.K = n;
    g1.alpha = -1.f; g1.beta = 1.f; g1.Z = C0; g1.ldz = p; g1.out = Y; g1.ldo = p; g1.split_k = 1;
    int sp = admmq_prof_begin(ctx, ADMMQ_TAG_GEMM);
    ADMMQ_TRY(admmq_gemm_tn(ctx, g1));
    admmq_prof_end(ctx, sp);
    float *S = (float *)F;
    double *carries = F + ((size_t)n * p + 1) / 2;
    sp = admmq_prof_begin(ctx, ADMMQ_TAG_TRIDIAG);
    ADMMQ_TRY(mid_apply(ctx, mf, t, n, p, Y, carries, S, nullptr));
    admmq_prof_end(ctx, sp);
    gemm_tn_args g2 = {};
    g2.A = f.Qt; g2.lda = n; g2.B = S; g2.ldb = p; g2.M = n; g2.N = p; g2.K = n;
    g2.alpha = 1.f; g2.beta = 1.f; g2.Z = B; g2.ldz = p; g2.out = W; g2.ldo = p; g2.split_k = 1;
    g2.proj = proj;
    sp = admmq_prof_begin(ctx, proj ? ADMMQ_TAG_GEMM_PROJECT : ADMMQ_TAG_GEMM);
    ADMMQ_TRY(admmq_gemm_tn(ctx, g2));
    admmq_prof_end(ctx, sp);
    return ADMMQ_OK;
}

// J = sum E .* (H E + lambda E); E and tmp are n x p scratch; the scalar lands in dev_out[0]
admmq_status objective_core(admmq_ctx *ctx, const float *H, double lambda, int64_t n, int64_t p, const float *E,
                            float *tmp, double *dev_out) {
    gemm_tn_args g = {};
    g.A = H; g.lda = n; g.B = E; g.ldb = p; g.M = n; g.N = p; g.K = n;
    g.alpha = 1.f; g.beta = (float)lambda; g.Z = E; g.ldz = p; g.out = tmp; g.ldo = p; g.split_k = 1;
    ADMMQ_TRY(admmq_gemm_tn(ctx, g));
    ADMMQ_TRY(admmq_k_fill_bytes(ctx, dev_out, 0, 8));
    ADMMQ_TRY(admmq_k_dot(ctx, E, tmp, n * p, dev_out));
    return ADMMQ_OK;
}

// both objectives of a result: J' = Tr(E^T H' E) and J = Tr(E^T H E) = J' - lambda ||E||_F^2 (the reconstruction
// error ||X E||_F^2 of eq. 2 without the damping term); dev_out: 2 doubles
admmq_status objectives_core(admmq_ctx *ctx, const float *H, double lambda, int64_t n, int64_t p, const float *E,
                             float *tmp, double *dev_out, double *j_damp, double *j_recon) {
    ADMMQ_TRY(objective_core(ctx, H, lambda, n, p, E, tmp, dev_out));
    ADMMQ_TRY(admmq_k_fill_bytes(ctx, dev_out + 1, 0, 8));
    ADMMQ_TRY(admmq_k_dot(ctx, E, E, n * p, dev_out + 1));
    double h[2];
    ADMMQ_TRY(read_back(ctx, h, dev_out, 16));
    *j_damp = h[0];
    *j_recon = h[0] - lambda * h[1];
    return ADMMQ_OK;
}

// One grid-refresh attempt (App. B).  new_sc / new_zr: [n/g][p] scratch; part: 2*blocks doubles scratch.
// On acceptance scales/zeros are overwritten (and inv_scales, when given).  Synchronises the stream.
admmq_status grid_refresh_core(admmq_ctx *ctx, const float *W, const float *V, int64_t n, int64_t p, const float *d,
                               const float *inv_d, int bits, int64_t g, double rho, float *scales, float *zeros,
                               float *inv_scales, float *new_sc, float *new_zr, double *part, int *accepted,
                               double *err_old, double *err_new) {
    const float inv_rho = 1.0f / (float)rho;
    const size_t ng = (size_t)(n / g) * p;
    ADMMQ_TRY(admmq_k_refit_grid(ctx, W, V, n, p, inv_d, inv_rho, bits, g, new_sc, new_zr));
    ADMMQ_TRY(admmq_k_refresh_error(ctx, W, V, n, p, d, inv_d, inv_rho, bits, g, scales, zeros, new_sc, new_zr, part));
    const int nb = admmq_refresh_error_blocks();
    std::vector<double> h((size_t)2 * nb);
    ADMMQ_TRY(read_back(ctx, h.data(), part, h.size() * 8));
    double eo = 0.0, en = 0.0;
    for (int b = 0; b < nb; ++b) {          // fixed order: the decision is reproducible
        eo += h[2 * b];
        en += h[2 * b + 1];
    }
    *accepted = en <= eo ? 1 : 0;
    if (err_old) *err_old = eo;
    if (err_new) *err_new = en;
    if (*accepted) {
        ADMMQ_HIP(hipMemcpyAsync(scales, new_sc, ng * 4, hipMemcpyDeviceToDevice, ctx->stream));
        ADMMQ_HIP(hipMemcpyAsync(zeros, new_zr, ng * 4, hipMemcpyDeviceToDevice, ctx->stream));
        if (inv_scales) ADMMQ_TRY(admmq_k_recip(ctx, scales, inv_scales, (int64_t)ng));
    }
    return ADMMQ_OK;
}

struct LsPlan {
    int rounds, batches, pairs;
};

LsPlan ls_plan(int64_t n, int rounds, int batches, int pairs) {
    LsPlan q;
    q.rounds = rounds;
    q.batches = batches > 0 ? batches : (int)((n + 1) / 2);
    q.pairs = pairs > 0 ? pairs : 64;
    return q;
}

// the search itself; arena must already be reserved for ls_transient_bytes
admmq_status local_search_core(admmq_ctx *ctx, const float *H, double lambda, const float *W0, int64_t n, int64_t p,
                               int64_t ldw, int bits, int64_t g, const float *scales, const float *zeros,
                               uint8_t *codes, LsPlan plan, uint64_t seed, const int32_t *explicit_pairs,
                               int32_t *moves_out, double *drop_out) {
    if (moves_out) *moves_out = 0;
    if (drop_out) *drop_out = 0.0;
    if (plan.rounds <= 0 || n < 2) return ADMMQ_OK;
    const size_t total = (size_t)plan.rounds * plan.batches * plan.pairs;
    float *E = nullptr, *G = nullptr, *partial = nullptr, *partial_b = nullptr, *pend_d = nullptr;
    int32_t *pairs = nullptr, *choice = nullptr, *pend_idx = nullptr;
    uint8_t *mv_a = nullptr, *mv_b = nullptr;
    float *hcol = nullptr;
    const int K = admmq_ls_defer();
    double *scal = nullptr;
    ADMMQ_TRY(take(ctx, E, (size_t)n * p));
    ADMMQ_TRY(take(ctx, G, (size_t)n * p));
    ADMMQ_TRY(take(ctx, pairs, total * 2));
    ADMMQ_TRY(take(ctx, partial, (size_t)plan.pairs * admmq_ls_chunks(p)));
    ADMMQ_TRY(take(ctx, partial_b, (size_t)plan.pairs * admmq_ls_chunks(p)));
    ADMMQ_TRY(take(ctx, pend_d, (size_t)2 * K * p));
    ADMMQ_TRY(take(ctx, mv_a, (size_t)plan.pairs * p));
    ADMMQ_TRY(take(ctx, mv_b, (size_t)plan.pairs * p));
    ADMMQ_TRY(take(ctx, hcol, (size_t)2 * K * n));
    ADMMQ_TRY(take(ctx, pend_idx, (size_t)2 * K));
    // coupling entries H'[own row of the next batch][candidate row of this batch], gathered one launch ahead
    const int FP = admmq_ls_fast_pairs();
    float *exs_a = nullptr, *exs_b = nullptr;
    ADMMQ_TRY(take(ctx, exs_a, (size_t)FP * FP * 4));
    ADMMQ_TRY(take(ctx, exs_b, (size_t)FP * FP * 4));
    float *exs[2] = {exs_a, exs_b};
    const bool ahead = plan.pairs <= FP;
    ADMMQ_TRY(take(ctx, choice, 4));
    ADMMQ_TRY(take(ctx, scal, 4));      // scal[0] = drop (double); as ints: scal[1] -> moves, scal[2] -> commit, abort
    int *dev_moves = (int *)(scal + 1);
    int *dev_commit = (int *)(scal + 2), *dev_abort = dev_commit + 1;
    // groups of K batches as single launches (blocks exchange their partial sums through memory) where the shape
    // allows; ADMMQ_LS_PERSISTENT=0 keeps one launch per batch; ADMMQ_LS_SPIN_TICKS sets the bound of a wait in
    // ticks of the device's wall clock (negative: every block gives up at its first wait - exercises the fall-back)
    const int group_pp = admmq_ls_group_pairs_per_thread(ctx, p, plan.pairs);
    bool grouped = group_pp > 0;
    {
        const char *e = getenv("ADMMQ_LS_PERSISTENT");
        if (e && atoi(e) == 0) grouped = false;
    }
    long long spin_ticks = 0;
    unsigned long long *xch = nullptr;
    unsigned *fin = nullptr;
    float *couple = nullptr;
    const int span = plan.batches < LS_COUPLE_SPAN ? plan.batches : LS_COUPLE_SPAN;
    if (grouped) {
        ADMMQ_TRY(take(ctx, couple, admmq_ls_couple_floats(span)));
        int khz = 0;
        if (hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, ctx->device) != hipSuccess || khz <= 0) {
            (void)hipGetLastError();
            khz = 100000;
        }
        spin_ticks = 20ll * khz;                                            // 20 ms
        const char *e = getenv("ADMMQ_LS_SPIN_TICKS");
        if (e) spin_ticks = atoll(e);
        ADMMQ_TRY(take(ctx, xch, admmq_ls_group_xch_words(p)));
        ADMMQ_TRY(take(ctx, fin, (size_t)admmq_ls_group_max_blocks(p)));
        ADMMQ_TRY(admmq_k_fill_bytes(ctx, xch, 0, admmq_ls_group_xch_words(p) * 8));
        ADMMQ_TRY(admmq_k_fill_bytes(ctx, fin, 0, (size_t)admmq_ls_group_max_blocks(p) * 4));
    }
    ctx->ls_fallback_groups = 0;

    std::vector<int32_t> hp;
    const int32_t *src = explicit_pairs;
    if (!src) {
        hp.resize(total * 2);
        size_t q = 0;
        for (int r = 0; r < plan.rounds; ++r)
            for (int m = 0; m < plan.batches; ++m)
                for (int s = 0; s < plan.pairs; ++s, ++q) admmq_sample_pair(seed, r, m, s, n, &hp[2 * q], &hp[2 * q + 1]);
        src = hp.data();
    } else {
        for (size_t q = 0; q < total; ++q) {
            const int32_t a = src[2 * q], b = src[2 * q + 1];
            if (a < 0 || b < 0 || a >= n || b >= n || a == b) return ADMMQ_ERR_PARAM;
        }
    }
    ADMMQ_HIP(hipMemcpyAsync(pairs, src, total * 2 * sizeof(int32_t), hipMemcpyHostToDevice, ctx->stream));
    ADMMQ_HIP(hipStreamSynchronize(ctx->stream));   // hp may go out of scope only after the copy

    // G = H'(W0 - Wq)
    ADMMQ_TRY(admmq_k_quant_error(ctx, W0, ldw, codes, n, p, g, scales, zeros, bits, 1, E));
    gemm_tn_args gg = {};
    gg.A = H; gg.lda = n; gg.B = E; gg.ldb = p; gg.M = n; gg.N = p; gg.K = n;
    gg.alpha = 1.f; gg.beta = (float)lambda; gg.Z = E; gg.ldz = p; gg.out = G; gg.ldo = p; gg.split_k = 1;
    ADMMQ_TRY(admmq_gemm_tn(ctx, gg));
    ADMMQ_TRY(admmq_k_fill_bytes(ctx, scal, 0, 32));
    ADMMQ_TRY(admmq_k_fill_bytes(ctx, hcol, 0, (size_t)2 * K * n * 4));     // finite before any slot is filled
    ADMMQ_TRY(admmq_k_fill_bytes(ctx, pend_d, 0, (size_t)2 * K * p * 4));

    int moves_total = 0;
    float *part[2] = {partial, partial_b};
    uint8_t *mv[2] = {mv_a, mv_b};
    auto batch_pairs = [&](int r, int b) { return pairs + ((size_t)r * plan.batches + b) * plan.pairs * 2; };
    // The batches of a round go in groups of K.  A group starts from codes and a gradient that hold every earlier
    // move, evaluates its batches one after the other against the moves of the batches before (kept as pending
    // slots), and ends with one pass over G (the flush).
    // One launch per batch: step s of a group evaluates its batch s (s < cnt) and plans its batch s-1 (s > 0).
    auto run_stepwise = [&](int r, int b0) -> admmq_status {
        for (int gb = b0; gb < plan.batches; gb += K) {
            const int cnt = plan.batches - gb < K ? plan.batches - gb : K;
            for (int s = 0; s <= cnt; ++s) {
                const int32_t *cur = s < cnt ? batch_pairs(r, gb + s) : nullptr;
                const int32_t *prev = s > 0 ? batch_pairs(r, gb + s - 1) : nullptr;
                const int slot_prev = s > 0 ? s - 1 : 0;
                const int32_t *next = (ahead && s + 1 < cnt) ? batch_pairs(r, gb + s + 1) : nullptr;
                ADMMQ_TRY(admmq_k_ls_step(ctx, H, (float)lambda, G, codes, n, p, bits, g, scales, prev,
                                          s > 0 ? plan.pairs : 0, part[(s + 1) & 1], mv[(s + 1) & 1], slot_prev, cur,
                                          plan.pairs, slot_prev, pend_idx, pend_d, hcol, part[s & 1], mv[s & 1],
                                          choice, dev_moves, scal, next, plan.pairs,
                                          (ahead && s > 0 && cur) ? exs[(s + 1) & 1] : nullptr,
                                          next ? exs[s & 1] : nullptr));
            }
            ADMMQ_TRY(admmq_k_ls_flush(ctx, H, (float)lambda, G, codes, n, p, pend_idx, pend_d, cnt));
        }
        return ADMMQ_OK;
    };
    int groups_launched = 0;       // group kernels issued so far in this call (= value the commit counter should reach)
    for (int r = 0; r < plan.rounds; ++r) {
        const int first_group = groups_launched;
        if (grouped) {
            for (int gb = 0; gb < plan.batches; gb += K) {
                const int cnt = plan.batches - gb < K ? plan.batches - gb : K;
                const unsigned seq0 = 1u + (unsigned)((size_t)r * plan.batches + gb);
                // (LS_COUPLE_SPAN is a multiple of K: a group never straddles two tables)
                const int span0 = gb / LS_COUPLE_SPAN * LS_COUPLE_SPAN;
                if (gb == span0)
                    ADMMQ_TRY(admmq_k_ls_couple(ctx, H, (float)lambda, n, batch_pairs(r, span0), plan.pairs,
                                                plan.batches - span0 < span ? plan.batches - span0 : span, couple));
                ADMMQ_TRY(admmq_k_ls_group(ctx, group_pp, H, (float)lambda, G, codes, n, p, bits, g, scales, batch_pairs(r, gb),
                                           plan.pairs, cnt, seq0, groups_launched, xch, fin, dev_commit, dev_abort,
                                           spin_ticks, pend_idx, pend_d, dev_moves, scal,
                                           couple + (size_t)(gb - span0) * admmq_ls_couple_floats(2)));
                ++groups_launched;
                ADMMQ_TRY(admmq_k_ls_flush(ctx, H, (float)lambda, G, codes, n, p, pend_idx, pend_d, cnt, dev_commit,
                                           groups_launched));
            }
        } else {
            ADMMQ_TRY(run_stepwise(r, 0));
        }
        double host[3];
        ADMMQ_TRY(read_back(ctx, host, scal, 24));
        if (grouped) {
            int committed;
            memcpy(&committed, &host[2], sizeof(int));
            if (committed < groups_launched) {
                // a group gave up waiting: nothing after it has run.  Its batches and the rest of the round go
                // one launch per batch, and so does the rest of the search.
                ctx->ls_fallback_groups += groups_launched - committed;
                grouped = false;
                ADMMQ_TRY(run_stepwise(r, (committed - first_group) * K));
                ADMMQ_TRY(read_back(ctx, host, scal, 24));
            }
        }
        int mvd;
        memcpy(&mvd, &host[1], sizeof(int));
        const bool none = mvd == moves_total;
        moves_total = mvd;
        if (drop_out) *drop_out = host[0];
        if (none) break;
    }
    if (moves_out) *moves_out = moves_total;
    return ADMMQ_OK;
}

}  // namespace

// ---- context -----------------------------------------------------------------------------------
// Scratch of admmq_project_dual_noalloc: part of the library's device image, so every GPU the library runs on holds
// a copy of its own at an address of its own.  In host code the name below is only a handle for
// hipGetSymbolAddress; the address a kernel may use is looked up once per device (with that device current)
// when a context is created on it, and only that address is ever passed on.
static __device__ __align__(256) unsigned char scratch[ADMMQ_NOALLOC_SCRATCH_BYTES];
enum { ADMMQ_MAX_DEVICES = 64 };
static void *fixed_scratch_of_device[ADMMQ_MAX_DEVICES];
static std::mutex fixed_scratch_lock;

static admmq_status fixed_scratch_lookup(int device, void **out) {
    *out = nullptr;
    if (device < 0 || device >= ADMMQ_MAX_DEVICES) return ADMMQ_OK;   // the no-alloc call reports the missing array
    std::lock_guard<std::mutex> hold(fixed_scratch_lock);
    if (!fixed_scratch_of_device[device]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
            (void)hipGetLastError();
            return ADMMQ_ERR_DEVICE;
        }
        fixed_scratch_of_device[device] = ptr;
    }
    *out = fixed_scratch_of_device[device];
    return ADMMQ_OK;
}

extern "C" admmq_status admmq_create(admmq_ctx **out, int device, void *hip_stream) {
    if (!out) return ADMMQ_ERR_NULL;
    *out = nullptr;
    if (device == -1) {
        // validation-only context: every call still checks its arguments, then stops at the device
        admmq_ctx *c = new (std::nothrow) admmq_ctx();
        if (!c) return ADMMQ_ERR_WORKSPACE;
        c->device = -1;
        *out = c;
        return ADMMQ_OK;
    }
    int count = 0;
    if (hipGetDeviceCount(&count) != hipSuccess || device < 0 || device >= count) {
        (void)hipGetLastError();
        return ADMMQ_ERR_DEVICE;
    }
    ADMMQ_HIP(hipSetDevice(device));
    void *fixed = nullptr;
    ADMMQ_TRY(fixed_scratch_lookup(device, &fixed));
    admmq_ctx *c = new (std::nothrow) admmq_ctx();
    if (!c) return ADMMQ_ERR_WORKSPACE;
    c->device = device;
    c->stream = (hipStream_t)hip_stream;
    c->fixed_scratch = fixed;
    *out = c;
    return ADMMQ_OK;
}

extern "C" void admmq_destroy(admmq_ctx *ctx) {
    if (!ctx) return;
    if (ctx->device >= 0) {
        float ms[ADMMQ_TAGS];
        int cnt[ADMMQ_TAGS];
        prof_collect(ctx, ms, cnt);
        (void)hipStreamSynchronize(ctx->stream);
        for (hipStream_t st : ctx->side)
            if (st) {
                (void)hipStreamSynchronize(st);
                (void)hipStreamDestroy(st);
            }
        if (ctx->side_ready) (void)hipEventDestroy(ctx->side_ready);
        for (int i = 0; i < ctx->panel_event_count; ++i) (void)hipEventDestroy(ctx->panel_events[i]);
        free(ctx->panel_events);
        if (ctx->arena && ctx->arena_owned) (void)hipFree(ctx->arena);
    }
    free(ctx->prof.spans);
    delete ctx;
}

extern "C" const char *admmq_status_string(admmq_status s) {
    switch (s) {
        case ADMMQ_OK: return "ok";
        case ADMMQ_ERR_NULL: return "null pointer";
        case ADMMQ_ERR_SHAPE: return "bad shape";
        case ADMMQ_ERR_PARAM: return "bad parameter";
        case ADMMQ_ERR_NOT_FINITE: return "non-finite input";
        case ADMMQ_ERR_ZERO_DIAG: return "non-positive Hessian diagonal";
        case ADMMQ_ERR_WORKSPACE: return "workspace too small or allocation failed";
        case ADMMQ_ERR_STATE: return "no factorisation in the context";
        case ADMMQ_ERR_DEVICE: return "HIP error";
    }
    return "unknown status";
}

extern "C" size_t admmq_workspace_bytes(int64_t n, int64_t p, int32_t T) {
    if (n < 1 || p < 1 || T < 1) return 0;
    const int64_t batches = (n + 1) / 2;
    size_t a = factor_transient_bytes(n);
    // + the per-group arrays of the loop (reciprocal scales, a refreshed grid, both grids of a dual-grid format):
    // at most three [n/g][p] arrays, bounded by one n x p array for any group size of 3 rows or more
    size_t b = admm_transient_bytes(n, p, T) + admmq_align_up((size_t)n * p * 4) + (1u << 20);
    size_t c = ls_transient_bytes(n, p, (int64_t)5 * batches * 64, 64) + 2 * admmq_align_up((size_t)n * p * 4);
    size_t m = a > b ? a : b;
    m = m > c ? m : c;
    return factor_persist_bytes(n) + m + 65536;
}

extern "C" admmq_status admmq_set_workspace(admmq_ctx *ctx, void *dev_ptr, size_t bytes) {
    if (!ctx || !dev_ptr) return ADMMQ_ERR_NULL;
    if (((uintptr_t)dev_ptr & 255) != 0) return ADMMQ_ERR_WORKSPACE;
    if (ctx->device < 0) return ADMMQ_ERR_DEVICE;
    ADMMQ_HIP(hipStreamSynchronize(ctx->stream));
    if (ctx->arena && ctx->arena_owned) ADMMQ_HIP(hipFree(ctx->arena));
    ctx->arena = (char *)dev_ptr;
    ctx->arena_bytes = bytes;
    ctx->arena_owned = false;
    ctx->persist_top = ctx->top = 0;
    ctx->fac = admmq_factor();
    return ADMMQ_OK;
}

extern "C" admmq_status admmq_set_fast_products(admmq_ctx *ctx, int32_t on) {
    if (!ctx) return ADMMQ_ERR_NULL;
    if (on != 0 && on != 1) return ADMMQ_ERR_PARAM;
    ctx->fast_on = on != 0;
    return ADMMQ_OK;
}

extern "C" size_t admmq_fast_products_bytes(int64_t n, int64_t p) {
    if (n < 1 || p < 1 || !admmq_gemm_f16x3_ok(n, p, n)) return 0;
    return fast_products_bytes(n, p);
}

// Measurement aid: a plain device-to-device copy by a kernel of this library.
extern "C" admmq_status admmq_stream_copy(admmq_ctx *ctx, void *dst, const void *src, size_t bytes) {
    if (!ctx || !dst || !src) return ADMMQ_ERR_NULL;
    if (bytes % 16 != 0 || (((uintptr_t)dst | (uintptr_t)src) & 15) != 0) return ADMMQ_ERR_SHAPE;
    if (ctx->device < 0) return ADMMQ_ERR_DEVICE;
    ADMMQ_HIP(hipSetDevice(ctx->device));
    return admmq_k_stream_copy(ctx, dst, src, bytes);
}

// ---- Hessian -----------------------------------------------------------------------------------
namespace {
// Bytes the partial sums of the token slices may take: whatever it needs in an arena the library grows itself,
// what is left beside a kept factorisation in a caller's workspace (fewer slices then; one always has to fit).
size_t hessian_slice_room(const admmq_ctx *ctx) {
    if (ctx->arena_owned || !ctx->arena) return ~(size_t)0;
    const size_t used = ctx->persist_top + 8192;
    return ctx->arena_bytes > used ? ctx->arena_bytes - used : 0;
}
}  // namespace

extern "C" admmq_status admmq_accumulate_hessian(admmq_ctx *ctx, float *H, int64_t n, const void *X,
                                                 admmq_dtype xdt, int64_t rows, int64_t ldx, uint64_t *n_samples) {
    if (!ctx || !H || !X) return ADMMQ_ERR_NULL;
    if (n < 1 || rows < 0 || ldx < n || n > (1 << 20)) return ADMMQ_ERR_SHAPE;
    if (xdt != ADMMQ_F32 && xdt != ADMMQ_BF16) return ADMMQ_ERR_PARAM;
    if (rows == 0) return ADMMQ_OK;
    if (ctx->device < 0) return ADMMQ_ERR_DEVICE;
    ADMMQ_HIP(hipSetDevice(ctx->device));
    // bf16 activations in whole 256-channel tiles: the bf16 matrix cores (products exact, fp32 accumulation)
    static int bf16_cores = -1;
    if (bf16_cores < 0) {
        const char *e = getenv("ADMMQ_HESSIAN_BF16");
        bf16_cores = e ? atoi(e) : 1;
    }
    if (xdt == ADMMQ_BF16 && bf16_cores && admmq_hessian_bf16_ok(X, n, ldx, rows)) {
        const int64_t k_main = admmq_hessian_bf16_main_rows(rows), k_tail = rows - k_main;
        const int64_t tm = n / 256, tiles = tm * (tm + 1) / 2;
        const size_t slice = (size_t)n * n;
        // Slices of the token axis: each XCD takes an eighth of the (slice, tile) list and runs it 32 blocks at a
        // time; more slices fill the last round better, fewer leave less partial-sum traffic (written and read
        // once, lower triangle only).  Both in seconds, from round numbers for this chip.
        int64_t split = 1;
        double best = 1e300;
        const size_t room = hessian_slice_room(ctx);
        const size_t tail_slice = k_tail > 0 ? 1 : 0;
        for (int64_t sp = 1; sp <= 64 && sp * 256 <= k_main + 255; ++sp) {
            if (sp > 1 && (sp * slice * 4 > ((size_t)8 << 30) ||
                           (sp + tail_slice) * admmq_align_up(slice * 4) + 4096 > room))
                break;
            const int64_t per_xcd = (tiles * sp + 7) / 8, rounds = (per_xcd + 31) / 32;
            const double t_mma = (double)rounds * (double)((k_main + sp - 1) / sp) * 131072.0 / 4.0e12;
            const double t_sum = (double)sp * (double)slice * 4.0 / 4.0e12;
            if (t_mma + t_sum < best) {
                best = t_mma + t_sum;
                split = sp;
            }
        }
        const int64_t slices = split + (k_tail > 0 ? 1 : 0);
        admmq_arena_reset_transient(ctx);
        ADMMQ_TRY(admmq_arena_reserve(ctx, (size_t)slices * admmq_align_up(slice * 4) + 4096));
        float *P = nullptr;
        ADMMQ_TRY(take(ctx, P, (size_t)slices * slice));
        ADMMQ_TRY(admmq_hessian_bf16(ctx, X, ldx, k_main, n, P, (int)split, (int64_t)slice));
        if (k_tail > 0) {
            // the last tokens (fewer than a stage) through the fp32 product, as one more slice
            gemm_tn_args g = {};
            g.A = g.B = (const unsigned short *)X + k_main * ldx;
            g.lda = g.ldb = ldx;
            g.a_bf16 = g.b_bf16 = 1;
            g.M = n; g.N = n; g.K = k_tail; g.alpha = 1.f; g.beta = 0.f; g.Z = nullptr;
            g.out = P + (size_t)split * slice; g.ldo = n; g.lower_only = 1; g.split_k = 1;
            g.slice_stride = (int64_t)slice;
            ADMMQ_TRY(admmq_gemm_tn(ctx, g));
        }
        ADMMQ_TRY(admmq_sym_reduce(ctx, H, n, P, (int)slices, (int64_t)slice, 1));
        if (n_samples) *n_samples += (uint64_t)rows;
        admmq_arena_reset_transient(ctx);
        return ADMMQ_OK;
    }
    // split the token axis so that the triangular tile set fills the chip a few times over
    const int64_t t256 = (n + 255) / 256, t128 = (n + 127) / 128, t64 = (n + 63) / 64;
    int64_t tiles = t256 * (t256 + 1) / 2;
    if (tiles * 8 < 200) tiles = t128 * (t128 + 1) / 2;
    if (tiles * 8 < 128) tiles = t64 * (t64 + 1) / 2;
    // one 256 x 256 tile block occupies a CU (128 KB of LDS), so blocks run in rounds of 256: pick the split
    // (at most 64 slices, at least 256 rows each) whose last round is fullest
    const int64_t max_by_rows = rows / 256 > 0 ? rows / 256 : 1;
    int64_t split = 1;
    double best_fill = 0.0;
    for (int64_t s = 1; s <= 64 && s <= max_by_rows; ++s) {
        const int64_t blocks = tiles * s;
        if (blocks < 256 && s < 64 && s < max_by_rows) continue;      // not even one full round yet
        const double fill = (double)blocks / (double)(((blocks + 255) / 256) * 256);
        if (fill > best_fill + 1e-9) {
            best_fill = fill;
            split = s;
        }
    }
    // the partial slices must fit the arena: shrink the split for very large n
    const size_t slice = (size_t)n * n;
    while (split > 1 && (split * slice * 4 > ((size_t)8 << 30) ||
                         (size_t)split * admmq_align_up(slice * 4) + 4096 > hessian_slice_room(ctx)))
        --split;
    admmq_arena_reset_transient(ctx);
    ADMMQ_TRY(admmq_arena_reserve(ctx, (size_t)split * admmq_align_up(slice * 4) + 4096));
    float *P = nullptr;
    ADMMQ_TRY(take(ctx, P, (size_t)split * slice));
    gemm_tn_args g = {};
    g.A = X; g.B = X; g.lda = ldx; g.ldb = ldx;
    g.a_bf16 = g.b_bf16 = (xdt == ADMMQ_BF16);
    g.M = n; g.N = n; g.K = rows; g.alpha = 1.f; g.beta = 0.f; g.Z = nullptr;
    g.out = P; g.ldo = n; g.lower_only = 1; g.split_k = (int)split; g.slice_stride = (int64_t)slice;
    ADMMQ_TRY(admmq_gemm_tn(ctx, g));
    ADMMQ_TRY(admmq_sym_reduce(ctx, H, n, P, (int)split, (int64_t)slice, 1));
    if (n_samples) *n_samples += (uint64_t)rows;
    admmq_arena_reset_transient(ctx);
    return ADMMQ_OK;
}

// ---- single steps --------------------------------------------------------------------------------
extern "C" admmq_status admmq_grid_init(admmq_ctx *ctx, const float *W0, int64_t n, int64_t p, int64_t ldw,
                                        int32_t bits, int32_t group_size, float *scales, float *zeros) {
    if (!ctx || !scales || !zeros) return ADMMQ_ERR_NULL;
    ADMMQ_TRY(check_layer_args(W0, W0, n, p, ldw, bits, group_size));
    if (ctx->device < 0) return ADMMQ_ERR_DEVICE;
    ADMMQ_HIP(hipSetDevice(ctx->device));
    const int64_t g = group_size > 0 ? group_size : n;
    return admmq_k_grid_init(ctx, W0, n, p, ldw, bits, g, scales, zeros);
}

extern "C" admmq_status admmq_grid_fit(admmq_ctx *ctx, const float *W0, int64_t n, int64_t p, int64_t ldw,
                                       int32_t bits, int32_t group_size, int32_t symmetric, int32_t clip_points,
                                       double clip_shrink, float *scales, float *zeros) {
    if (!ctx || !scales || !zeros) return ADMMQ_ERR_NULL;
    ADMMQ_TRY(check_layer_args(W0, W0, n, p, ldw, bits, group_size));
    if (clip_points < 0 || clip_points > 100000 || !(clip_shrink >= 0.0) || !(clip_shrink < 1.0)) return ADMMQ_ERR_PARAM;
    if (ctx->device < 0) return ADMMQ_ERR_DEVICE;
    ADMMQ_HIP(hipSetDevice(ctx->device));
    const int64_t g = group_size > 0 ? group_size : n;
    return admmq_k_grid_fit(ctx, W0, n, p, ldw, bits, g, symmetric != 0, clip_points, clip_shrink, scales, zeros);
}

extern "C" admmq_status admmq_factorize(admmq_ctx *ctx, const float *H, int64_t n, double damp,
                                        int32_t precondition, float *d_out, double *lambda_out) {
    if (!ctx || !H) return ADMMQ_ERR_NULL;
    if (n < 1 || n > (1 << 20)) return ADMMQ_ERR_SHAPE;
    if (!(damp >= 0.0) || !isfinite(damp)) return ADMMQ_ERR_PARAM;
    if (ctx->device < 0) return ADMMQ_ERR_DEVICE;
    ADMMQ_HIP(hipSetDevice(ctx->device));
    ADMMQ_TRY(do_factorize(ctx, H, n, damp, precondition, lambda_out));
    if (d_out)
        ADMMQ_HIP(hipMemcpyAsync(d_out, ctx->fac.d, (size_t)n * 4, hipMemcpyDeviceToDevice, ctx->stream));
    return ADMMQ_OK;
}

extern "C" admmq_status admmq_w_update(admmq_ctx *ctx, const float *Ws, const float *D, const float *V, int64_t n,
                                       int64_t p, double rho, float *W_out) {
    if (!ctx || !Ws || !D || !V || !W_out) return ADMMQ_ERR_NULL;
    if (n < 1 || p < 1) return ADMMQ_ERR_SHAPE;
    if (!(rho > 0.0) || !isfinite(rho)) return ADMMQ_ERR_PARAM;
    if (!ctx->fac.valid || ctx->fac.n != n) return ADMMQ_ERR_STATE;
    if (ctx->device < 0) return ADMMQ_ERR_DEVICE;
    ADMMQ_HIP(hipSetDevice(ctx->device));
    admmq_arena_reset_transient(ctx);
    const size_t np = (size_t)n * p;
    const bool fast = fast_wanted(ctx, n, p);
    ADMMQ_TRY(admmq_arena_reserve(ctx, 3 * admmq_align_up(np * 4) + admmq_align_up((np + (size_t)p) * 8) +
                                           mid_factor_bytes(n, 1) + admmq_align_up((size_t)n * 8) + 8192 +
                                           (fast ? fast_products_bytes(n, p) : 0)));
    float *B = nullptr, *C0 = nullptr, *Y = nullptr;
    double *F = nullptr, *rho_dev = nullptr;
    MidFactors mf;
    ADMMQ_TRY(take(ctx, B, np));
    ADMMQ_TRY(take(ctx, C0, np));
    ADMMQ_TRY(take(ctx, Y, np));
    ADMMQ_TRY(take(ctx, F, np + (size_t)p));
    ADMMQ_TRY(mid_factors_take(ctx, n, 1, mf));
    ADMMQ_TRY(take(ctx, rho_dev, 1));
    const admmq_factor &f = ctx->fac;
    ADMMQ_HIP(hipMemcpyAsync(rho_dev, &rho, 8, hipMemcpyHostToDevice, ctx->stream));
    ADMMQ_HIP(hipStreamSynchronize(ctx->stream));
    ADMMQ_TRY(mid_factors_compute(ctx, n, rho_dev, 1, mf));
    gemm_tn_args g0 = {};
    g0.A = f.Q; g0.lda = n; g0.B = Ws; g0.ldb = p; g0.M = n; g0.N = p; g0.K = n;
    g0.alpha = 1.f; g0.Z = nullptr; g0.out = C0; g0.ldo = p; g0.split_k = 1;
    ADMMQ_TRY(admmq_gemm_tn(ctx, g0));
    const float inv_rho = 1.0f / (float)rho;
    ADMMQ_TRY(admmq_k_form_b(ctx, D, V, inv_rho, (int64_t)np, B));
    FastBufs fbufs;
    if (fast) ADMMQ_TRY(fast_setup(ctx, n, p, fbufs));
    ADMMQ_TRY(w_update_core(ctx, C0, B, n, p, mf, 0, Y, F, W_out, fast ? &fbufs : nullptr));
    admmq_arena_reset_transient(ctx);
    return ADMMQ_OK;
}

extern "C" admmq_status admmq_project_dual(admmq_ctx *ctx, const float *W, float *V, int64_t n, int64_t p,
                                           const float *d, int32_t bits, int32_t group_size, const float *scales,
                                           const float *zeros, double rho, double rho_next, uint8_t *codes,
                                           float *B_out, double *res_sq) {
    if (!ctx || !W || !V || !d || !scales || !zeros || !B_out) return ADMMQ_ERR_NULL;
    ADMMQ_TRY(check_layer_args(W, W, n, p, p, bits, group_size));
    if (!(rho > 0.0) || !(rho_next > 0.0) || !isfinite(rho) || !isfinite(rho_next)) return ADMMQ_ERR_PARAM;
    if (ctx->device < 0) return ADMMQ_ERR_DEVICE;
    ADMMQ_HIP(hipSetDevice(ctx->device));
    const int64_t g = group_size > 0 ? group_size : n;
    const size_t ng = (size_t)(n / g) * p;
    admmq_arena_reset_transient(ctx);
    ADMMQ_TRY(admmq_arena_reserve(ctx, admmq_align_up(ng * 4) + admmq_align_up((size_t)n * 4) + 8192));
    float *inv_scales = nullptr, *inv_d = nullptr;
    double *dev_res = nullptr;
    ADMMQ_TRY(take(ctx, inv_scales, ng));
    ADMMQ_TRY(take(ctx, inv_d, (size_t)n));
    ADMMQ_TRY(take(ctx, dev_res, 2));
    ADMMQ_TRY(admmq_k_recip(ctx, scales, inv_scales, (int64_t)ng));
    ADMMQ_TRY(admmq_k_recip(ctx, d, inv_d, n));
    ADMMQ_TRY(admmq_k_fill_bytes(ctx, dev_res, 0, 16));
    const float rf = (float)rho;
    ADMMQ_TRY(admmq_k_project_dual(ctx, W, V, n, p, d, inv_d, bits, g, scales, inv_scales, zeros, rf, 1.0f / rf,
                                   1.0f / (float)rho_next, codes, 0, B_out, res_sq ? dev_res : nullptr, nullptr, p));
    if (res_sq) ADMMQ_TRY(read_back(ctx, res_sq, dev_res, 8));
    admmq_arena_reset_transient(ctx);
    return ADMMQ_OK;
}

// The same pass for callers that cannot allocate: reciprocals in the library's fixed per-GPU array, the residual
// summed straight into the caller's device scalar (cleared by a kernel), no arena, no read-back, no synchronisation.
extern "C" admmq_status admmq_project_dual_noalloc(admmq_ctx *ctx, const float *W, float *V, int64_t n, int64_t p,
                                                   const float *d, int32_t bits, int32_t group_size,
                                                   const float *scales, const float *zeros, double rho,
                                                   double rho_next, uint8_t *codes, float *B_out, double *res_sq) {
    if (!ctx || !W || !V || !d || !scales || !zeros || !B_out) return ADMMQ_ERR_NULL;
    ADMMQ_TRY(check_layer_args(W, W, n, p, p, bits, group_size));
    if (!(rho > 0.0) || !(rho_next > 0.0) || !isfinite(rho) || !isfinite(rho_next)) return ADMMQ_ERR_PARAM;
    if (res_sq && ((uintptr_t)res_sq & 7) != 0) return ADMMQ_ERR_PARAM;
    const int64_t g = group_size > 0 ? group_size : n;
    const size_t ng = (size_t)(n / g) * p;
    const size_t off_scales = admmq_align_up((size_t)n * 4);
    if (off_scales + admmq_align_up(ng * 4) > (size_t)ADMMQ_NOALLOC_SCRATCH_BYTES) return ADMMQ_ERR_WORKSPACE;
    if (ctx->device < 0) return ADMMQ_ERR_DEVICE;
    if (!ctx->fixed_scratch) return ADMMQ_ERR_DEVICE;
    ADMMQ_HIP(hipSetDevice(ctx->device));
    float *inv_d = (float *)ctx->fixed_scratch;
    float *inv_scales = (float *)((char *)ctx->fixed_scratch + off_scales);
    ADMMQ_TRY(admmq_k_recip(ctx, scales, inv_scales, (int64_t)ng));
    ADMMQ_TRY(admmq_k_recip(ctx, d, inv_d, n));
    if (res_sq) ADMMQ_TRY(admmq_k_fill_bytes(ctx, res_sq, 0, 8));
    const float rf = (float)rho;
    return admmq_k_project_dual(ctx, W, V, n, p, d, inv_d, bits, g, scales, inv_scales, zeros, rf, 1.0f / rf,
                                1.0f / (float)rho_next, codes, 0, B_out, res_sq, nullptr, p);
}

extern "C" admmq_status admmq_grid_refresh(admmq_ctx *ctx, const float *W, const float *V, int64_t n, int64_t p,
                                           const float *d, int32_t bits, int32_t group_size, double rho,
                                           float *scales, float *zeros, int32_t *accepted, double *err_old,
                                           double *err_new) {
    if (!ctx || !W || !V || !d || !scales || !zeros || !accepted) return ADMMQ_ERR_NULL;
    ADMMQ_TRY(check_layer_args(W, W, n, p, p, bits, group_size));
    if (!(rho > 0.0) || !isfinite(rho)) return ADMMQ_ERR_PARAM;
    if (ctx->device < 0) return ADMMQ_ERR_DEVICE;
    ADMMQ_HIP(hipSetDevice(ctx->device));
    const int64_t g = group_size > 0 ? group_size : n;
    const size_t ng = (size_t)(n / g) * p;
    admmq_arena_reset_transient(ctx);
    ADMMQ_TRY(admmq_arena_reserve(ctx, 2 * admmq_align_up(ng * 4) + admmq_align_up((size_t)n * 4) +
                                           admmq_align_up((size_t)2 * admmq_refresh_error_blocks() * 8) + 8192));
    float *new_sc = nullptr, *new_zr = nullptr, *inv_d = nullptr;
    double *part = nullptr;
    ADMMQ_TRY(take(ctx, new_sc, ng));
    ADMMQ_TRY(take(ctx, new_zr, ng));
    ADMMQ_TRY(take(ctx, inv_d, (size_t)n));
    ADMMQ_TRY(take(ctx, part, (size_t)2 * admmq_refresh_error_blocks()));
    ADMMQ_TRY(admmq_k_recip(ctx, d, inv_d, n));
    int acc = 0;
    ADMMQ_TRY(admmq_guarded([&] {
        return grid_refresh_core(ctx, W, V, n, p, d, inv_d, bits, g, rho, scales, zeros, nullptr, new_sc, new_zr, part,
                                 &acc, err_old, err_new);
    }));
    *accepted = acc;
    ADMMQ_HIP(hipStreamSynchronize(ctx->stream));
    admmq_arena_reset_transient(ctx);
    return ADMMQ_OK;
}

extern "C" admmq_status admmq_objective(admmq_ctx *ctx, const float *H, const float *W0, int64_t n, int64_t p,
                                        int64_t ldw, int32_t group_size, const float *scales, const float *zeros,
                                        const uint8_t *codes, double damp, double *j_out) {
    if (!ctx || !scales || !zeros || !codes || !j_out) return ADMMQ_ERR_NULL;
    ADMMQ_TRY(check_layer_args(H, W0, n, p, ldw, 8, group_size));
    if (!(damp >= 0.0)) return ADMMQ_ERR_PARAM;
    if (ctx->device < 0) return ADMMQ_ERR_DEVICE;
    ADMMQ_HIP(hipSetDevice(ctx->device));
    const int64_t g = group_size > 0 ? group_size : n;
    const size_t np = (size_t)n * p;
    admmq_arena_reset_transient(ctx);
    ADMMQ_TRY(admmq_arena_reserve(ctx, 2 * admmq_align_up(np * 4) + 8192));
    double lambda = 0.0;
    ADMMQ_TRY(hessian_scalars(ctx, H, n, damp, &lambda));
    float *E = nullptr, *tmp = nullptr;
    double *dev = nullptr;
    ADMMQ_TRY(take(ctx, E, np));
    ADMMQ_TRY(take(ctx, tmp, np));
    ADMMQ_TRY(take(ctx, dev, 2));
    ADMMQ_TRY(admmq_k_quant_error(ctx, W0, ldw, (uint8_t *)codes, n, p, g, scales, zeros, 8, 0, E));
    ADMMQ_TRY(objective_core(ctx, H, lambda, n, p, E, tmp, dev));
    ADMMQ_TRY(read_back(ctx, j_out, dev, 8));
    admmq_arena_reset_transient(ctx);
    return ADMMQ_OK;
}

extern "C" admmq_status admmq_ls_evaluate(admmq_ctx *ctx, const float *H, double lambda, const float *G,
                                          const uint8_t *codes, int64_t n, int64_t p, int32_t bits,
                                          int32_t group_size, const float *scales, const int32_t *pairs,
                                          int32_t npairs, float *totals) {
    if (!ctx || !G || !codes || !scales || !pairs || !totals) return ADMMQ_ERR_NULL;
    ADMMQ_TRY(check_layer_args(H, G, n, p, p, bits, group_size));
    if (npairs < 1) return ADMMQ_ERR_SHAPE;
    if (ctx->device < 0) return ADMMQ_ERR_DEVICE;
    ADMMQ_HIP(hipSetDevice(ctx->device));
    const int64_t g = group_size > 0 ? group_size : n;
    const int chunks = admmq_ls_chunks(p);
    admmq_arena_reset_transient(ctx);
    ADMMQ_TRY(admmq_arena_reserve(ctx, admmq_align_up((size_t)npairs * chunks * 4) + 4096));
    float *partial = nullptr;
    ADMMQ_TRY(take(ctx, partial, (size_t)npairs * chunks));
    ADMMQ_TRY(admmq_k_ls_step(ctx, H, (float)lambda, G, (uint8_t *)codes, n, p, bits, g, scales, nullptr, 0, nullptr,
                              nullptr, 0, pairs, npairs, 0, nullptr, nullptr, nullptr, partial, nullptr, nullptr,
                              nullptr, nullptr, nullptr, 0, nullptr, nullptr));
    ADMMQ_TRY(admmq_k_ls_totals(ctx, partial, chunks, npairs, totals));
    admmq_arena_reset_transient(ctx);
    return ADMMQ_OK;
}

extern "C" void admmq_sample_pair(uint64_t seed, int32_t round, int32_t batch, int32_t slot, int64_t n,
                                  int32_t *i1, int32_t *i2) {
    const uint64_t key = ((uint64_t)(uint32_t)round << 48) ^ ((uint64_t)(uint32_t)batch << 16) ^ (uint64_t)(uint32_t)slot;
    const uint64_t c = mix64(seed ^ mix64(key));
    const uint64_t a = (c & 0xFFFFFFFFull) % (uint64_t)n;
    const uint64_t b = (a + 1 + ((c >> 32) % (uint64_t)(n - 1))) % (uint64_t)n;
    *i1 = (int32_t)a;
    *i2 = (int32_t)b;
}

extern "C" int32_t admmq_ls_fallback_count(const admmq_ctx *ctx) { return ctx ? ctx->ls_fallback_groups : 0; }

// ---- local search alone --------------------------------------------------------------------------
extern "C" admmq_status admmq_local_search(admmq_ctx *ctx, const float *H, const float *W0, int64_t n, int64_t p,
                                           int64_t ldw, int32_t bits, int32_t group_size, const float *scales,
                                           const float *zeros, uint8_t *codes, const admmq_ls_params *prm,
                                           const int32_t *explicit_pairs, int32_t *moves_out, double *drop_out) {
    if (!ctx || !scales || !zeros || !codes || !prm) return ADMMQ_ERR_NULL;
    ADMMQ_TRY(check_layer_args(H, W0, n, p, ldw, bits, group_size));
    if (prm->rounds < 0 || prm->batches_per_round < 0 || prm->pairs_per_batch < 0 || !(prm->damp >= 0.0))
        return ADMMQ_ERR_PARAM;
    if (n < 2) return ADMMQ_ERR_SHAPE;
    if (ctx->device < 0) return ADMMQ_ERR_DEVICE;
    ADMMQ_HIP(hipSetDevice(ctx->device));
    const int64_t g = group_size > 0 ? group_size : n;
    LsPlan plan = ls_plan(n, prm->rounds > 0 ? prm->rounds : 5, prm->batches_per_round, prm->pairs_per_batch);
    admmq_arena_reset_transient(ctx);
    ADMMQ_TRY(admmq_arena_reserve(
        ctx, ls_transient_bytes(n, p, (int64_t)plan.rounds * plan.batches * plan.pairs, plan.pairs)));
    double lambda = 0.0;
    ADMMQ_TRY(hessian_scalars(ctx, H, n, prm->damp, &lambda));
    admmq_status s = admmq_guarded([&] {
        return local_search_core(ctx, H, lambda, W0, n, p, ldw, bits, g, scales, zeros, codes, plan, prm->seed,
                                 explicit_pairs, moves_out, drop_out);
    });
    admmq_arena_reset_transient(ctx);
    return s;
}

// ---- whole layer -----------------------------------------------------------------------------------
// ---- other formats (Sec. 4.3) --------------------------------------------------------------------------
namespace {

admmq_status check_format(const admmq_format *fmt, int64_t n) {
    if (!fmt) return ADMMQ_ERR_NULL;
    if (fmt->kind == ADMMQ_FORMAT_DUAL_GRID) {
        if (!fmt->flags || !fmt->scales || !fmt->zeros) return ADMMQ_ERR_NULL;
        if (fmt->bits < 2 || fmt->bits > 8) return ADMMQ_ERR_PARAM;
        if (fmt->group_size < 0 || (fmt->group_size > 0 && n % fmt->group_size != 0)) return ADMMQ_ERR_SHAPE;
    } else if (fmt->kind == ADMMQ_FORMAT_CODEBOOK) {
        if (!fmt->codebook) return ADMMQ_ERR_NULL;
        if (fmt->bits < 1 || fmt->bits > 4 || fmt->group_size != 0) return ADMMQ_ERR_PARAM;
    } else {
        return ADMMQ_ERR_PARAM;
    }
    return ADMMQ_OK;
}

// a codebook must be finite and strictly ascending per column (synchronises)
admmq_status check_codebook(admmq_ctx *ctx, const float *codebook, int bits, int64_t p) {
    double *dev = nullptr;
    ADMMQ_TRY(take(ctx, dev, 2));
    ADMMQ_TRY(admmq_k_fill_bytes(ctx, dev, 0, 16));
    ADMMQ_TRY(admmq_k_codebook_check(ctx, codebook, 1 << bits, p, dev));
    double bad = 0.0;
    ADMMQ_TRY(read_back(ctx, &bad, dev, 8));
    return bad > 0.0 ? ADMMQ_ERR_PARAM : ADMMQ_OK;
}

}  // namespace

// ---- the whole layer (Alg. 1), for the uniform grid and for the other formats of Sec. 4.3 ------------------
namespace {

// What the D-update projects onto.  kind 0: the uniform grid of eq. 10 (scales / zeros [n/g][p], fitted here with
// the schedule's options, refreshed if asked, local search afterwards).  kind 1 / 2: admmq_format_kind (dual grid:
// scales / zeros [2][n/g][p]; codebook: levels and optional flags); Wq receives the dense result.
struct Projection {
    int kind;
    int bits;
    int64_t g;
    float *scales, *zeros;
    const uint8_t *flags;
    const float *codebook;
    float *Wq;
};

admmq_status quantize_core(admmq_ctx *ctx, const float *H, const float *W0, int64_t n, int64_t p, int64_t ldw,
                           const Projection &pj, const admmq_schedule *sched, uint8_t *codes, admmq_stats *stats) {
    const bool uniform = pj.kind == 0;
    const int bits = pj.bits;
    const int64_t g = pj.g;
    const int T = sched->T;
    const size_t np = (size_t)n * p;
    const size_t ng = (size_t)(n / g) * p * (pj.kind == ADMMQ_FORMAT_DUAL_GRID ? 2 : 1);     // grid entries
    const bool want = stats != nullptr;
    const bool want_obj = want && stats->skip_objectives == 0;        // the objectives are reports, not steps of Alg. 1
    Timer t_total(ctx->stream, want), t_phase(ctx->stream, want);
    t_total.start();
    float prof_ms[ADMMQ_TAGS] = {};
    int prof_cnt[ADMMQ_TAGS] = {};
    prof_collect(ctx, prof_ms, prof_cnt);            // drops spans a failed earlier call may have left
    ctx->prof.on = want && stats->profile != 0;

    // --- input checks on the device, before anything is written -------------------------------
    t_phase.start();
    admmq_arena_reset_transient(ctx);
    ADMMQ_TRY(admmq_arena_reserve(ctx, 8192));
    {
        double *dev = nullptr;
        ADMMQ_TRY(take(ctx, dev, 2));
        ADMMQ_TRY(admmq_k_fill_bytes(ctx, dev, 0, 16));
        ADMMQ_TRY(admmq_k_count_nonfinite(ctx, W0, n, p, ldw, dev));
        double bad = 0.0;
        ADMMQ_TRY(read_back(ctx, &bad, dev, 8));
        if (bad > 0.0) return ADMMQ_ERR_NOT_FINITE;
        if (pj.kind == ADMMQ_FORMAT_CODEBOOK) ADMMQ_TRY(check_codebook(ctx, pj.codebook, bits, p));
    }
    float ms_setup = t_phase.stop();

    // --- Alg. 1 lines 1-3 ----------------------------------------------------------------------
    t_phase.start();
    double lambda = 0.0;
    if (sched->reuse_factor) {
        const admmq_factor &have = ctx->fac;
        if (!have.valid || have.n != n || have.H_src != H || have.damp != sched->damp ||
            have.precondition != sched->precondition)
            return ADMMQ_ERR_STATE;
        lambda = have.lambda;
        admmq_arena_reset_transient(ctx);
    } else {
        ADMMQ_TRY(do_factorize(ctx, H, n, sched->damp, sched->precondition, &lambda));
    }
    float ms_factor = t_phase.stop();
    const admmq_factor &f = ctx->fac;

    // --- grid, initial state, schedule -----------------------------------------------------------
    t_phase.start();
    LsPlan plan = ls_plan(n, uniform ? sched->ls_rounds : 0, sched->ls_batches, sched->ls_pairs);
    const bool fast = fast_wanted(ctx, n, p);
    size_t need = admm_transient_bytes(n, p, T) + 3 * admmq_align_up(ng * 4) +
                  admmq_align_up((size_t)2 * admmq_refresh_error_blocks() * 8) + (fast ? fast_products_bytes(n, p) : 0);
    if (plan.rounds > 0 && n >= 2) {
        const size_t ls = ls_transient_bytes(n, p, (int64_t)plan.rounds * plan.batches * plan.pairs, plan.pairs);
        if (ls > need) need = ls;
    }
    ADMMQ_TRY(admmq_arena_reserve(ctx, need));
    float *B = nullptr, *V = nullptr, *W = nullptr, *C0 = nullptr, *Y = nullptr, *inv_scales = nullptr;
    double *F = nullptr, *rhos = nullptr, *res = nullptr, *jdev = nullptr;
    MidFactors mf;
    unsigned long long *flips = nullptr;
    ADMMQ_TRY(take(ctx, B, np));
    ADMMQ_TRY(take(ctx, V, np));
    ADMMQ_TRY(take(ctx, W, np));
    ADMMQ_TRY(take(ctx, C0, np));
    ADMMQ_TRY(take(ctx, Y, np));
    ADMMQ_TRY(take(ctx, F, np + (size_t)p));
    ADMMQ_TRY(take(ctx, inv_scales, ng));
    float *new_sc = nullptr, *new_zr = nullptr;
    double *rpart = nullptr;
    ADMMQ_TRY(take(ctx, new_sc, ng));
    ADMMQ_TRY(take(ctx, new_zr, ng));
    ADMMQ_TRY(take(ctx, rpart, (size_t)2 * admmq_refresh_error_blocks()));
    int refresh_accepted = 0;
    double refresh_eo = 0.0, refresh_en = 0.0;
    ADMMQ_TRY(take(ctx, rhos, (size_t)T));
    ADMMQ_TRY(mid_factors_take(ctx, n, T, mf));
    ADMMQ_TRY(take(ctx, res, (size_t)T));
    ADMMQ_TRY(take(ctx, flips, (size_t)T));
    ADMMQ_TRY(take(ctx, jdev, 4));
    FastBufs fbufs;
    if (fast) ADMMQ_TRY(fast_setup(ctx, n, p, fbufs));

    if (uniform)
        ADMMQ_TRY(admmq_k_grid_fit(ctx, W0, n, p, ldw, bits, g, sched->symmetric != 0, sched->clip_points,
                                   sched->clip_shrink, pj.scales, pj.zeros));
    else if (pj.kind == ADMMQ_FORMAT_DUAL_GRID)
        ADMMQ_TRY(admmq_k_dual_grid_init(ctx, W0, n, p, ldw, bits, g, pj.flags, pj.scales, pj.zeros));
    if (pj.kind != ADMMQ_FORMAT_CODEBOOK) ADMMQ_TRY(admmq_k_recip(ctx, pj.scales, inv_scales, (int64_t)ng));
    // D^(0) = Ws, V^(0) = 0  =>  B^(0) = Ws
    ADMMQ_TRY(admmq_k_scale_rows(ctx, W0, ldw, f.d, n, p, B, p));
    ADMMQ_TRY(admmq_k_fill_bytes(ctx, V, 0, np * 4));
    ADMMQ_TRY(admmq_k_fill_bytes(ctx, res, 0, (size_t)T * 8));
    ADMMQ_TRY(admmq_k_fill_bytes(ctx, flips, 0, (size_t)T * 8));
    // the stopping rule needs the number of codes that changed, every iteration (as the flip history does)
    const int quiet_stop = uniform ? sched->quiet_stop : 0;
    const bool report_flips = uniform && want && stats->code_flips != nullptr;
    const bool want_flips = report_flips || quiet_stop > 0;
    if (want_flips) ADMMQ_TRY(admmq_k_fill_bytes(ctx, codes, 0, np));
    std::vector<double> hrho((size_t)T + 1);
    {
        double r = sched->rho0;
        for (int t = 0; t <= T; ++t) {
            hrho[t] = r;
            r *= sched->gamma;
        }
    }
    ADMMQ_HIP(hipMemcpyAsync(rhos, hrho.data(), (size_t)T * 8, hipMemcpyHostToDevice, ctx->stream));
    ADMMQ_HIP(hipStreamSynchronize(ctx->stream));
    ADMMQ_TRY(mid_factors_compute(ctx, n, rhos, T, mf));
    // C0 = Q^T Ws
    gemm_tn_args g0 = {};
    g0.A = f.Q; g0.lda = n; g0.B = B; g0.ldb = p; g0.M = n; g0.N = p; g0.K = n;
    g0.alpha = 1.f; g0.Z = nullptr; g0.out = C0; g0.ldo = p; g0.split_k = 1;
    ADMMQ_TRY(admmq_gemm_tn(ctx, g0));
    if (want_obj) {
        // the plain projection of W0 (round-to-nearest on the initial grid) as the baseline objective; W, Y and F
        // are still free
        if (uniform)
            ADMMQ_TRY(admmq_k_quant_error(ctx, W0, ldw, (uint8_t *)F, n, p, g, pj.scales, pj.zeros, bits, 2, W));
        else
            ADMMQ_TRY(admmq_k_nearest_error(ctx, pj.kind, W0, ldw, n, p, bits, g, pj.flags, pj.scales, pj.zeros,
                                            pj.codebook, nullptr, W));
        ADMMQ_TRY(objective_core(ctx, H, lambda, n, p, W, Y, jdev));
        ADMMQ_TRY(read_back(ctx, &stats->j_damp_rtn, jdev, 8));
    }
    ms_setup += t_phase.stop();

    // --- ADMM loop (Alg. 1 lines 5-9) -------------------------------------------------------------
    t_phase.start();
    // W and B trade places every iteration: the projection pass writes B^(t+1) over the W it has just read
    float *Bcur = B, *Wcur = W;
    int iters = 0, quiet = 0;
    // Iterations that need neither codes nor W itself run the projection pass as the epilogue of the second
    // product (W never goes to memory, B^(t+1) replaces B^(t) in place) where the product's shape allows it.
    gemm_proj_args pa = {};
    bool fuse = uniform && !fast && !want_flips && fuse_projection_enabled();
    if (fuse) {
        int sh = -1;
        if (g == n) sh = 62;
        else if (g > 0 && (g & (g - 1)) == 0)
            for (sh = 0; ((int64_t)1 << sh) < g; ++sh) {}
        if (sh < 0) {
            fuse = false;
        } else {
            pa.V = V; pa.ldv = p; pa.d = f.d; pa.inv_d = f.inv_d; pa.scales = pj.scales; pa.inv_scales = inv_scales;
            pa.zeros = pj.zeros; pa.ld_grid = p; pa.g_shift = sh; pa.levels = (float)((1 << bits) - 1);
            pa.res_sq = res;
            gemm_tn_args probe = {};
            probe.A = f.Qt; probe.lda = n; probe.B = F; probe.ldb = p; probe.M = n; probe.N = p; probe.K = n;
            probe.alpha = 1.f; probe.beta = 1.f; probe.Z = B; probe.ldz = p; probe.out = B; probe.ldo = p;
            probe.split_k = 1; probe.proj = &pa;
            fuse = admmq_gemm_tn_can_project(probe) && ((uintptr_t)W & 15) == 0;
        }
    }
    for (int t = 0; t < T; ++t) {
        const float rf = (float)hrho[t], rf_next = (float)hrho[t + 1];
        const bool last = t == T - 1;
        if (fuse && t > 0 && !last && !(uniform && t == sched->refresh_iter)) {
            pa.rho = rf; pa.inv_rho = 1.0f / rf; pa.inv_rho_next = 1.0f / rf_next; pa.res_sq = res + t;
            ADMMQ_TRY(w_update_core(ctx, C0, Bcur, n, p, mf, t, Y, F, Bcur, nullptr, &pa));
            iters = t + 1;
            continue;
        }
        if (t == 0) {
            // D^(0) = Ws and V^(0) = 0 make eq. 7 return Ws exactly: no product needed
            ADMMQ_HIP(hipMemcpyAsync(Wcur, Bcur, np * 4, hipMemcpyDeviceToDevice, ctx->stream));
        } else {
            ADMMQ_TRY(w_update_core(ctx, C0, Bcur, n, p, mf, t, Y, F, Wcur,
                                    fast ? &fbufs : nullptr));
        }
        if (uniform && t == sched->refresh_iter)
            ADMMQ_TRY(grid_refresh_core(ctx, Wcur, V, n, p, f.d, f.inv_d, bits, g, hrho[t], pj.scales, pj.zeros,
                                        inv_scales, new_sc, new_zr, rpart, &refresh_accepted, &refresh_eo,
                                        &refresh_en));
        const int sp = admmq_prof_begin(ctx, ADMMQ_TAG_PROJECT);
        if (uniform)
            ADMMQ_TRY(admmq_k_project_dual(ctx, Wcur, V, n, p, f.d, f.inv_d, bits, g, pj.scales, inv_scales, pj.zeros,
                                           rf, 1.0f / rf, 1.0f / rf_next, (last || want_flips) ? codes : nullptr,
                                           want_flips ? 1 : 0, Wcur, res + t, want_flips ? flips + t : nullptr, p,
                                           fast ? (unsigned *)fbufs.slotsO[0] : nullptr));
        else
            ADMMQ_TRY(admmq_k_project_format(ctx, pj.kind, Wcur, V, n, p, f.d, f.inv_d, bits, g, pj.flags, pj.scales,
                                             inv_scales, pj.zeros, pj.codebook, rf, 1.0f / rf, 1.0f / rf_next,
                                             last ? 1 : 0, codes, Wcur, pj.Wq, res + t,
                                             fast ? (unsigned *)fbufs.slotsO[0] : nullptr));
        admmq_prof_end(ctx, sp);
        if (fast) fbufs.b_max_ready = true;                // (the pass has left the largest |B| in its slot)
        float *tmpp = Bcur;
        Bcur = Wcur;
        Wcur = tmpp;
        iters = t + 1;
        if (quiet_stop > 0 && t >= 1) {
            unsigned long long changed = 0;
            ADMMQ_TRY(read_back(ctx, &changed, flips + t, 8));
            quiet = changed == 0 ? quiet + 1 : 0;
            if (quiet >= quiet_stop) break;           // the codes of this iteration are in `codes`
        }
    }
    float ms_admm = t_phase.stop();

    if (want) {
        stats->iters_done = iters;
        stats->lambda = lambda;
        stats->refresh_accepted = refresh_accepted;
        stats->refresh_err_old = refresh_eo;
        stats->refresh_err_new = refresh_en;
        if (stats->primal_res) {
            std::vector<double> h((size_t)T);
            ADMMQ_TRY(read_back(ctx, h.data(), res, (size_t)T * 8));
            for (int t = 0; t < T; ++t) stats->primal_res[t] = (float)sqrt(h[t]);
        }
        if (report_flips) {
            std::vector<unsigned long long> h((size_t)T);
            ADMMQ_TRY(read_back(ctx, h.data(), flips, (size_t)T * 8));
            for (int t = 0; t < T; ++t) stats->code_flips[t] = (int64_t)h[t];
        }
        // objective of the ADMM result; W, Y are free now
        stats->j_damp_admm = stats->j_recon = 0.0;
        if (!want_obj) stats->j_damp_rtn = 0.0;
        if (want_obj) {
            if (uniform)
                ADMMQ_TRY(admmq_k_quant_error(ctx, W0, ldw, codes, n, p, g, pj.scales, pj.zeros, bits, 0, W));
            else
                ADMMQ_TRY(admmq_k_diff(ctx, pj.Wq, W0, ldw, n, p, W));
            ADMMQ_TRY(objectives_core(ctx, H, lambda, n, p, W, Y, jdev, &stats->j_damp_admm, &stats->j_recon));
        }
        stats->j_damp = stats->j_damp_admm;
        stats->ls_moves = 0;
    }

    // --- local search (Alg. 1 line 11; uniform grids only) -----------------------------------------
    t_phase.start();
    float ms_ls = 0.f;
    if (plan.rounds > 0 && n >= 2) {
        admmq_arena_reset_transient(ctx);
        int32_t moves = 0;
        double drop = 0.0;
        ADMMQ_TRY(local_search_core(ctx, H, lambda, W0, n, p, ldw, bits, g, pj.scales, pj.zeros, codes, plan,
                                    sched->seed, nullptr, &moves, &drop));
        ms_ls = t_phase.stop();
        if (want) stats->ls_moves = moves;
        if (want_obj) {
            admmq_arena_reset_transient(ctx);
            float *E = nullptr, *tmp = nullptr;
            double *jd = nullptr;
            ADMMQ_TRY(take(ctx, E, np));
            ADMMQ_TRY(take(ctx, tmp, np));
            ADMMQ_TRY(take(ctx, jd, 2));
            ADMMQ_TRY(admmq_k_quant_error(ctx, W0, ldw, codes, n, p, g, pj.scales, pj.zeros, bits, 0, E));
            ADMMQ_TRY(objectives_core(ctx, H, lambda, n, p, E, tmp, jd, &stats->j_damp, &stats->j_recon));
        }
    }
    // (the call's time ends here: reading the per-launch events back is the caller's measurement, not the method)
    const float ms_call = want ? t_total.stop() : 0.f;
    prof_collect(ctx, prof_ms, prof_cnt);
    if (want) {
        stats->ms_gemm = prof_ms[ADMMQ_TAG_GEMM];       stats->n_gemm = prof_cnt[ADMMQ_TAG_GEMM];
        stats->ms_tridiag = prof_ms[ADMMQ_TAG_TRIDIAG]; stats->n_tridiag = prof_cnt[ADMMQ_TAG_TRIDIAG];
        stats->ms_project = prof_ms[ADMMQ_TAG_PROJECT]; stats->n_project = prof_cnt[ADMMQ_TAG_PROJECT];
        stats->ms_ls_apply = prof_ms[ADMMQ_TAG_LS_APPLY]; stats->n_ls_apply = prof_cnt[ADMMQ_TAG_LS_APPLY];
        stats->ms_gemm_project = prof_ms[ADMMQ_TAG_GEMM_PROJECT];
        stats->n_gemm_project = prof_cnt[ADMMQ_TAG_GEMM_PROJECT];
        stats->ms_setup = ms_setup;
        stats->ms_factor = ms_factor;
        stats->ms_admm = ms_admm;
        stats->ms_local_search = ms_ls;
        stats->ms_total = ms_call;
    }
    admmq_arena_reset_transient(ctx);
    return ADMMQ_OK;
}

// Several matrices on one Hessian: one factorisation, the W-update products over all columns at once, everything
// that depends on a matrix's own grid matrix by matrix.  State W, B, C0, Y: [n][P] with the matrices side by side;
// V, codes and grids: one contiguous array per matrix.
admmq_status quantize_many_core(admmq_ctx *ctx, const float *H, int64_t n, const admmq_layer *L, int count,
                                const admmq_schedule *sched, admmq_stats *stats) {
    const int T = sched->T;
    const bool want = stats != nullptr;
    const bool want_obj = want && stats[0].skip_objectives == 0;
    int64_t P = 0;
    std::vector<int64_t> off((size_t)count), grp((size_t)count);
    int64_t pmax = 0;
    for (int i = 0; i < count; ++i) {
        off[i] = P;
        grp[i] = L[i].group_size > 0 ? L[i].group_size : n;
        P += L[i].p;
        if (L[i].p > pmax) pmax = L[i].p;
    }
    const size_t nP = (size_t)n * P;
    Timer t_total(ctx->stream, want), t_phase(ctx->stream, want);
    t_total.start();
    float prof_ms[ADMMQ_TAGS] = {};
    int prof_cnt[ADMMQ_TAGS] = {};
    prof_collect(ctx, prof_ms, prof_cnt);
    ctx->prof.on = want && stats[0].profile != 0;

    t_phase.start();
    admmq_arena_reset_transient(ctx);
    ADMMQ_TRY(admmq_arena_reserve(ctx, 8192));
    {
        double *dev = nullptr;
        ADMMQ_TRY(take(ctx, dev, 2));
        ADMMQ_TRY(admmq_k_fill_bytes(ctx, dev, 0, 16));
        for (int i = 0; i < count; ++i) ADMMQ_TRY(admmq_k_count_nonfinite(ctx, L[i].W0, n, L[i].p, L[i].ldw, dev));
        double bad = 0.0;
        ADMMQ_TRY(read_back(ctx, &bad, dev, 8));
        if (bad > 0.0) return ADMMQ_ERR_NOT_FINITE;
    }
    float ms_setup = t_phase.stop();

    // --- Alg. 1 lines 1-3, once ----------------------------------------------------------------
    t_phase.start();
    double lambda = 0.0;
    if (sched->reuse_factor) {
        const admmq_factor &have = ctx->fac;
        if (!have.valid || have.n != n || have.H_src != H || have.damp != sched->damp ||
            have.precondition != sched->precondition)
            return ADMMQ_ERR_STATE;
        lambda = have.lambda;
        admmq_arena_reset_transient(ctx);
    } else {
        ADMMQ_TRY(do_factorize(ctx, H, n, sched->damp, sched->precondition, &lambda));
    }
    float ms_factor = t_phase.stop();
    const admmq_factor &f = ctx->fac;

    // --- grids, initial state, schedule -----------------------------------------------------------
    t_phase.start();
    LsPlan plan = ls_plan(n, sched->ls_rounds, sched->ls_batches, sched->ls_pairs);
    size_t ng_total = 0;
    for (int i = 0; i < count; ++i) ng_total += admmq_align_up((size_t)(n / grp[i]) * L[i].p * 4);
    const bool fast = fast_wanted(ctx, n, P);
    size_t need = admm_transient_bytes(n, P, T) + ng_total + (size_t)count * (2 * admmq_align_up((size_t)T * 8) + 1024) +
                  (fast ? fast_products_bytes(n, P) : 0);
    if (plan.rounds > 0 && n >= 2) {
        const size_t ls = ls_transient_bytes(n, pmax, (int64_t)plan.rounds * plan.batches * plan.pairs, plan.pairs);
        if (ls > need) need = ls;
    }
    ADMMQ_TRY(admmq_arena_reserve(ctx, need));
    float *B = nullptr, *W = nullptr, *C0 = nullptr, *Y = nullptr;
    double *F = nullptr, *rhos = nullptr, *jdev = nullptr;
    MidFactors mf;
    std::vector<float *> V((size_t)count), inv_scales((size_t)count);
    std::vector<double *> res((size_t)count);
    ADMMQ_TRY(take(ctx, B, nP));
    ADMMQ_TRY(take(ctx, W, nP));
    ADMMQ_TRY(take(ctx, C0, nP));
    ADMMQ_TRY(take(ctx, Y, nP));
    ADMMQ_TRY(take(ctx, F, nP + (size_t)P));
    for (int i = 0; i < count; ++i) {
        ADMMQ_TRY(take(ctx, V[i], (size_t)n * L[i].p));
        ADMMQ_TRY(take(ctx, inv_scales[i], (size_t)(n / grp[i]) * L[i].p));
        ADMMQ_TRY(take(ctx, res[i], (size_t)T));
    }
    ADMMQ_TRY(take(ctx, rhos, (size_t)T));
    ADMMQ_TRY(mid_factors_take(ctx, n, T, mf));
    ADMMQ_TRY(take(ctx, jdev, 4));
    FastBufs fbufs;
    if (fast) ADMMQ_TRY(fast_setup(ctx, n, P, fbufs));
    // the stopping rule: codes changed per iteration and matrix, [T][count]; the loop ends once no matrix has
    // changed a code for quiet_stop iterations in a row
    const int quiet_stop = sched->quiet_stop;
    unsigned long long *flips = nullptr;
    if (quiet_stop > 0) {
        ADMMQ_TRY(take(ctx, flips, (size_t)T * count));
        ADMMQ_TRY(admmq_k_fill_bytes(ctx, flips, 0, (size_t)T * count * 8));
        for (int i = 0; i < count; ++i) ADMMQ_TRY(admmq_k_fill_bytes(ctx, L[i].codes, 0, (size_t)n * L[i].p));
    }
    for (int i = 0; i < count; ++i) {
        const admmq_layer &l = L[i];
        ADMMQ_TRY(admmq_k_grid_fit(ctx, l.W0, n, l.p, l.ldw, l.bits, grp[i], sched->symmetric != 0, sched->clip_points,
                                   sched->clip_shrink, l.scales, l.zeros));
        ADMMQ_TRY(admmq_k_recip(ctx, l.scales, inv_scales[i], (int64_t)((n / grp[i]) * l.p)));
        ADMMQ_TRY(admmq_k_scale_rows(ctx, l.W0, l.ldw, f.d, n, l.p, B + off[i], P));
        ADMMQ_TRY(admmq_k_fill_bytes(ctx, V[i], 0, (size_t)n * l.p * 4));
        ADMMQ_TRY(admmq_k_fill_bytes(ctx, res[i], 0, (size_t)T * 8));
    }
    std::vector<double> hrho((size_t)T + 1);
    {
        double r = sched->rho0;
        for (int t = 0; t <= T; ++t) {
            hrho[t] = r;
            r *= sched->gamma;
        }
    }
    ADMMQ_HIP(hipMemcpyAsync(rhos, hrho.data(), (size_t)T * 8, hipMemcpyHostToDevice, ctx->stream));
    ADMMQ_HIP(hipStreamSynchronize(ctx->stream));
    ADMMQ_TRY(mid_factors_compute(ctx, n, rhos, T, mf));
    gemm_tn_args g0 = {};
    g0.A = f.Q; g0.lda = n; g0.B = B; g0.ldb = P; g0.M = n; g0.N = P; g0.K = n;
    g0.alpha = 1.f; g0.Z = nullptr; g0.out = C0; g0.ldo = P; g0.split_k = 1;
    ADMMQ_TRY(admmq_gemm_tn(ctx, g0));
    if (want_obj) {
        // round-to-nearest on the initial grid as the baseline objective; W, Y and F are still free
        for (int i = 0; i < count; ++i) {
            const admmq_layer &l = L[i];
            ADMMQ_TRY(admmq_k_quant_error(ctx, l.W0, l.ldw, (uint8_t *)F, n, l.p, grp[i], l.scales, l.zeros, l.bits, 2, W));
            ADMMQ_TRY(objective_core(ctx, H, lambda, n, l.p, W, Y, jdev));
            ADMMQ_TRY(read_back(ctx, &stats[i].j_damp_rtn, jdev, 8));
        }
    }
    ms_setup += t_phase.stop();

    // --- ADMM loop (Alg. 1 lines 5-9) -------------------------------------------------------------
    t_phase.start();
    float *Bcur = B, *Wcur = W;
    int iters = 0, quiet = 0;
    for (int t = 0; t < T; ++t) {
        const float rf = (float)hrho[t], rf_next = (float)hrho[t + 1];
        if (t == 0)
            ADMMQ_HIP(hipMemcpyAsync(Wcur, Bcur, nP * 4, hipMemcpyDeviceToDevice, ctx->stream));
        else
            ADMMQ_TRY(w_update_core(ctx, C0, Bcur, n, P, mf, t, Y, F, Wcur,
                                    fast ? &fbufs : nullptr));
        const bool last = t == T - 1;
        const int sp = admmq_prof_begin(ctx, ADMMQ_TAG_PROJECT);
        for (int i = 0; i < count; ++i) {
            const admmq_layer &l = L[i];
            ADMMQ_TRY(admmq_k_project_dual(ctx, Wcur + off[i], V[i], n, l.p, f.d, f.inv_d, l.bits, grp[i], l.scales,
                                           inv_scales[i], l.zeros, rf, 1.0f / rf, 1.0f / rf_next,
                                           (last || quiet_stop > 0) ? l.codes : nullptr, quiet_stop > 0 ? 1 : 0,
                                           Wcur + off[i], res[i] + t,
                                           quiet_stop > 0 ? flips + (size_t)t * count + i : nullptr, P,
                                           fast ? (unsigned *)fbufs.slotsO[0] : nullptr));
        }
        admmq_prof_end(ctx, sp);
        if (fast) fbufs.b_max_ready = true;
        float *tmpp = Bcur;
        Bcur = Wcur;
        Wcur = tmpp;
        iters = t + 1;
        if (quiet_stop > 0 && t >= 1) {
            std::vector<unsigned long long> changed((size_t)count);
            ADMMQ_TRY(read_back(ctx, changed.data(), flips + (size_t)t * count, (size_t)count * 8));
            bool still = true;
            for (int i = 0; i < count; ++i) still = still && changed[i] == 0;
            quiet = still ? quiet + 1 : 0;
            if (quiet >= quiet_stop) break;
        }
    }
    float ms_admm = t_phase.stop();

    if (want) {
        for (int i = 0; i < count; ++i) {
            const admmq_layer &l = L[i];
            admmq_stats &st = stats[i];
            st.iters_done = iters;
            st.lambda = lambda;
            st.refresh_accepted = 0;
            st.refresh_err_old = st.refresh_err_new = 0.0;
            if (st.primal_res) {
                std::vector<double> h((size_t)T);
                ADMMQ_TRY(read_back(ctx, h.data(), res[i], (size_t)T * 8));
                for (int t = 0; t < T; ++t) st.primal_res[t] = (float)sqrt(h[t]);
            }
            if (st.code_flips)
                for (int t = 0; t < T; ++t) st.code_flips[t] = -1;       // not counted on this path
            st.j_damp_admm = st.j_recon = 0.0;
            if (!want_obj) st.j_damp_rtn = 0.0;
            if (want_obj) {
                ADMMQ_TRY(admmq_k_quant_error(ctx, l.W0, l.ldw, l.codes, n, l.p, grp[i], l.scales, l.zeros, l.bits, 0, W));
                ADMMQ_TRY(objectives_core(ctx, H, lambda, n, l.p, W, Y, jdev, &st.j_damp_admm, &st.j_recon));
            }
            st.j_damp = st.j_damp_admm;
            st.ls_moves = 0;
        }
    }

    // --- local search (Alg. 1 line 11), matrix by matrix ------------------------------------------
    // The search is a chain of short dependent launches that leaves most of the chip idle, and the matrices'
    // searches are independent of each other: up to four run side by side, each on a stream and a host thread of
    // its own with its own slice of the scratch arena (the result of each is what it would be alone).
    t_phase.start();
    float ms_ls = 0.f;
    if (plan.rounds > 0 && n >= 2) {
        admmq_arena_reset_transient(ctx);
        std::vector<int32_t> moves((size_t)count, 0);
        const int64_t total_pairs = (int64_t)plan.rounds * plan.batches * plan.pairs;
        int workers = count < 4 ? count : 4;
        std::vector<size_t> slice((size_t)workers, 0), start((size_t)workers, 0);
        size_t all = 0;
        if (workers > 1) {
            for (int i = 0; i < count; ++i) {
                const size_t b = admmq_align_up(ls_transient_bytes(n, L[i].p, total_pairs, plan.pairs));
                if (b > slice[i % workers]) slice[i % workers] = b;
            }
            for (int w = 0; w < workers; ++w) {
                start[w] = all;
                all += slice[w];
            }
            if (admmq_arena_reserve(ctx, all) != ADMMQ_OK) workers = 1;     // a caller's arena too small for that
        }
        if (workers > 1) {
            if (!ctx->side_ready) ADMMQ_HIP(hipEventCreateWithFlags(&ctx->side_ready, hipEventDisableTiming));
            for (int w = 1; w < workers; ++w)
                if (!ctx->side[w - 1]) ADMMQ_HIP(hipStreamCreateWithFlags(&ctx->side[w - 1], hipStreamNonBlocking));
            ADMMQ_HIP(hipEventRecord(ctx->side_ready, ctx->stream));          // the codes of the ADMM loop
            for (int w = 1; w < workers; ++w) ADMMQ_HIP(hipStreamWaitEvent(ctx->side[w - 1], ctx->side_ready, 0));
            char *base = ctx->arena + ctx->persist_top;
            std::vector<admmq_status> result((size_t)workers, ADMMQ_OK);
            std::vector<int> redone((size_t)workers, 0);
            auto run = [&](int w) {
                if (hipSetDevice(ctx->device) != hipSuccess) {
                    result[w] = ADMMQ_ERR_DEVICE;
                    return;
                }
                admmq_ctx child;
                child.device = ctx->device;
                child.stream = w == 0 ? ctx->stream : ctx->side[w - 1];
                child.arena = base + start[w];
                child.arena_bytes = slice[w];
                child.arena_owned = false;
                child.ls_side_by_side = workers;      // the searches share the chip: each may hold its share of blocks
                for (int i = w; i < count; i += workers) {
                    const admmq_layer &l = L[i];
                    child.top = child.persist_top = 0;
                    double drop = 0.0;
                    const admmq_status s = admmq_guarded([&] {
                        return local_search_core(&child, H, lambda, l.W0, n, l.p, l.ldw, l.bits, grp[i], l.scales,
                                                 l.zeros, l.codes, plan, sched->seed, nullptr, &moves[i], &drop);
                    });
                    if (s != ADMMQ_OK) {
                        result[w] = s;
                        break;
                    }
                    redone[w] += child.ls_fallback_groups;
                }
                // every search ends with a read-back on its stream; after a failure, drain what was queued
                if (result[w] != ADMMQ_OK) (void)hipStreamSynchronize(child.stream);
            };
            std::vector<std::thread> helpers;
            std::vector<int> inline_share;
            for (int w = 1; w < workers; ++w) {
                try {
                    helpers.emplace_back(run, w);
                } catch (...) {
                    inline_share.push_back(w);          // no thread to be had: this share runs here, afterwards
                }
            }
            run(0);
            for (int w : inline_share) run(w);
            for (auto &h : helpers) h.join();
            ctx->ls_fallback_groups = 0;
            for (int w = 0; w < workers; ++w) {
                ADMMQ_TRY(result[w]);
                ctx->ls_fallback_groups += redone[w];
            }
        } else {
            int redone_all = 0;
            for (int i = 0; i < count; ++i) {
                const admmq_layer &l = L[i];
                admmq_arena_reset_transient(ctx);
                double drop = 0.0;
                ADMMQ_TRY(local_search_core(ctx, H, lambda, l.W0, n, l.p, l.ldw, l.bits, grp[i], l.scales, l.zeros,
                                            l.codes, plan, sched->seed, nullptr, &moves[i], &drop));
                redone_all += ctx->ls_fallback_groups;
            }
            ctx->ls_fallback_groups = redone_all;
        }
        ms_ls = t_phase.stop();
        if (want)
            for (int i = 0; i < count; ++i) stats[i].ls_moves = moves[i];
        if (want_obj) {
            for (int i = 0; i < count; ++i) {
                const admmq_layer &l = L[i];
                admmq_arena_reset_transient(ctx);
                float *E = nullptr, *tmp = nullptr;
                double *jd = nullptr;
                ADMMQ_TRY(take(ctx, E, (size_t)n * l.p));
                ADMMQ_TRY(take(ctx, tmp, (size_t)n * l.p));
                ADMMQ_TRY(take(ctx, jd, 2));
                ADMMQ_TRY(admmq_k_quant_error(ctx, l.W0, l.ldw, l.codes, n, l.p, grp[i], l.scales, l.zeros, l.bits, 0, E));
                ADMMQ_TRY(objectives_core(ctx, H, lambda, n, l.p, E, tmp, jd, &stats[i].j_damp, &stats[i].j_recon));
            }
        }
    }
    const float ms_all = want ? t_total.stop() : 0.f;
    prof_collect(ctx, prof_ms, prof_cnt);
    if (want) {
        for (int i = 0; i < count; ++i) {
            admmq_stats &st = stats[i];
            st.ms_gemm = prof_ms[ADMMQ_TAG_GEMM];       st.n_gemm = prof_cnt[ADMMQ_TAG_GEMM];
            st.ms_tridiag = prof_ms[ADMMQ_TAG_TRIDIAG]; st.n_tridiag = prof_cnt[ADMMQ_TAG_TRIDIAG];
            st.ms_project = prof_ms[ADMMQ_TAG_PROJECT]; st.n_project = prof_cnt[ADMMQ_TAG_PROJECT];
            st.ms_ls_apply = prof_ms[ADMMQ_TAG_LS_APPLY]; st.n_ls_apply = prof_cnt[ADMMQ_TAG_LS_APPLY];
            st.ms_gemm_project = 0.f;
            st.n_gemm_project = 0;
            st.ms_setup = ms_setup;
            st.ms_factor = ms_factor;
            st.ms_admm = ms_admm;
            st.ms_local_search = ms_ls;
            st.ms_total = ms_all;
        }
    }
    admmq_arena_reset_transient(ctx);
    return ADMMQ_OK;
}

// The loop hands rho_t and its reciprocal to the kernels in fp32, and the dual V = rho_t (W - D) is an fp32 array:
// a schedule whose last penalty leaves [1e-30, 1e30] would turn them into 0, inf or NaN without any error.
bool penalty_range_ok(const admmq_schedule *s) {
    const double last = log(s->rho0) + (double)s->T * log(s->gamma);
    return s->rho0 >= 1e-30 && last <= log(1e30);
}

bool schedule_ok(const admmq_schedule *s) {
    return s->T >= 1 && s->T <= (1 << 20) && s->rho0 > 0.0 && s->gamma >= 1.0 && isfinite(s->rho0) &&
           isfinite(s->gamma) && penalty_range_ok(s) && s->damp >= 0.0 && isfinite(s->damp) && s->ls_rounds >= 0 &&
           s->ls_batches >= 0 && s->ls_pairs >= 0 &&
           s->refresh_iter >= -1 && s->quiet_stop >= 0 && s->clip_points >= 0 && s->clip_points <= 100000 &&
           (s->clip_points == 0 || (s->clip_shrink >= 0.0 && s->clip_shrink < 1.0));
}

}  // namespace

extern "C" admmq_status admmq_quantize_layer(admmq_ctx *ctx, const float *H, const float *W0, int64_t n, int64_t p,
                                             int64_t ldw, int32_t bits, int32_t group_size,
                                             const admmq_schedule *sched, uint8_t *codes, float *scales, float *zeros,
                                             admmq_stats *stats) {
    if (!ctx || !sched || !codes || !scales || !zeros) return ADMMQ_ERR_NULL;
    ADMMQ_TRY(check_layer_args(H, W0, n, p, ldw, bits, group_size));
    if (!schedule_ok(sched)) return ADMMQ_ERR_PARAM;
    if (ctx->device < 0) return ADMMQ_ERR_DEVICE;
    ADMMQ_HIP(hipSetDevice(ctx->device));
    Projection pj = {0, bits, group_size > 0 ? group_size : n, scales, zeros, nullptr, nullptr, nullptr};
    return admmq_guarded([&] { return quantize_core(ctx, H, W0, n, p, ldw, pj, sched, codes, stats); });
}

extern "C" admmq_status admmq_quantize_layers(admmq_ctx *ctx, const float *H, int64_t n, const admmq_layer *layers,
                                              int32_t count, const admmq_schedule *sched, admmq_stats *stats) {
    if (!ctx || !sched || !layers || !H) return ADMMQ_ERR_NULL;
    if (count < 1 || count > 64) return ADMMQ_ERR_SHAPE;
    int64_t P = 0;
    for (int i = 0; i < count; ++i) {
        const admmq_layer &l = layers[i];
        if (!l.codes || !l.scales || !l.zeros) return ADMMQ_ERR_NULL;
        ADMMQ_TRY(check_layer_args(H, l.W0, n, l.p, l.ldw, l.bits, l.group_size));
        P += l.p;
    }
    if (P > (1 << 24)) return ADMMQ_ERR_SHAPE;
    if (!schedule_ok(sched) || sched->refresh_iter != -1) return ADMMQ_ERR_PARAM;
    if (ctx->device < 0) return ADMMQ_ERR_DEVICE;
    ADMMQ_HIP(hipSetDevice(ctx->device));
    return admmq_guarded([&] { return quantize_many_core(ctx, H, n, layers, count, sched, stats); });
}

extern "C" admmq_status admmq_grid_init_dual(admmq_ctx *ctx, const float *W0, int64_t n, int64_t p, int64_t ldw,
                                             const admmq_format *fmt) {
    if (!ctx || !W0) return ADMMQ_ERR_NULL;
    ADMMQ_TRY(check_format(fmt, n));
    if (fmt->kind != ADMMQ_FORMAT_DUAL_GRID) return ADMMQ_ERR_PARAM;
    ADMMQ_TRY(check_layer_args(W0, W0, n, p, ldw, fmt->bits, fmt->group_size));
    if (ctx->device < 0) return ADMMQ_ERR_DEVICE;
    ADMMQ_HIP(hipSetDevice(ctx->device));
    const int64_t g = fmt->group_size > 0 ? fmt->group_size : n;
    return admmq_k_dual_grid_init(ctx, W0, n, p, ldw, fmt->bits, g, fmt->flags, fmt->scales, fmt->zeros);
}

extern "C" admmq_status admmq_project_dual_format(admmq_ctx *ctx, const float *W, float *V, int64_t n, int64_t p,
                                                  const float *d, const admmq_format *fmt, double rho,
                                                  double rho_next, uint8_t *codes, float *B_out, float *Xq_out,
                                                  double *res_sq) {
    if (!ctx || !W || !V || !d || !B_out) return ADMMQ_ERR_NULL;
    ADMMQ_TRY(check_format(fmt, n));
    ADMMQ_TRY(check_layer_args(W, W, n, p, p, 2, fmt->group_size));
    if (!(rho > 0.0) || !(rho_next > 0.0) || !isfinite(rho) || !isfinite(rho_next)) return ADMMQ_ERR_PARAM;
    if (ctx->device < 0) return ADMMQ_ERR_DEVICE;
    ADMMQ_HIP(hipSetDevice(ctx->device));
    const int64_t g = fmt->group_size > 0 ? fmt->group_size : n;
    const size_t ng2 = 2 * (size_t)(n / g) * p;
    admmq_arena_reset_transient(ctx);
    ADMMQ_TRY(admmq_arena_reserve(ctx, admmq_align_up(ng2 * 4) + admmq_align_up((size_t)n * 4) + 8192));
    float *inv_scales = nullptr, *inv_d = nullptr;
    double *dev_res = nullptr;
    ADMMQ_TRY(take(ctx, inv_scales, ng2));
    ADMMQ_TRY(take(ctx, inv_d, (size_t)n));
    ADMMQ_TRY(take(ctx, dev_res, 2));
    if (fmt->kind == ADMMQ_FORMAT_CODEBOOK) ADMMQ_TRY(check_codebook(ctx, fmt->codebook, fmt->bits, p));
    if (fmt->kind == ADMMQ_FORMAT_DUAL_GRID) ADMMQ_TRY(admmq_k_recip(ctx, fmt->scales, inv_scales, (int64_t)ng2));
    ADMMQ_TRY(admmq_k_recip(ctx, d, inv_d, n));
    ADMMQ_TRY(admmq_k_fill_bytes(ctx, dev_res, 0, 16));
    const float rf = (float)rho;
    ADMMQ_TRY(admmq_k_project_format(ctx, fmt->kind, W, V, n, p, d, inv_d, fmt->bits, g, fmt->flags, fmt->scales,
                                     inv_scales, fmt->zeros, fmt->codebook, rf, 1.0f / rf, 1.0f / (float)rho_next, 1,
                                     codes, B_out, Xq_out, res_sq ? dev_res : nullptr));
    if (res_sq) ADMMQ_TRY(read_back(ctx, res_sq, dev_res, 8));
    admmq_arena_reset_transient(ctx);
    return ADMMQ_OK;
}

extern "C" admmq_status admmq_quantize_layer_format(admmq_ctx *ctx, const float *H, const float *W0, int64_t n,
                                                    int64_t p, int64_t ldw, const admmq_format *fmt,
                                                    const admmq_schedule *sched, uint8_t *codes, float *Wq,
                                                    admmq_stats *stats) {
    if (!ctx || !sched || !codes || !Wq) return ADMMQ_ERR_NULL;
    ADMMQ_TRY(check_format(fmt, n));
    ADMMQ_TRY(check_layer_args(H, W0, n, p, ldw, 2, fmt->group_size));
    if (!schedule_ok(sched) || sched->ls_rounds != 0 || sched->refresh_iter != -1 || sched->symmetric != 0 ||
        sched->clip_points != 0 || sched->quiet_stop != 0)
        return ADMMQ_ERR_PARAM;
    if (stats && stats->code_flips) return ADMMQ_ERR_PARAM;
    if (ctx->device < 0) return ADMMQ_ERR_DEVICE;
    ADMMQ_HIP(hipSetDevice(ctx->device));
    Projection pj = {fmt->kind, fmt->bits, fmt->group_size > 0 ? fmt->group_size : n, fmt->scales, fmt->zeros,
                     fmt->flags, fmt->codebook, Wq};
    return admmq_guarded([&] { return quantize_core(ctx, H, W0, n, p, ldw, pj, sched, codes, stats); });
}
