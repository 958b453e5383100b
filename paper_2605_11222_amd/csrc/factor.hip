// One-off factorisation of the scaled, damped Hessian (Alg. 1 lines 1-3) and its per-iteration use.
//
// The paper diagonalises Hs once so that (Hs + rho I)^{-1} costs two products for any rho (Sec. 3.3).
// Here Hs = Q T Q^T is reduced only to TRIDIAGONAL form (Householder reflections, fp64):
//   (Hs + rho I)^{-1} Hs = Q (T + rho I)^{-1} T Q^T,
// and the middle factor is applied with an LDL^T solve that is linear in n per column.  The
// tridiagonal-to-diagonal stage of an eigensolver is serial and gains nothing here: the per-iteration
// cost stays two n x n x p products plus an O(np) pass.
//
// The reduction itself lives in householder.hip; this file holds the scaling, the LDL^T factors of
// T + rho I for the whole penalty schedule, and the per-iteration tridiagonal solve.
#include <stdlib.h>

#include "common.h"

namespace {

// d_i = fp32(sqrt(H_ii + lambda)), inv_d = 1/d (fp32), flags[0] += 1 for a non-positive diagonal
__global__ void scaling_kernel(const float *__restrict__ H, long n, double lambda, int precondition,
                               float *__restrict__ d, float *__restrict__ inv_d, double *__restrict__ flags) {
    long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    double v = (double)H[i * n + i] + lambda;
    if (!(v > 0.0)) {
        atomicAdd(flags, 1.0);
        v = 1.0;
    }
    float di = precondition ? (float)sqrt(v) : 1.0f;
    d[i] = di;
    inv_d[i] = __fdiv_rn(1.0f, di);
}

// A[i][j] = (H[i][j] + lambda [i==j]) / (d_i d_j) in fp64, from the fp32-rounded d that the rest of the
// solver uses (so that the scaled problem is exactly consistent with the projection's Sigma).
__global__ void build_scaled_kernel(const float *__restrict__ H, long n, double lambda,
                                    const float *__restrict__ d, double *__restrict__ A) {
    long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= n * n) return;
    long i = idx / n, j = idx - i * n;
    // symmetrise on the way in: the two triangles of an accumulated Hessian agree, but a caller's may not
    double h = 0.5 * ((double)H[idx] + (double)H[j * n + i]);
    if (i == j) h += lambda;
    A[idx] = h / ((double)d[i] * (double)d[j]);
}

// ---- (T + rho I) = L D L^T for a whole schedule of rho, one thread per rho -------------------
__global__ void tridiag_factor_kernel(const double *__restrict__ ta, const double *__restrict__ tb, long n,
                                      const double *__restrict__ rhos, int count, double *__restrict__ dinv,
                                      double *__restrict__ lfac) {
    int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= count) return;
    const double rho = rhos[t];
    double *di = dinv + (long)t * n, *lf = lfac + (long)t * n;
    double delta = ta[0] + rho;
    for (long i = 0; i < n; ++i) {
        const double inv = 1.0 / delta;
        di[i] = inv;
        if (i + 1 < n) {
            const double b = tb[i];
            const double l = b * inv;
            lf[i] = l;
            delta = ta[i + 1] + rho - l * b;
        } else {
            lf[i] = 0.0;
        }
    }
}

// S = (T + rho I)^{-1} T Y, all columns.
//   z_i = b_{i-1} y_{i-1} + a_i y_i + b_i y_{i+1}
//   f_i = z_i - l_{i-1} f_{i-1}                         (forward recurrence)
//   s_i = f_i / delta_i - l_i s_{i+1}                   (backward recurrence)
// A first-order linear recurrence splits exactly: over a segment of rows a..b with incoming value c,
//   f_i = ft_i + P_i c,  ft = the recurrence started from 0,  P_i = prod_{k=a..i} (-l_{k-1}).
// A block owns C columns and walks the rows in tiles of TR = NS*SL rows; thread (s, c) runs the local
// recurrence of segment s (SL rows) of column c in registers, all NS segments at once; the NS segment
// ends are then chained (NS short steps, done redundantly by every thread, so one barrier per tile
// suffices) and each thread corrects its own rows.  The sequential depth per tile is SL + NS instead
// of TR.  Row coefficients, which all columns share, are staged in LDS once per tile.
// The forward pass keeps only the value of f that enters each tile (`carries`, [tiles][p] doubles); the
// backward pass, tile by tile from the bottom, forms the tile's f again from Y and consumes it in registers.
// HBM traffic: Y twice, S once = 12 B per element (with f stored in fp64 in between it was 24).
// S must not be Y: the backward pass reads Y rows next to tiles it has already written.
// (Measured at n = p = 4096: 0.120 ms; it is bound by the latency of its dependent steps with one block per
// compute unit, not by bytes: 1024-thread blocks of 8-row segments take 0.152 ms.)
template <int C, int NT, int SL>
__global__ __launch_bounds__(NT) void tridiag_apply_split_kernel(const double *__restrict__ ta,
                                                                  const double *__restrict__ tb,
                                                                  const double *__restrict__ dinv,
                                                                  const double *__restrict__ lfac, long n, long p,
                                                                  const float *__restrict__ Y,
                                                                  double *__restrict__ carries,
                                                                  float *__restrict__ S,
                                                                  unsigned *__restrict__ amax_out) {
    constexpr int NS = NT / C;                // segments per tile (SL rows each)
    unsigned smax = 0;                        // largest |S| written, as the float's bit pattern
    constexpr int TR = NS * SL;               // rows per tile
    // the row coefficients of a tile, in two buffers: tile t lives in buffer t & 1 (both passes), and the next
    // tile's are requested at the start of a tile and stored at its end, so no pass waits for them
    __shared__ double s_a[2][TR], s_b[2][TR + 1], s_l[2][TR + 1], s_di[2][TR];
    __shared__ double endf[2][NS][C], endP[2][NS][C];
    const int tid = threadIdx.x;
    const int c = tid % C, sg = tid / C;
    // blocks whose ids are congruent mod 8 run on the same XCD: they get neighbouring strips, so that the pieces of a
    // 128-byte line of Y that belong to two strips are asked for by the same L2
    long strip = blockIdx.x;
    if ((gridDim.x & 7) == 0) strip = (long)(blockIdx.x & 7) * (gridDim.x >> 3) + (blockIdx.x >> 3);
    const long j = strip * C + c;
    const bool jok = j < p;
    const long ntile = (n + TR - 1) / TR;

    float ycur[SL + 2], ynext[SL + 2];
    auto load_y = [&](long t, float *dst) {
        const long a = t * TR + (long)sg * SL;
#pragma unroll
        for (int u = 0; u < SL + 2; ++u) {
            const long i = a - 1 + u;
            dst[u] = (jok && i >= 0 && i < n) ? Y[i * p + j] : 0.f;
        }
    };
    // s_a[r] = a_i, s_b[r] = b_{i-1}, s_l[r] = l_{i-1}, s_di[r] = 1/delta_i, i = i0 + r (s_l[r + 1] = l_i)
    constexpr int KR = (TR + NT) / NT;        // coefficient rows per thread (TR + 1 rows over NT threads)
    double q_a[KR], q_b[KR], q_l[KR], q_d[KR];
    auto coef_load = [&](long i0) {
#pragma unroll
        for (int k = 0; k < KR; ++k) {
            const int r = tid + k * NT;
            const long i = i0 + r;
            const bool row = r < TR && i < n, link = r <= TR && i >= 1 && i < n;
            q_a[k] = row ? ta[i] : 0.0;
            q_d[k] = row ? dinv[i] : 0.0;
            q_b[k] = link ? tb[i - 1] : 0.0;
            q_l[k] = link ? lfac[i - 1] : 0.0;
        }
    };
    auto coef_store = [&](int buf) {
#pragma unroll
        for (int k = 0; k < KR; ++k) {
            const int r = tid + k * NT;
            if (r < TR) {
                s_a[buf][r] = q_a[k];
                s_di[buf][r] = q_d[k];
            }
            if (r <= TR) {
                s_b[buf][r] = q_b[k];
                s_l[buf][r] = q_l[k];
            }
        }
    };
    // the segment's forward recurrence from zero: fl[u] = local f, Pl[u] = product of the -l up to row u
    auto forward_local = [&](int cb, const float *y, double *fl, double *Pl) {
        double f = 0.0, P = 1.0;
        const int r0 = sg * SL;
#pragma unroll
        for (int u = 0; u < SL; ++u) {
            const int r = r0 + u;
            const double z = fma(s_b[cb][r + 1], (double)y[u + 2], fma(s_a[cb][r], (double)y[u + 1], s_b[cb][r] * (double)y[u]));
            const double ml = -s_l[cb][r];
            f = fma(ml, f, z);
            P = ml * P;
            fl[u] = f;
            Pl[u] = P;
        }
    };

    // ---------------- forward: only the value of f entering each tile is kept ----------------
    double carry = 0.0;                       // f of the row just above the current tile
    coef_load(0);
    load_y(0, ycur);
    coef_store(0);
    __syncthreads();
    for (long t = 0; t < ntile; ++t) {
        const int par = (int)(t & 1), cb = par;
        if (t + 1 < ntile) {
            load_y(t + 1, ynext);
            coef_load((t + 1) * TR);
        }
        if (jok && sg == 0) carries[t * p + j] = carry;
        {
            double fl[SL], Pl[SL];
            forward_local(cb, ycur, fl, Pl);
            endf[par][sg][c] = fl[SL - 1];
            endP[par][sg][c] = Pl[SL - 1];
        }
        if (t + 1 < ntile) coef_store(cb ^ 1);      // its last readers passed the barrier of the tile before
        __syncthreads();
        double run = carry;
#pragma unroll
        for (int q = 0; q < NS; ++q) run = fma(endP[par][q][c], run, endf[par][q][c]);
        carry = run;
#pragma unroll
        for (int u = 0; u < SL + 2; ++u) ycur[u] = ynext[u];
    }

    // ---------------- backward: each tile's f is formed again from Y, then consumed in registers --------
    // (the last tile's coefficients are still in their buffer)
    __syncthreads();
    double below = 0.0;                       // s of the row just below the current tile
    load_y(ntile - 1, ycur);
    for (long t = ntile - 1; t >= 0; --t) {
        const long i0 = t * TR;
        const int cb = (int)(t & 1);
        if (t > 0) {
            load_y(t - 1, ynext);
            coef_load((t - 1) * TR);
        }
        const double tile_in = jok ? carries[t * p + j] : 0.0;
        double fl[SL], Pl[SL];
        forward_local(cb, ycur, fl, Pl);
        endf[0][sg][c] = fl[SL - 1];
        endP[0][sg][c] = Pl[SL - 1];
        __syncthreads();
        {
            double cin = tile_in, run = tile_in;
#pragma unroll
            for (int q = 0; q < NS; ++q) {
                if (q == sg) cin = run;
                run = fma(endP[0][q][c], run, endf[0][q][c]);
            }
#pragma unroll
            for (int u = 0; u < SL; ++u) fl[u] = fma(Pl[u], cin, fl[u]);      // the f of rows a .. a + SL - 1
        }
        {
            double sv = 0.0, P = 1.0;
            const int r0 = sg * SL;
#pragma unroll
            for (int u = SL - 1; u >= 0; --u) {
                const int r = r0 + u;
                const double ml = -s_l[cb][r + 1];                             // l_i
                sv = fma(ml, sv, fl[u] * s_di[cb][r]);
                P = ml * P;
                fl[u] = sv;
                Pl[u] = P;
            }
            endf[1][sg][c] = sv;
            endP[1][sg][c] = P;
        }
        if (t > 0) coef_store(cb ^ 1);              // read last by the tile above this one's predecessor: done
        __syncthreads();
        double cin = below, run = below;
#pragma unroll
        for (int q = NS - 1; q >= 0; --q) {
            if (q == sg) cin = run;
            run = fma(endP[1][q][c], run, endf[1][q][c]);
        }
        below = run;
        {
            const long a = i0 + (long)sg * SL;
#pragma unroll
            for (int u = 0; u < SL; ++u) {
                const long i = a + u;
                if (jok && i < n) {
                    const float sv = (float)fma(Pl[u], cin, fl[u]);
                    S[i * p + j] = sv;
                    smax = max(smax, __float_as_uint(fabsf(sv)));
                }
            }
        }
#pragma unroll
        for (int u = 0; u < SL + 2; ++u) ycur[u] = ynext[u];
    }
    if (amax_out) {
        // for the split-fp16 products: the largest |S| of the whole solve, one atomic per wave
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) smax = max(smax, (unsigned)__shfl_xor((int)smax, o));
        // (most waves find a value at least as large already there and skip the atomic: thousands of atomics on
        // one address would take longer than the pass itself)
        if ((threadIdx.x & 63) == 0 && smax > __atomic_load_n(amax_out, __ATOMIC_RELAXED)) atomicMax(amax_out, smax);
    }
}

inline unsigned blocks_for(long count, int bs) { return (unsigned)((count + bs - 1) / bs); }

}  // namespace

admmq_status admmq_k_scaling(admmq_ctx *ctx, const float *H, int64_t n, double lambda, int precondition, float *d,
                             float *inv_d, double *dev_flags) {
    hipLaunchKernelGGL(scaling_kernel, dim3(blocks_for(n, 256)), dim3(256), 0, ctx->stream, H, (long)n, lambda,
                       precondition, d, inv_d, dev_flags);
    ADMMQ_HIP(hipGetLastError());
    return ADMMQ_OK;
}

admmq_status admmq_k_householder(admmq_ctx *ctx, double *A64, int64_t n, double *R64, double *vecs, float *Q,
                                 float *Qt, double *ta, double *tb);
admmq_status admmq_k_band_reduce(admmq_ctx *ctx, double *A64, int64_t n, double *R64, double *vecs, float *Q, float *Qt,
                                 double *bd);

// The form of the factorisation for an n x n Hessian.  The band form costs a fraction of the one-stage tridiagonal
// reduction (block reflectors: one pass over the trailing matrix per 16 columns instead of one per column: 34 ms
// against 92 ms at n = 4096, 0.38 s against 1.0 s at n = 12288), but its per-iteration solve is 16 x 16 block
// elimination on the fp64 matrix cores, about twice the cost of the scalar recurrence of the tridiagonal form
// (0.15 against 0.08 ms at 4096 x 4096).  From n = 4096 on the reduction's saving outweighs that for any schedule
// of fewer than about 800 iterations; below, the chain of the tridiagonal form is short anyway.
// ADMMQ_FACTOR=band / tridiag forces one form (read at every call).
bool admmq_factor_is_band(int64_t n) {
    const char *e = getenv("ADMMQ_FACTOR");
    if (e && e[0] == 't') return false;
    if (e && e[0] == 'b') return true;
    return n >= 4096;
}

// band != NULL: reduction to band form (ta, tb unused); else to tridiagonal form
admmq_status admmq_k_factorize(admmq_ctx *ctx, const float *H, int64_t n, double lambda, const float *d,
                               double *A64, double *R64, double *vecs, float *Q, float *Qt, double *ta,
                               double *tb, double *band) {
    const long N = (long)n;
    hipLaunchKernelGGL(build_scaled_kernel, dim3(blocks_for(N * N, 256)), dim3(256), 0, ctx->stream, H, N, lambda, d,
                       A64);
    ADMMQ_HIP(hipGetLastError());
    if (band) return admmq_k_band_reduce(ctx, A64, n, R64, vecs, Q, Qt, band);
    return admmq_k_householder(ctx, A64, n, R64, vecs, Q, Qt, ta, tb);
}

admmq_status admmq_k_tridiag_factor(admmq_ctx *ctx, const double *ta, const double *tb, int64_t n,
                                    const double *rhos_dev, int count, double *dinv, double *lfac) {
    hipLaunchKernelGGL(tridiag_factor_kernel, dim3(blocks_for(count, 64)), dim3(64), 0, ctx->stream, ta, tb, (long)n,
                       rhos_dev, count, dinv, lfac);
    ADMMQ_HIP(hipGetLastError());
    return ADMMQ_OK;
}

admmq_status admmq_k_tridiag_apply(admmq_ctx *ctx, const double *ta, const double *tb, const double *dinv,
                                   const double *lfac, int64_t n, int64_t p, const float *Y, double *carries,
                                   float *S, unsigned *amax_out) {
    if ((const float *)S == Y) return ADMMQ_ERR_PARAM;       // the second pass reads Y again: not in place
    // the widest column strip that still gives every CU a block
    int C = 64;
    if ((p + 63) / 64 < 256) C = 32;
    if ((p + 31) / 32 < 256) C = 16;
    if ((p + 15) / 16 < 128) C = 8;           // measured at p = 1024: 0.081 ms against 0.107 ms with 16 columns
    static int forced = -1;
    if (forced < 0) {
        const char *e = getenv("ADMMQ_TRIDIAG_COLS");
        forced = e ? atoi(e) : 0;
    }
    if (forced == 8 || forced == 16 || forced == 32 || forced == 64) C = forced;
    const unsigned nb = (unsigned)((p + C - 1) / C);
    // 16-column strips: 512 threads run 32 segments of 16 rows (two waves per SIMD hide the latency of the dependent
    // steps and of the LDS reads; 512-row tiles as before): 80 us against 100 us with 256 threads x 32 rows at
    // n = p = 4096; 8-row segments or 1024 threads are slower (longer chain of segment ends, fewer registers)
    static int narrow = -1;
    if (narrow < 0) {
        const char *e = getenv("ADMMQ_TRIDIAG_THREADS");
        narrow = (e && atoi(e) == 256) ? 1 : 0;
    }
    if (C == 16 && !narrow) {
        hipLaunchKernelGGL((tridiag_apply_split_kernel<16, 512, 16>), dim3(nb), dim3(512), 0, ctx->stream, ta, tb, dinv,
                           lfac, (long)n, (long)p, Y, carries, S, amax_out);
        ADMMQ_HIP(hipGetLastError());
        return ADMMQ_OK;
    }
    if (C == 8)
        hipLaunchKernelGGL((tridiag_apply_split_kernel<8, 256, 32>), dim3(nb), dim3(256), 0, ctx->stream, ta, tb, dinv,
                           lfac, (long)n, (long)p, Y, carries, S, amax_out);
    else if (C == 64)
        hipLaunchKernelGGL((tridiag_apply_split_kernel<64, 256, 32>), dim3(nb), dim3(256), 0, ctx->stream, ta, tb, dinv,
                           lfac, (long)n, (long)p, Y, carries, S, amax_out);
    else if (C == 32)
        hipLaunchKernelGGL((tridiag_apply_split_kernel<32, 256, 32>), dim3(nb), dim3(256), 0, ctx->stream, ta, tb, dinv,
                           lfac, (long)n, (long)p, Y, carries, S, amax_out);
    else
        hipLaunchKernelGGL((tridiag_apply_split_kernel<16, 256, 32>), dim3(nb), dim3(256), 0, ctx->stream, ta, tb, dinv,
                           lfac, (long)n, (long)p, Y, carries, S, amax_out);
    ADMMQ_HIP(hipGetLastError());
    return ADMMQ_OK;
}
