// One-off factorisation of the scaled, damped Hessian (Alg. 1 lines 1-3) and its per-iteration use.
//
// The paper diagonalises Hs once so that (Hs + rho I)^{-1} costs two products for any rho (Sec. 3.3).
// Here Hs = Q T Q^T is reduced only to TRIDIAGONAL form (Householder reflections, fp64):
//   (Hs + rho I)^{-1} Hs = Q (T + rho I)^{-1} T Q^T,
// and the middle factor is applied with an LDL^T solve that is linear in n per column.  The
// tridiagonal-to-diagonal stage of an eigensolver is serial and gains nothing here: the per-iteration
// cost stays two n x n x p products plus an O(np) pass.
//
// Both the reduction and the accumulation of Q^T are written as ONE streaming pass over the trailing
// matrix per step: the rank-2 (rank-1) update left pending by the previous step is applied while the
// matrix-vector product needed by the current step is formed, so each trailing element is read and
// written once per step.  One 64-lane wave owns one matrix row, so every reduction has a fixed order.
#include <stdlib.h>

#include "common.h"

namespace {

__device__ inline double wave_sum(double v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o, 64);
    return v;
}
__device__ inline double wave_bcast_sum(double v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// sum over a 1024-thread block, result in every thread
__device__ inline double block_sum_all(double v, double *sh) {
    v = wave_bcast_sum(v);
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    __syncthreads();
    if (lane == 0) sh[w] = v;
    __syncthreads();
    double r = 0.0;
    const int nw = blockDim.x >> 6;
    for (int q = 0; q < nw; ++q) r += sh[q];
    return r;
}

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

// ---- Householder reduction to tridiagonal form ----------------------------------------------
// Vector step k (single block).  Finishes step k-1 (w from p), forms row k of the virtually updated
// matrix, extracts T's entries and builds the reflector v_k = (1, x_tail/(alpha-beta)), tau_k.
__global__ __launch_bounds__(1024) void tridiag_vec_kernel(double *__restrict__ A, long n, long k,
                                                           const double *__restrict__ vprev,
                                                           double *__restrict__ vcur, double *__restrict__ w,
                                                           const double *__restrict__ p, double *__restrict__ xbuf,
                                                           double *__restrict__ tau, double *__restrict__ ta,
                                                           double *__restrict__ tb) {
    __shared__ double sh[16];
    const int tid = threadIdx.x;
    double *rowk = A + k * n;
    if (k > 0) {
        const double tp = tau[k - 1];
        double dot = 0.0;
        for (long i = k + tid; i < n; i += 1024) dot += p[i] * vprev[i];
        dot = block_sum_all(dot, sh);
        const double c = 0.5 * tp * tp * dot;
        for (long i = k + tid; i < n; i += 1024) w[i] = tp * p[i] - c * vprev[i];
        __syncthreads();
        const double vk = vprev[k], wk = w[k];
        for (long j = k + tid; j < n; j += 1024) xbuf[j] = rowk[j] - vk * w[j] - wk * vprev[j];
    } else {
        for (long j = tid; j < n; j += 1024) xbuf[j] = rowk[j];
    }
    __syncthreads();
    if (tid == 0) ta[k] = xbuf[k];
    if (k >= n - 1) {            // last row: nothing below the diagonal
        if (tid == 0) tb[k] = 0.0;
        return;
    }
    double sig = 0.0;
    for (long j = k + 2 + tid; j < n; j += 1024) {
        double x = xbuf[j];
        sig += x * x;
    }
    sig = block_sum_all(sig, sh);
    const double alpha = xbuf[k + 1];
    double beta, tk, scale;
    if (sig == 0.0) {
        beta = alpha; tk = 0.0; scale = 0.0;
    } else {
        const double nrm = sqrt(alpha * alpha + sig);
        beta = alpha >= 0.0 ? -nrm : nrm;
        tk = (beta - alpha) / beta;
        scale = 1.0 / (alpha - beta);
    }
    if (tid == 0) {
        tb[k] = beta;
        tau[k] = tk;
    }
    for (long j = k + 1 + tid; j < n; j += 1024) {
        double v = j == k + 1 ? 1.0 : xbuf[j] * scale;
        vcur[j] = v;
        rowk[j] = v;            // permanent home of the reflector: row k, right of the diagonal
    }
}

// Matrix step k: rows/cols >= k+1.  Applies the pending update of step k-1 (if any) and forms
// p[i] = sum_j A_new[i][j] * v[j].  One wave per row.
__global__ __launch_bounds__(256) void tridiag_mat_kernel(double *__restrict__ A, long n, long k, int pending,
                                                          const double *__restrict__ vprev,
                                                          const double *__restrict__ w,
                                                          const double *__restrict__ v, double *__restrict__ p) {
    const int lane = threadIdx.x & 63;
    const long i = k + 1 + (long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (i >= n) return;
    double *row = A + i * n;
    double acc = 0.0;
    if (pending) {
        const double vi = vprev[i], wi = w[i];
        for (long j = k + 1 + lane; j < n; j += 64) {
            double a = row[j] - vi * w[j] - wi * vprev[j];
            row[j] = a;
            acc += a * v[j];
        }
    } else {
        for (long j = k + 1 + lane; j < n; j += 64) acc += row[j] * v[j];
    }
    acc = wave_sum(acc);
    if (lane == 0) p[i] = acc;
}

// Closes the reduction: the last pending update (step n-3) on the trailing 2 x 2 block.
__global__ void tridiag_tail_kernel(const double *__restrict__ A, long n, const double *__restrict__ vprev,
                                    const double *__restrict__ p, const double *__restrict__ tau,
                                    double *__restrict__ ta, double *__restrict__ tb) {
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    const long k = n - 2;            // vprev = v_{n-3} lives on indices n-2, n-1
    const double tp = tau[n - 3];
    const double dot = p[k] * vprev[k] + p[k + 1] * vprev[k + 1];
    const double c = 0.5 * tp * tp * dot;
    const double w0 = tp * p[k] - c * vprev[k], w1 = tp * p[k + 1] - c * vprev[k + 1];
    ta[k] = A[k * n + k] - 2.0 * vprev[k] * w0;
    tb[k] = A[k * n + k + 1] - vprev[k] * w1 - w0 * vprev[k + 1];
    ta[k + 1] = A[(k + 1) * n + k + 1] - 2.0 * vprev[k + 1] * w1;
    tb[k + 1] = 0.0;
}

// ---- accumulation of R = Q^T = H_{n-3} ... H_0 -----------------------------------------------
__global__ void identity_kernel(double *__restrict__ R, long n) {
    long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= n * n) return;
    long i = idx / n;
    R[idx] = (idx - i * n == i) ? 1.0 : 0.0;
}

// Step k (k = n-3 ... 0), rows j and columns i >= k+2 of R:
//   pending (reflector k+1):  R[j][i] -= tau_{k+1} g'[j] v_{k+1}[i]
//   g[j] = sum_i R_new[j][i] v_k[i];   row k+1 of R is still a unit row, so g[k+1] = v_k[k+1] = 1.
// Reflector v_q is read from row q of A (entries right of the diagonal).
__global__ __launch_bounds__(256) void qform_kernel(double *__restrict__ R, const double *__restrict__ A, long n,
                                                    long k, int pending, const double *__restrict__ tau,
                                                    const double *__restrict__ gprev, double *__restrict__ g) {
    const int lane = threadIdx.x & 63;
    const long j = k + 1 + (long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (j >= n) return;
    if (j == k + 1) {
        if (lane == 0) g[j] = 1.0;
        return;
    }
    double *row = R + j * n;
    const double *vk = A + k * n;
    double acc = 0.0;
    if (pending) {
        const double *vp = A + (k + 1) * n;
        const double c = tau[k + 1] * gprev[j];
        for (long i = k + 2 + lane; i < n; i += 64) {
            double r = row[i] - c * vp[i];
            row[i] = r;
            acc += r * vk[i];
        }
    } else {
        for (long i = k + 2 + lane; i < n; i += 64) acc += row[i] * vk[i];
    }
    acc = wave_sum(acc);
    if (lane == 0) g[j] = acc;
}

// Applies the last pending reflector (k = 0): rows/cols >= 1.
__global__ __launch_bounds__(256) void qform_last_kernel(double *__restrict__ R, const double *__restrict__ A,
                                                         long n, const double *__restrict__ tau,
                                                         const double *__restrict__ g) {
    const int lane = threadIdx.x & 63;
    const long j = 1 + (long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (j >= n) return;
    double *row = R + j * n;
    const double c = tau[0] * g[j];
    for (long i = 1 + lane; i < n; i += 64) row[i] -= c * A[i];   // v_0 = row 0 of A
}

// Qt = fp32(R) row-major, Q = fp32(R^T) row-major, through a 32 x 32 LDS tile.
__global__ void emit_q_kernel(const double *__restrict__ R, long n, float *__restrict__ Q,
                              float *__restrict__ Qt) {
    __shared__ float tile[32][33];
    const int tx = threadIdx.x, ty = threadIdx.y;     // 32 x 8
    const long r0 = (long)blockIdx.y * 32, c0 = (long)blockIdx.x * 32;
    for (int r = ty; r < 32; r += 8) {
        long i = r0 + r, j = c0 + tx;
        float v = 0.f;
        if (i < n && j < n) {
            v = (float)R[i * n + j];
            Qt[i * n + j] = v;
        }
        tile[r][tx] = v;
    }
    __syncthreads();
    for (int r = ty; r < 32; r += 8) {
        long i = c0 + r, j = r0 + tx;                 // Q[i][j] = R[j][i]
        if (i < n && j < n) Q[i * n + j] = tile[tx][r];
    }
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
template <int C>
__global__ __launch_bounds__(256) void tridiag_apply_split_kernel(const double *__restrict__ ta,
                                                                  const double *__restrict__ tb,
                                                                  const double *__restrict__ dinv,
                                                                  const double *__restrict__ lfac, long n, long p,
                                                                  const float *Y, double *__restrict__ F, float *S) {
    constexpr int NS = 256 / C;               // segments per tile
    constexpr int SL = 32;                    // rows per segment
    constexpr int TR = NS * SL;               // rows per tile
    __shared__ double s_a[TR], s_b[TR + 1], s_l[TR + 1], s_di[TR];
    __shared__ double endf[2][NS][C], endP[2][NS][C];
    const int tid = threadIdx.x;
    const int c = tid % C, sg = tid / C;
    const long j = (long)blockIdx.x * C + c;
    const bool jok = j < p;
    const long ntile = (n + TR - 1) / TR;

    // ---------------- forward ----------------
    float ycur[SL + 2], ynext[SL + 2];
    auto load_y = [&](long t, float *dst) {
        const long a = t * TR + (long)sg * SL;
#pragma unroll
        for (int u = 0; u < SL + 2; ++u) {
            const long i = a - 1 + u;
            dst[u] = (jok && i >= 0 && i < n) ? Y[i * p + j] : 0.f;
        }
    };
    double carry = 0.0;                       // f of the row just above the current tile
    load_y(0, ycur);
    for (long t = 0; t < ntile; ++t) {
        const long i0 = t * TR;
        const int par = (int)(t & 1);
        // stage the tile's coefficients: s_a[r] = a_i, s_b[r] = b_{i-1}, s_l[r] = l_{i-1}, i = i0 + r
        for (int r = tid; r <= TR; r += 256) {
            const long i = i0 + r;
            if (r < TR) s_a[r] = i < n ? ta[i] : 0.0;
            s_b[r] = (i >= 1 && i < n) ? tb[i - 1] : 0.0;
            s_l[r] = (i >= 1 && i < n) ? lfac[i - 1] : 0.0;
        }
        __syncthreads();
        if (t + 1 < ntile) load_y(t + 1, ynext);
        double fl[SL], Pl[SL];
        {
            double f = 0.0, P = 1.0;
            const int r0 = sg * SL;
#pragma unroll
            for (int u = 0; u < SL; ++u) {
                const int r = r0 + u;
                const double z = s_b[r] * (double)ycur[u] + s_a[r] * (double)ycur[u + 1] +
                                 s_b[r + 1] * (double)ycur[u + 2];
                const double ml = -s_l[r];
                f = fma(ml, f, z);
                P = ml * P;
                fl[u] = f;
                Pl[u] = P;
            }
            endf[par][sg][c] = f;
            endP[par][sg][c] = P;
        }
        __syncthreads();
        double cin = carry, run = carry;
#pragma unroll
        for (int q = 0; q < NS; ++q) {
            if (q == sg) cin = run;
            run = fma(endP[par][q][c], run, endf[par][q][c]);
        }
        carry = run;
        {
            const long a = i0 + (long)sg * SL;
#pragma unroll
            for (int u = 0; u < SL; ++u) {
                const long i = a + u;
                if (jok && i < n) F[i * p + j] = fma(Pl[u], cin, fl[u]);
            }
        }
#pragma unroll
        for (int u = 0; u < SL + 2; ++u) ycur[u] = ynext[u];
    }

    // ---------------- backward ----------------
    __syncthreads();
    double gcur[SL], gnext[SL];
    auto load_f = [&](long t, double *dst) {
        const long a = t * TR + (long)sg * SL;
#pragma unroll
        for (int u = 0; u < SL; ++u) {
            const long i = a + u;
            dst[u] = (jok && i < n) ? F[i * p + j] : 0.0;
        }
    };
    carry = 0.0;                              // s of the row just below the current tile
    load_f(ntile - 1, gcur);
    for (long t = ntile - 1; t >= 0; --t) {
        const long i0 = t * TR;
        const int par = (int)(t & 1);
        // s_l[r] = l_i, s_di[r] = 1/delta_i, i = i0 + r
        for (int r = tid; r < TR; r += 256) {
            const long i = i0 + r;
            s_l[r] = i < n ? lfac[i] : 0.0;
            s_di[r] = i < n ? dinv[i] : 0.0;
        }
        __syncthreads();
        if (t > 0) load_f(t - 1, gnext);
        double sl[SL], Pl[SL];
        {
            double sv = 0.0, P = 1.0;
            const int r0 = sg * SL;
#pragma unroll
            for (int u = SL - 1; u >= 0; --u) {
                const int r = r0 + u;
                const double ml = -s_l[r];
                sv = fma(ml, sv, gcur[u] * s_di[r]);
                P = ml * P;
                sl[u] = sv;
                Pl[u] = P;
            }
            endf[par][sg][c] = sv;
            endP[par][sg][c] = P;
        }
        __syncthreads();
        double cin = carry, run = carry;
#pragma unroll
        for (int q = NS - 1; q >= 0; --q) {
            if (q == sg) cin = run;
            run = fma(endP[par][q][c], run, endf[par][q][c]);
        }
        carry = run;
        {
            const long a = i0 + (long)sg * SL;
#pragma unroll
            for (int u = 0; u < SL; ++u) {
                const long i = a + u;
                if (jok && i < n) S[i * p + j] = (float)fma(Pl[u], cin, sl[u]);
            }
        }
#pragma unroll
        for (int u = 0; u < SL; ++u) gcur[u] = gnext[u];
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

admmq_status admmq_k_factorize(admmq_ctx *ctx, const float *H, int64_t n, double lambda, const float *d,
                               double *A64, double *R64, double *vecs, float *Q, float *Qt, double *ta,
                               double *tb) {
    hipStream_t st = ctx->stream;
    const long N = (long)n;
    double *v0 = vecs, *v1 = vecs + N, *w = vecs + 2 * N, *pv = vecs + 3 * N, *xbuf = vecs + 4 * N,
           *tau = vecs + 5 * N, *g0 = vecs + 6 * N, *g1 = vecs + 7 * N;
    hipLaunchKernelGGL(build_scaled_kernel, dim3(blocks_for(N * N, 256)), dim3(256), 0, st, H, N, lambda, d, A64);
    if (N == 1) {
        // T = A, Q = 1
        hipLaunchKernelGGL(tridiag_vec_kernel, dim3(1), dim3(1024), 0, st, A64, N, 0L, v1, v0, w, pv, xbuf, tau, ta,
                           tb);
    } else if (N == 2) {
        hipLaunchKernelGGL(tridiag_vec_kernel, dim3(1), dim3(1024), 0, st, A64, N, 0L, v1, v0, w, pv, xbuf, tau, ta,
                           tb);
        // v_0 = (1) has tau = 0: the trailing 1 x 1 block is A[1][1] itself
        hipLaunchKernelGGL(tridiag_mat_kernel, dim3(1), dim3(256), 0, st, A64, N, 0L, 0, v1, w, v0, pv);
        hipLaunchKernelGGL(tridiag_vec_kernel, dim3(1), dim3(1024), 0, st, A64, N, 1L, v0, v1, w, pv, xbuf, tau, ta,
                           tb);
    } else {
        for (long k = 0; k <= N - 3; ++k) {
            double *vc = (k & 1) ? v1 : v0, *vp = (k & 1) ? v0 : v1;
            hipLaunchKernelGGL(tridiag_vec_kernel, dim3(1), dim3(1024), 0, st, A64, N, k, vp, vc, w, pv, xbuf, tau,
                               ta, tb);
            const long m = N - k - 1;
            hipLaunchKernelGGL(tridiag_mat_kernel, dim3(blocks_for(m, 4)), dim3(256), 0, st, A64, N, k, k > 0 ? 1 : 0,
                               vp, w, vc, pv);
        }
        double *vlast = ((N - 3) & 1) ? v1 : v0;
        hipLaunchKernelGGL(tridiag_tail_kernel, dim3(1), dim3(64), 0, st, A64, N, vlast, pv, tau, ta, tb);
    }
    ADMMQ_HIP(hipGetLastError());
    // R = Q^T
    hipLaunchKernelGGL(identity_kernel, dim3(blocks_for(N * N, 256)), dim3(256), 0, st, R64, N);
    if (N >= 3) {
        for (long k = N - 3; k >= 0; --k) {
            double *gc = (k & 1) ? g1 : g0, *gp = (k & 1) ? g0 : g1;
            const long m = N - k - 1;
            hipLaunchKernelGGL(qform_kernel, dim3(blocks_for(m, 4)), dim3(256), 0, st, R64, A64, N, k,
                               k < N - 3 ? 1 : 0, tau, gp, gc);
        }
        hipLaunchKernelGGL(qform_last_kernel, dim3(blocks_for(N - 1, 4)), dim3(256), 0, st, R64, A64, N, tau, g0);
    }
    dim3 tb32(32, 8), tg((unsigned)((N + 31) / 32), (unsigned)((N + 31) / 32));
    hipLaunchKernelGGL(emit_q_kernel, tg, tb32, 0, st, R64, N, Q, Qt);
    ADMMQ_HIP(hipGetLastError());
    return ADMMQ_OK;
}

admmq_status admmq_k_tridiag_factor(admmq_ctx *ctx, const double *ta, const double *tb, int64_t n,
                                    const double *rhos_dev, int count, double *dinv, double *lfac) {
    hipLaunchKernelGGL(tridiag_factor_kernel, dim3(blocks_for(count, 64)), dim3(64), 0, ctx->stream, ta, tb, (long)n,
                       rhos_dev, count, dinv, lfac);
    ADMMQ_HIP(hipGetLastError());
    return ADMMQ_OK;
}

admmq_status admmq_k_tridiag_apply(admmq_ctx *ctx, const double *ta, const double *tb, const double *dinv,
                                   const double *lfac, int64_t n, int64_t p, const float *Y, double *F,
                                   float *S) {
    // the widest column strip that still gives every CU a block
    int C = 64;
    if ((p + 63) / 64 < 256) C = 32;
    if ((p + 31) / 32 < 256) C = 16;
    static int forced = -1;
    if (forced < 0) {
        const char *e = getenv("ADMMQ_TRIDIAG_COLS");
        forced = e ? atoi(e) : 0;
    }
    if (forced == 16 || forced == 32 || forced == 64) C = forced;
    const unsigned nb = (unsigned)((p + C - 1) / C);
    if (C == 64)
        hipLaunchKernelGGL(tridiag_apply_split_kernel<64>, dim3(nb), dim3(256), 0, ctx->stream, ta, tb, dinv, lfac,
                           (long)n, (long)p, Y, F, S);
    else if (C == 32)
        hipLaunchKernelGGL(tridiag_apply_split_kernel<32>, dim3(nb), dim3(256), 0, ctx->stream, ta, tb, dinv, lfac,
                           (long)n, (long)p, Y, F, S);
    else
        hipLaunchKernelGGL(tridiag_apply_split_kernel<16>, dim3(nb), dim3(256), 0, ctx->stream, ta, tb, dinv, lfac,
                           (long)n, (long)p, Y, F, S);
    ADMMQ_HIP(hipGetLastError());
    return ADMMQ_OK;
}
