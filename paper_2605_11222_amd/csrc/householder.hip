// Reduction of the scaled Hessian to tridiagonal form, Hs = Q T Q^T, and accumulation of Q^T, in fp64.
// This is the "computed once" part of the W-update (paper Sec. 3.3, Alg. 1 line 3).
//
// Phase 1 (panels of NB Householder reflectors):
//   for each column k of the panel          start : row k of the matrix as it would look after the
//                                                   panel's earlier updates -> T entries, reflector v_k
//                                           mat   : p = A v_k over the trailing matrix (READ ONLY: the
//                                                   panel's updates are not applied to A yet)
//                                           finish: p corrected by the panel's earlier (v, w) pairs,
//                                                   w_k = tau (p - tau/2 (p.v) v)
//   once per panel                          update: A -= V W^T + W V^T   (rank-2NB, read+write once)
//   so every column costs one read of the trailing matrix and every panel one read+write.
// Phase 2: R = Q^T = H_{n-3} ... H_0 is accumulated block by block from the last reflectors to the
//   first, each block of NB reflectors in compact WY form  H_k0 ... H_k0+nb-1 = I - V T V^T :
//   R <- R (I - V T^T V^T) = R - ((R V) T^T) V^T, two tall-skinny products per block, so R is read and
//   written once per NB reflectors.
// Every reduction has a fixed order (one wave or one thread per output), so the result is reproducible.
#include "common.h"

namespace {

constexpr int NB = 32;

__device__ inline double wave_sum(double v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o, 64);
    return v;
}
// load that is coherent across the chip (bypasses the per-CU cache): used by the block that finishes last
__device__ inline double coherent_load(const double *ptr) {
    return __hip_atomic_load(ptr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// ---- phase 1 -------------------------------------------------------------------------------------
// Scalars shared between the two kernels of a column (device doubles):
//   sc[0] unused, sc[1] = 1/(alpha - beta) of the current reflector,
//   sc[2 + 2q] = W_q . v,  sc[3 + 2q] = V_q . v   for the earlier panel slots q.
// Block-level partial sums are combined by the block that finishes last, in index order, so every
// reduction has a fixed order although many blocks take part.
enum { SC_SCALE = 1, SC_DOTS = 2, SC_COUNT = 2 + 2 * NB };
constexpr int ROW_CHUNK = 256;       // elements per block of tri_row_kernel (one per thread)
constexpr int PART_W = 2 * NB + 1;   // partials per block: squared norm + 2 dots per slot

__device__ inline bool last_block_done(unsigned *counter, unsigned nblocks) {
    __shared__ int is_last;
    __threadfence();
    __syncthreads();
    if (threadIdx.x == 0) is_last = (atomicAdd(counter, 1u) == nblocks - 1) ? 1 : 0;
    __syncthreads();
    if (is_last) __threadfence();
    return is_last != 0;
}

// Column k, panel slot c.  With do_finish: w of column k-1 (slot c-1) from its corrected product p'.
// With do_start: row k of the matrix as the panel's earlier updates would leave it (xbuf), its squared
// tail norm and its dots with the earlier W_q, V_q; the last block turns these into the reflector's
// scalars.  The normalised reflector itself is written by tri_mat_kernel.
// One thread per element of the row; the per-slot dots are shared out over the block's four waves.
__global__ __launch_bounds__(256) void tri_row_kernel(const double *__restrict__ A, long n, long k, int c,
                                                      int do_finish, int do_start, const double *__restrict__ Vp,
                                                      double *__restrict__ Wp, const double *__restrict__ pbuf,
                                                      double *__restrict__ xbuf, double *__restrict__ tau,
                                                      double *__restrict__ ta, double *__restrict__ tb,
                                                      double *__restrict__ sc, double *__restrict__ part,
                                                      unsigned *__restrict__ counter,
                                                      const double *__restrict__ part2, int nparts2) {
    __shared__ double vk[NB], wk[NB];
    __shared__ double xs[ROW_CHUNK];
    __shared__ double red[4][PART_W];
    __shared__ double tot[PART_W];
    __shared__ double scale_sh;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const long j = k + (long)blockIdx.x * ROW_CHUNK + tid;
    const bool ok = j < n;
    double wnew = 0.0, wk_last = 0.0;
    if (do_finish) {
        const int cf = c - 1;
        // p'.v of column k-1: the block partials of its tri_mat_kernel, added in a fixed order
        double ds = 0.0;
        for (int b = tid; b < nparts2; b += 256) ds += part2[b];
        xs[tid] = ds;
        __syncthreads();
        for (int h = 128; h > 0; h >>= 1) {
            if (tid < h) xs[tid] += xs[tid + h];
            __syncthreads();
        }
        const double pdotv = xs[0];
        __syncthreads();
        const double tp = tau[k - 1];
        const double cc = 0.5 * tp * tp * pdotv;
        const double *vprev = Vp + (long)cf * n;
        if (ok) {
            wnew = tp * pbuf[j] - cc * vprev[j];
            Wp[(long)cf * n + j] = wnew;
        }
        wk_last = tp * pbuf[k] - cc * vprev[k];
    }
    if (!do_start) return;
    if (tid < c) {
        vk[tid] = Vp[(long)tid * n + k];
        wk[tid] = (tid == c - 1) ? wk_last : Wp[(long)tid * n + k];
    }
    __syncthreads();
    // This element's entries of every earlier slot are loaded once (all loads in flight together) and serve
    // both the row update and the dots below.  Slots >= c are predicated off; c is uniform.
    const long jj = ok ? j : n - 1;              // clamped index: loads stay in bounds, results unused
    double wq[NB], vq[NB];
#pragma unroll
    for (int q = 0; q < NB; ++q) {
        if (q < c) {
            wq[q] = (q == c - 1) ? wnew : Wp[(long)q * n + jj];
            vq[q] = Vp[(long)q * n + jj];
        } else {
            wq[q] = 0.0;
            vq[q] = 0.0;
        }
    }
    double x = ok ? A[k * n + j] : 0.0;
#pragma unroll
    for (int q = 0; q < NB; ++q)
        if (q < c) x -= vk[q] * wq[q] + wk[q] * vq[q];
    if (ok) xbuf[j] = x;
    const double xt = (ok && j >= k + 2) ? x : 0.0;      // the reflector's tail
    // block partials: [0] squared tail norm, [1+2q] W_q . x_tail, [2+2q] V_q . x_tail
    const int nred = 1 + 2 * c;
    {
        const double s0 = wave_sum(xt * xt);
        if (lane == 0) red[wave][0] = s0;
    }
#pragma unroll
    for (int q = 0; q < NB; ++q) {
        if (q < c) {
            const double sw = wave_sum(wq[q] * xt);
            const double sv = wave_sum(vq[q] * xt);
            if (lane == 0) {
                red[wave][1 + 2 * q] = sw;
                red[wave][2 + 2 * q] = sv;
            }
        }
    }
    __syncthreads();
    if (tid < nred)
        part[(long)blockIdx.x * PART_W + tid] = (red[0][tid] + red[1][tid]) + (red[2][tid] + red[3][tid]);
    if (!last_block_done(counter, gridDim.x)) return;
    // add the block partials in block order; four blocks' worth is fetched per round trip by the whole block
    double run = 0.0;
    for (unsigned b0 = 0; b0 < gridDim.x; b0 += 4) {
        for (int e = tid; e < 4 * PART_W; e += 256) {
            const unsigned b = b0 + e / PART_W;
            const int r = e % PART_W;
            red[e / PART_W][r] = (b < gridDim.x && r < nred) ? coherent_load(part + (long)b * PART_W + r) : 0.0;
        }
        __syncthreads();
        if (tid < nred) run += ((red[0][tid] + red[1][tid]) + red[2][tid]) + red[3][tid];
        __syncthreads();
    }
    if (tid < nred) tot[tid] = run;
    __syncthreads();
    if (tid == 0) {
        const double sig = tot[0];
        const double alpha = coherent_load(xbuf + k + 1);
        double beta, tk, scale;
        if (sig == 0.0) {
            beta = alpha; tk = 0.0; scale = 0.0;
        } else {
            const double nrm = sqrt(alpha * alpha + sig);
            beta = alpha >= 0.0 ? -nrm : nrm;
            tk = (beta - alpha) / beta;
            scale = 1.0 / (alpha - beta);
        }
        ta[k] = coherent_load(xbuf + k);
        tb[k] = beta;
        tau[k] = tk;
        sc[SC_SCALE] = scale;
        scale_sh = scale;
        *counter = 0u;
    }
    __syncthreads();
    if (tid < c) {
        // v = (1, scale * x_tail): dots with the earlier slots, the leading 1 sits at index k+1
        const double scale = scale_sh;
        sc[SC_DOTS + 2 * tid] = scale * tot[1 + 2 * tid] + coherent_load(Wp + (long)tid * n + k + 1);
        sc[SC_DOTS + 2 * tid + 1] = scale * tot[2 + 2 * tid] + Vp[(long)tid * n + k + 1];
    }
}

// p'[i] = sum_{j >= k+1} A[i][j] v[j] - sum_q (V_q[i] (W_q.v) + W_q[i] (V_q.v)) for i >= k+1, with
// v = (1, scale * xbuf) formed on the fly.  A is only read below row k; the normalised v is stored
// in panel slot c and in row k of A (its permanent home).  One wave per row, 4 rows per block.
__global__ __launch_bounds__(256) void tri_mat_kernel(double *__restrict__ A, long n, long k, int c,
                                                      double *__restrict__ Vp, const double *__restrict__ Wp,
                                                      const double *__restrict__ xbuf, double *__restrict__ pbuf,
                                                      const double *__restrict__ sc, double *__restrict__ part) {
    __shared__ double ad[NB], bd[NB];
    __shared__ double wsum[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const double scale = sc[SC_SCALE];
    if (tid < c) {
        ad[tid] = sc[SC_DOTS + 2 * tid];
        bd[tid] = sc[SC_DOTS + 2 * tid + 1];
    }
    __syncthreads();
    double wdot = 0.0;
    const long i = k + 1 + (long)blockIdx.x * 4 + wave;
    if (i < n) {
        const double *row = A + i * n;
        double a0 = 0.0, a1 = 0.0;
        long j = k + 1 + lane;
        if (lane == 0) {                     // v[k+1] = 1
            a0 = row[j];
            j += 64;
        }
        for (; j + 64 < n; j += 128) {
            a0 += row[j] * (xbuf[j] * scale);
            a1 += row[j + 64] * (xbuf[j + 64] * scale);
        }
        if (j < n) a0 += row[j] * (xbuf[j] * scale);
        double t = a0 + a1;
        if (lane < c) t -= Vp[(long)lane * n + i] * ad[lane] + Wp[(long)lane * n + i] * bd[lane];
        t = wave_sum(t);
        if (lane == 0) {
            const double vi = (i == k + 1) ? 1.0 : xbuf[i] * scale;
            pbuf[i] = t;
            Vp[(long)c * n + i] = vi;
            A[k * n + i] = vi;
            wdot = t * vi;
        }
    }
    if (lane == 0) wsum[wave] = wdot;
    __syncthreads();
    // block partial of p'.v; the next tri_row_kernel adds the partials up in index order
    if (tid == 0) part[blockIdx.x] = (wsum[0] + wsum[1]) + (wsum[2] + wsum[3]);
}

// A[i][j] -= sum_c V_c[i] W_c[j] + W_c[i] V_c[j] for i, j >= r0.  64 x 64 tile per block, 4 x 4 per thread.
__global__ __launch_bounds__(256) void tri_update_kernel(double *__restrict__ A, long n, long r0, int nbc,
                                                         const double *__restrict__ Vp,
                                                         const double *__restrict__ Wp) {
    constexpr int CC = 16;
    __shared__ double Vi[CC][64], Wi[CC][64], Vj[CC][64], Wj[CC][64];
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
    const long i0 = r0 + (long)blockIdx.y * 64, j0 = r0 + (long)blockIdx.x * 64;
    double acc[4][4];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) acc[a][b] = 0.0;
    for (int cb = 0; cb < nbc; cb += CC) {
        __syncthreads();
        for (int e = tid; e < CC * 64; e += 256) {
            const int c = e >> 6, o = e & 63;
            const bool ok = cb + c < nbc;
            const long ii = i0 + o, jj = j0 + o;
            Vi[c][o] = (ok && ii < n) ? Vp[(long)(cb + c) * n + ii] : 0.0;
            Wi[c][o] = (ok && ii < n) ? Wp[(long)(cb + c) * n + ii] : 0.0;
            Vj[c][o] = (ok && jj < n) ? Vp[(long)(cb + c) * n + jj] : 0.0;
            Wj[c][o] = (ok && jj < n) ? Wp[(long)(cb + c) * n + jj] : 0.0;
        }
        __syncthreads();
#pragma unroll
        for (int c = 0; c < CC; ++c) {
            double vi[4], wi[4], vj[4], wj[4];
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                vi[a] = Vi[c][ty * 4 + a];
                wi[a] = Wi[c][ty * 4 + a];
                vj[a] = Vj[c][tx * 4 + a];
                wj[a] = Wj[c][tx * 4 + a];
            }
#pragma unroll
            for (int a = 0; a < 4; ++a)
#pragma unroll
                for (int b = 0; b < 4; ++b) acc[a][b] += vi[a] * wj[b] + wi[a] * vj[b];
        }
    }
#pragma unroll
    for (int a = 0; a < 4; ++a) {
        const long i = i0 + ty * 4 + a;
        if (i >= n) continue;
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const long j = j0 + tx * 4 + b;
            if (j < n) A[i * n + j] -= acc[a][b];
        }
    }
}

// after the last panel update the trailing 2 x 2 block holds the end of T
__global__ void tri_tail_kernel(const double *__restrict__ A, long n, double *__restrict__ ta,
                                double *__restrict__ tb) {
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    const long k = n - 2;
    ta[k] = A[k * n + k];
    tb[k] = A[k * n + k + 1];
    ta[k + 1] = A[(k + 1) * n + k + 1];
    tb[k + 1] = 0.0;
}

// n <= 2: T is the matrix itself, Q = I
__global__ void tri_tiny_kernel(const double *__restrict__ A, long n, double *__restrict__ ta,
                                double *__restrict__ tb) {
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    ta[0] = A[0];
    tb[n - 1] = 0.0;
    if (n == 2) {
        tb[0] = A[1];
        ta[1] = A[3];
    }
}

// ---- phase 2 -------------------------------------------------------------------------------------
__global__ void identity_kernel(double *__restrict__ R, long n) {
    long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= n * n) return;
    long i = idx / n;
    R[idx] = (idx - i * n == i) ? 1.0 : 0.0;
}

// Reflector k0+c is row k0+c of A on indices >= k0+c+1 (leading 1 stored).  S[c1][c2] = v_c1 . v_c2.
// grid (nbc, nbc), block 256; only c1 <= c2 is computed (and mirrored).
__global__ __launch_bounds__(256) void q_gram_kernel(const double *__restrict__ A, long n, long k0, int nbc,
                                                     double *__restrict__ S) {
    __shared__ double sh[4];
    const int c1 = blockIdx.y, c2 = blockIdx.x;
    if (c1 > c2) return;
    const double *v1 = A + (k0 + c1) * n, *v2 = A + (k0 + c2) * n;
    double s = 0.0;
    for (long i = k0 + c2 + 1 + threadIdx.x; i < n; i += 256) s += v1[i] * v2[i];
    s = wave_sum(s);
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        const double t = (sh[0] + sh[1]) + (sh[2] + sh[3]);
        S[c1 * NB + c2] = t;
        S[c2 * NB + c1] = t;
    }
}

// T of the compact WY form (forward, column-wise): T[c][c] = tau_c,
// T[0:c, c] = -tau_c T[0:c, 0:c] S[0:c, c].  One block of NB threads (thread r owns row r).
__global__ void q_tfactor_kernel(const double *__restrict__ S, const double *__restrict__ tau, long k0, int nbc,
                                 double *__restrict__ T) {
    __shared__ double Ts[NB][NB + 1];
    const int r = threadIdx.x;
    for (int c = 0; c < NB; ++c) Ts[r][c] = 0.0;
    __syncthreads();
    for (int c = 0; c < nbc; ++c) {
        const double tc = tau[k0 + c];
        if (r < c) {
            double s = 0.0;
            for (int q = r; q < c; ++q) s += Ts[r][q] * S[q * NB + c];
            Ts[r][c] = -tc * s;
        } else if (r == c) {
            Ts[r][c] = tc;
        }
        __syncthreads();
    }
    for (int c = 0; c < NB; ++c) T[r * NB + c] = Ts[r][c];
}

// Gp[s][j][c] = sum over slice s of i of R[j][i] v_c[i]  for rows j >= k0+1 (the slices of the
// contraction index give the chip enough blocks; they are added in a fixed order by the consumer).
// Block: 64 rows x NB columns, thread (ty, tx): rows ty*4..+3, columns tx*2, tx*2+1.
// grid (ceil((n-k0-1)/64), KS).
constexpr int WY_KS_MAX = 16;
__global__ __launch_bounds__(256) void q_wy_g_kernel(const double *__restrict__ R, const double *__restrict__ A,
                                                     long n, long k0, int nbc, long chunk,
                                                     double *__restrict__ Gp) {
    constexpr int KC = 32;
    __shared__ double Rs[64][KC + 1];
    __shared__ double Vs[NB][KC + 1];
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
    const long j0 = k0 + 1 + (long)blockIdx.x * 64;
    const long ibeg = k0 + 1 + (long)blockIdx.y * chunk;
    const long iend = min(n, ibeg + chunk);
    double acc[4][2];
#pragma unroll
    for (int a = 0; a < 4; ++a) acc[a][0] = acc[a][1] = 0.0;
    for (long i0 = ibeg; i0 < iend; i0 += KC) {
        __syncthreads();
        for (int e = tid; e < 64 * KC; e += 256) {
            const int r = e / KC, q = e % KC;
            const long j = j0 + r, i = i0 + q;
            Rs[r][q] = (j < n && i < iend) ? R[j * n + i] : 0.0;
        }
        for (int e = tid; e < NB * KC; e += 256) {
            const int c = e / KC, q = e % KC;
            const long i = i0 + q;
            Vs[c][q] = (c < nbc && i < iend && i >= k0 + c + 1) ? A[(k0 + c) * n + i] : 0.0;
        }
        __syncthreads();
#pragma unroll 8
        for (int q = 0; q < KC; ++q) {
            const double v0 = Vs[tx * 2][q], v1 = Vs[tx * 2 + 1][q];
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                const double r = Rs[ty * 4 + a][q];
                acc[a][0] += r * v0;
                acc[a][1] += r * v1;
            }
        }
    }
    double *out = Gp + (long)blockIdx.y * n * NB;
#pragma unroll
    for (int a = 0; a < 4; ++a) {
        const long j = j0 + ty * 4 + a;
        if (j < n) {
            out[j * NB + tx * 2] = acc[a][0];
            out[j * NB + tx * 2 + 1] = acc[a][1];
        }
    }
}

// R[j][i] -= sum_c G2[j][c] v_c[i]  for j, i >= k0+1, with G2 = (sum_s Gp[s]) T^T formed per tile.
// 64 x 64 tile per block, 4 x 4 per thread.
__global__ __launch_bounds__(256) void q_wy_update_kernel(double *__restrict__ R, const double *__restrict__ A,
                                                          long n, long k0, int nbc, int ks,
                                                          const double *__restrict__ Gp,
                                                          const double *__restrict__ T) {
    __shared__ double Gs[64][NB + 1];
    __shared__ double G2s[64][NB + 1];
    __shared__ double Vs[NB][64];
    __shared__ double Ts[NB][NB + 1];
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
    const long j0 = k0 + 1 + (long)blockIdx.y * 64, i0 = k0 + 1 + (long)blockIdx.x * 64;
    for (int e = tid; e < NB * NB; e += 256) Ts[e / NB][e % NB] = T[e];
    for (int e = tid; e < 64 * NB; e += 256) {
        const int r = e / NB, c = e % NB;
        const long j = j0 + r;
        double g = 0.0;
        if (j < n && c < nbc)
            for (int s = 0; s < ks; ++s) g += Gp[((long)s * n + j) * NB + c];
        Gs[r][c] = g;
    }
    for (int e = tid; e < NB * 64; e += 256) {
        const int c = e >> 6, o = e & 63;
        const long i = i0 + o;
        Vs[c][o] = (c < nbc && i < n && i >= k0 + c + 1) ? A[(k0 + c) * n + i] : 0.0;
    }
    __syncthreads();
    for (int e = tid; e < 64 * NB; e += 256) {
        const int r = e / NB, c = e % NB;
        double s = 0.0;
        for (int q = c; q < nbc; ++q) s += Gs[r][q] * Ts[c][q];          // T is upper triangular
        G2s[r][c] = s;
    }
    __syncthreads();
    double acc[4][4];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) acc[a][b] = 0.0;
#pragma unroll 8
    for (int c = 0; c < NB; ++c) {
        double g[4], v[4];
#pragma unroll
        for (int a = 0; a < 4; ++a) {
            g[a] = G2s[ty * 4 + a][c];
            v[a] = Vs[c][tx * 4 + a];
        }
#pragma unroll
        for (int a = 0; a < 4; ++a)
#pragma unroll
            for (int b = 0; b < 4; ++b) acc[a][b] += g[a] * v[b];
    }
#pragma unroll
    for (int a = 0; a < 4; ++a) {
        const long j = j0 + ty * 4 + a;
        if (j >= n) continue;
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const long i = i0 + tx * 4 + b;
            if (i < n) R[j * n + i] -= acc[a][b];
        }
    }
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

inline unsigned blocks_for(long count, int bs) { return (unsigned)((count + bs - 1) / bs); }

}  // namespace

size_t admmq_householder_scratch_doubles(int64_t n) {
    const size_t N = (size_t)n;
    return (3 + 2 * NB + WY_KS_MAX * NB) * N + 2 * NB * NB + SC_COUNT + (N / ROW_CHUNK + 2) * PART_W + (N / 4 + 2) + 64;
}

// A64: [n][n] scaled Hessian (destroyed: reflectors end up in its rows); R64: [n][n] scratch;
// vecs: admmq_householder_scratch_doubles(n) doubles.  Outputs: Q, Qt (fp32), ta, tb (fp64).
admmq_status admmq_k_householder(admmq_ctx *ctx, double *A64, int64_t n, double *R64, double *vecs, float *Q,
                                 float *Qt, double *ta, double *tb) {
    hipStream_t st = ctx->stream;
    const long N = (long)n;
    double *pbuf = vecs, *xbuf = vecs + N, *tau = vecs + 2 * N, *Vp = vecs + 3 * N, *Wp = Vp + (long)NB * N,
           *Gp = Wp + (long)NB * N, *S = Gp + (long)WY_KS_MAX * NB * N, *T = S + NB * NB, *sc = T + NB * NB,
           *part1 = sc + SC_COUNT, *part2 = part1 + (N / ROW_CHUNK + 2) * PART_W, *cnt = part2 + (N / 4 + 2);
    unsigned *counters = (unsigned *)cnt;          // [0]: tri_row, [2]: tri_mat (8-byte slots)
    ADMMQ_TRY(admmq_k_fill_bytes(ctx, cnt, 0, 32));
    ADMMQ_TRY(admmq_k_fill_bytes(ctx, sc, 0, SC_COUNT * 8));
    if (N <= 2) {
        hipLaunchKernelGGL(tri_tiny_kernel, dim3(1), dim3(64), 0, st, A64, N, ta, tb);
    } else {
        for (long k0 = 0; k0 <= N - 3; k0 += NB) {
            const int nbc = (int)((N - 2 - k0) < NB ? (N - 2 - k0) : NB);
            for (int c = 0; c < nbc; ++c) {
                const long k = k0 + c;
                // the previous column's tri_mat_kernel had blocks_for(N - k, 4) blocks
                hipLaunchKernelGGL(tri_row_kernel, dim3(blocks_for(N - k, ROW_CHUNK)), dim3(256), 0, st, A64, N, k, c,
                                   c > 0 ? 1 : 0, 1, Vp, Wp, pbuf, xbuf, tau, ta, tb, sc, part1, counters, part2,
                                   (int)blocks_for(N - k, 4));
                hipLaunchKernelGGL(tri_mat_kernel, dim3(blocks_for(N - k - 1, 4)), dim3(256), 0, st, A64, N, k, c, Vp,
                                   Wp, xbuf, pbuf, sc, part2);
            }
            // close the panel's last column, then apply the panel to the trailing matrix
            const long r0 = k0 + nbc;
            hipLaunchKernelGGL(tri_row_kernel, dim3(blocks_for(N - r0, ROW_CHUNK)), dim3(256), 0, st, A64, N, r0, nbc,
                               1, 0, Vp, Wp, pbuf, xbuf, tau, ta, tb, sc, part1, counters, part2,
                               (int)blocks_for(N - r0, 4));
            const unsigned tiles = blocks_for(N - r0, 64);
            hipLaunchKernelGGL(tri_update_kernel, dim3(tiles, tiles), dim3(256), 0, st, A64, N, r0, nbc, Vp, Wp);
        }
        hipLaunchKernelGGL(tri_tail_kernel, dim3(1), dim3(64), 0, st, A64, N, ta, tb);
    }
    ADMMQ_HIP(hipGetLastError());
    hipLaunchKernelGGL(identity_kernel, dim3(blocks_for(N * N, 256)), dim3(256), 0, st, R64, N);
    if (N >= 3) {
        const long nref = N - 2;
        const long nblk = (nref + NB - 1) / NB;
        for (long b = nblk - 1; b >= 0; --b) {
            const long k0 = b * NB;
            const int nbc = (int)((nref - k0) < NB ? (nref - k0) : NB);
            hipLaunchKernelGGL(q_gram_kernel, dim3(nbc, nbc), dim3(256), 0, st, A64, N, k0, nbc, S);
            hipLaunchKernelGGL(q_tfactor_kernel, dim3(1), dim3(NB), 0, st, S, tau, k0, nbc, T);
            const long m = N - k0 - 1;
            const unsigned tiles = blocks_for(m, 64);
            long ks = 512 / (long)tiles;
            if (ks > WY_KS_MAX) ks = WY_KS_MAX;
            if (ks > m / 256) ks = m / 256;
            if (ks < 1) ks = 1;
            long chunk = (m + ks - 1) / ks;
            chunk = (chunk + 31) / 32 * 32;
            hipLaunchKernelGGL(q_wy_g_kernel, dim3(tiles, (unsigned)ks), dim3(256), 0, st, R64, A64, N, k0, nbc, chunk,
                               Gp);
            hipLaunchKernelGGL(q_wy_update_kernel, dim3(tiles, tiles), dim3(256), 0, st, R64, A64, N, k0, nbc, (int)ks,
                               Gp, T);
        }
    }
    dim3 tb32(32, 8), tg((unsigned)((N + 31) / 32), (unsigned)((N + 31) / 32));
    hipLaunchKernelGGL(emit_q_kernel, tg, tb32, 0, st, R64, N, Q, Qt);
    ADMMQ_HIP(hipGetLastError());
    return ADMMQ_OK;
}
