// Per-iteration use of the band form Hs = Q Bd Q^T (Alg. 1 line 3, Sec. 3.3; the reduction itself is in
// householder.hip): the middle factor of eq. 7 in its correction form,
//     S = (Bd + rho I)^-1 Bd Y = Y - rho (Bd + rho I)^-1 Y,
// for all columns of Y at once.  Bd has half-bandwidth 16, i.e. it is block tridiagonal in 16 x 16 blocks
// (diagonal blocks D_I, blocks E_I = Bd[I+1][I] below them, upper triangular), and the solve is block elimination:
//     Delta_0 = D_0 + rho I,  Delta_I = D_I + rho I - F_I E_{I-1}^T,  F_I = E_{I-1} Delta_{I-1}^-1
//     forward :  yh_I = y_I - F_I yh_{I-1}
//     backward:  u_I  = (rho Delta_I^-1) yh_I - G_I u_{I+1},  G_I = Delta_I^-1 E_I^T,   S_I = y_I - u_I
// (u = rho x).  The three 16 x 16 matrices per block row depend on rho only; they are formed once per penalty of
// the schedule (band_factor_kernel, fp64) and stored in the order the fp64 matrix-core instruction wants its first
// operand, so that the per-iteration kernel is nothing but v_mfma_f64_16x16x4 on 16-column strips of Y.
// Between the two sweeps only r_I = yh_I - y_I = -F_I yh_{I-1} is kept, in fp32, in the output array: it shrinks
// like 1/rho, so what its rounding adds to S stays relative to S as rho grows (storing yh itself would leave an
// error of 2^-24 |Y| in S that the dual update multiplies by rho).
#include <stdlib.h>

#include "common.h"

typedef double doublex4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int BW = 16;

// position of M[i][j] in the order of the matrix core's first operand: lane l holds M[l % 16][4 s + l / 16] at
// s * 64 + l
__device__ inline int a_operand_index(int i, int j) { return (j >> 2) * 64 + (j & 3) * 16 + i; }

// One block (256 threads, thread = entry (i, j)) per penalty; block rows in sequence.
// bd[t][c] = Bd[c + t][c], t = 0 .. 16, c < npad.  fac[((t * nbk + I) * 3 + w) * 256 + ..]: w = 0: F_I, 1: rho Delta_I^-1,
// 2: G_I.
__global__ __launch_bounds__(256) void band_factor_kernel(const double *__restrict__ bd, long npad, int nbk,
                                                          const double *__restrict__ rhos, int count,
                                                          double *__restrict__ fac) {
    __shared__ double Dl[16][17], Ep[16][17], En[16][17], Fm[16][17], Inv[16][17];
    const int t = blockIdx.x;
    if (t >= count) return;
    const int tid = threadIdx.x, i = tid >> 4, j = tid & 15;
    const double rho = rhos[t];
    double *out = fac + (long)t * nbk * 3 * 256;
    Inv[i][j] = 0.0;
    Ep[i][j] = 0.0;
    __syncthreads();
    for (int I = 0; I < nbk; ++I) {
        const long c0 = (long)I * 16;
        // D_I (symmetric) and E_I (upper triangular: rows of block I+1, columns of block I; zero in the last block row)
        const int lo = i < j ? i : j, df = i < j ? j - i : i - j;
        const double d = bd[(long)df * npad + c0 + lo];
        const double e = (i <= j && I + 1 < nbk) ? bd[(long)(16 + i - j) * npad + c0 + j] : 0.0;
        En[i][j] = e;
        // F_I = E_{I-1} Delta_{I-1}^-1
        double f = 0.0;
#pragma unroll
        for (int k = 0; k < 16; ++k) f += Ep[i][k] * Inv[k][j];
        Fm[i][j] = f;
        __syncthreads();
        // Delta_I = D_I + rho I - F_I E_{I-1}^T
        double dl = d + (i == j ? rho : 0.0);
#pragma unroll
        for (int k = 0; k < 16; ++k) dl -= Fm[i][k] * Ep[j][k];
        Dl[i][j] = dl;
        __syncthreads();
        // inverse by Gauss-Jordan elimination without pivoting (Delta is symmetric positive definite)
        for (int k = 0; k < 16; ++k) {
            const double p = 1.0 / Dl[k][k], aik = Dl[i][k], akj = Dl[k][j], aij = Dl[i][j];
            __syncthreads();
            double v;
            if (i == k) v = j == k ? p : akj * p;
            else v = j == k ? -aik * p : aij - aik * akj * p;
            Dl[i][j] = v;
            __syncthreads();
        }
        Inv[i][j] = Dl[i][j];
        __syncthreads();
        // G_I = Delta_I^-1 E_I^T
        double g = 0.0;
#pragma unroll
        for (int k = 0; k < 16; ++k) g += Inv[i][k] * En[j][k];
        double *o = out + (long)I * 3 * 256;
        const int idx = a_operand_index(i, j);
        o[idx] = f;
        o[256 + idx] = rho * Inv[i][j];
        o[512 + idx] = g;
        Ep[i][j] = e;
        __syncthreads();
    }
}

// Block = four waves, one strip of 16 columns each.  Lane l of a wave works at column l % 16 of its strip on the rows
// 4 s + l / 16 (s = 0 .. 3) of each block row: that is at once where the second operand of the matrix-core product
// wants row 4 s + l / 16 of a 16 x 16 block and where its result register s holds it, so both recurrences run in
// registers.  The matrices of a block row are the same for every strip: the block fetches them once, through
// registers into LDS, for all four waves (with one wave per block every compute unit of the chip asked the cache
// for the same 2 KB at the same time, and the kernel ran at a fifth of the speed of its products).
// The sweeps go in stages of GS block rows.  Everything stage k + 2 needs is requested at the start of stage k: the
// rows of Y (and of r) into one of three named register sets, the matrices into one of three more, from which they
// move to LDS at the end of stage k + 1, a whole stage after they were asked for - so no wait stands between a
// request and two stages of products.  (Named sets and a loop unrolled three times instead of rotating copies: a
// copy of a value still on its way would wait for it.)
constexpr int GS = 8;            // block rows per stage

template <int WPB>
struct BandStageRegs {
    float y[GS][4], r[GS][4];
    doublex4 m[(GS * 2 * 256) / (64 * WPB * 4)];      // this thread's share of a stage's matrices (two per block row at most)
};

template <bool BACKWARD, int WPB, bool FULL>
struct BandSweep {
    const double *fac;
    int nbk;
    long n, p;
    const float *Y;
    float *S;
    int lane, wave, tid, col, kq;
    long j;
    bool jok;
    double (*lds)[GS * 2 * 256];          // [2] stage buffers
    static constexpr int NM = BACKWARD ? 2 : 1;                  // matrices per block row
    static constexpr int NT = 64 * WPB;
    static constexpr int MV = GS * NM * 256 / (NT * 4);          // doublex4 per thread and stage

    // block row of position q (0 .. GS-1) of stage k
    __device__ __forceinline__ int row_of(int k, int q) const { return BACKWARD ? nbk - 1 - (k * GS + q) : k * GS + q; }

    __device__ __forceinline__ void request(int k, BandStageRegs<WPB> &R) const {
#pragma unroll
        for (int q = 0; q < GS; ++q) {
            const int I = row_of(k, q);
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const long row = (long)I * 16 + 4 * s + kq;
                const bool ok = FULL || (jok && I >= 0 && I < nbk && row < n);
                R.y[q][s] = ok ? Y[row * p + j] : 0.f;
                if (BACKWARD) R.r[q][s] = ok ? S[row * p + j] : 0.f;
            }
        }
        // matrices: stage buffer entry e (in doubles) = (q * NM + w) * 256 + i  <-  fac[(I * 3 + (BACKWARD ? 1 + w : 0)) * 256 + i]
#pragma unroll
        for (int v = 0; v < MV; ++v) {
            const int e = (tid + NT * v) * 4, mat = e >> 8, i = e & 255, q = mat / NM, w = mat - q * NM;
            const int I = row_of(k, q);
            doublex4 z = {0.0, 0.0, 0.0, 0.0};
            if (FULL || (I >= 0 && I < nbk)) z = *(const doublex4 *)(fac + ((long)I * 3 + (BACKWARD ? 1 + w : 0)) * 256 + i);
            R.m[v] = z;
        }
    }
    __device__ __forceinline__ void deposit(int k, const BandStageRegs<WPB> &R) const {
        double *dst = lds[k & 1];
#pragma unroll
        for (int v = 0; v < MV; ++v) *(doublex4 *)(dst + (tid + NT * v) * 4) = R.m[v];
    }
};

// FULL: n a multiple of 16, the number of block rows a multiple of GS and p a multiple of 16 WPB, so that no access
// needs a guard: the sweeps are then free of branches (a stage is one basic block, which lets the compiler overlap
// one block row's stores with the next one's products), and the backward sweep issues the product that does not
// hang on the recurrence, (rho Delta^-1) yh of the NEXT block row, between the steps of the one that does.
template <int WPB, bool FULL>
__global__ __launch_bounds__(64 * WPB) __attribute__((amdgpu_waves_per_eu(1, 1))) void band_apply_kernel(const double *__restrict__ fac, int nbk, long n, long p,
                                                         const float *__restrict__ Y, float *__restrict__ S,
                                                         unsigned *__restrict__ amax_out) {
    __shared__ __align__(32) double lds[2][GS * 2 * 256];           // 64 KB
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, col = lane & 15, kq = lane >> 4;
    const long j = ((long)blockIdx.x * WPB + wave) * 16 + col;
    const bool jok = j < p;
    const int nst = (nbk + GS - 1) / GS;
    unsigned smax = 0;
    BandStageRegs<WPB> RA, RB, RC;
    // (a barrier that orders LDS traffic only: __syncthreads() would also wait for the requests two stages ahead)
    auto lds_barrier = [&]() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); };

    // ---- forward: yh_I = y_I - F_I yh_{I-1}; r_I = yh_I - y_I goes to S ---------------------------------------
    {
        BandSweep<false, WPB, FULL> sw{fac, nbk, n, p, Y, S, lane, wave, tid, col, kq, j, jok, lds};
        double yh[4] = {0.0, 0.0, 0.0, 0.0};
        auto stage = [&](int k, BandStageRegs<WPB> &cur, BandStageRegs<WPB> &nxt, BandStageRegs<WPB> &far) __attribute__((always_inline)) {
            // cur: stage k (its matrices are in LDS already); nxt: stage k+1 (requested a stage ago); far: free
            if (k + 2 < nst) sw.request(k + 2, far);
            const double *mat = lds[k & 1];
#pragma unroll
            for (int q = 0; q < GS; ++q) {
                const int I = k * GS + q;
                doublex4 acc = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
                for (int s = 0; s < 4; ++s)
                    acc = __builtin_amdgcn_mfma_f64_16x16x4f64(mat[q * 256 + s * 64 + lane], yh[s], acc, 0, 0, 0);
#pragma unroll
                for (int s = 0; s < 4; ++s) {
                    const long row = (long)I * 16 + 4 * s + kq;
                    const float r = (float)(-acc[s]);
                    yh[s] = (double)cur.y[q][s] + (double)r;       // (the backward sweep forms yh from the same rounded r)
                    if (FULL || (jok && I < nbk && row < n)) S[row * p + j] = r;
                }
            }
            if (k + 1 < nst) sw.deposit(k + 1, nxt);
            lds_barrier();
        };
        sw.request(0, RA);
        if (nst > 1) sw.request(1, RB);
        sw.deposit(0, RA);
        lds_barrier();
        for (int k = 0; k < nst; k += 3) {
            stage(k, RA, RB, RC);
            if (k + 1 < nst) stage(k + 1, RB, RC, RA);
            if (k + 2 < nst) stage(k + 2, RC, RA, RB);
        }
    }
    // (every thread reads back below exactly the entries of r it has written itself)
    // ---- backward: u_I = (rho Delta_I^-1) yh_I - G_I u_{I+1}; S_I = y_I - u_I ----------------------------------------
    {
        BandSweep<true, WPB, FULL> sw{fac, nbk, n, p, Y, S, lane, wave, tid, col, kq, j, jok, lds};
        double un[4] = {0.0, 0.0, 0.0, 0.0};
        auto stage = [&](int k, BandStageRegs<WPB> &cur, BandStageRegs<WPB> &nxt, BandStageRegs<WPB> &far) __attribute__((always_inline)) {
            if (k + 2 < nst) sw.request(k + 2, far);
            const double *mat = lds[k & 1];
            if (FULL) {
                // pa: (rho Delta^-1) yh of the block row in hand, formed while the row before it was on the recurrence
                doublex4 pa = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
                for (int s = 0; s < 4; ++s)
                    pa = __builtin_amdgcn_mfma_f64_16x16x4f64(mat[s * 64 + lane], (double)cur.y[0][s] + (double)cur.r[0][s], pa, 0, 0, 0);
#pragma unroll
                for (int q = 0; q < GS; ++q) {
                    const int I = nbk - 1 - (k * GS + q);
                    doublex4 acc2 = {0.0, 0.0, 0.0, 0.0}, pn = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
                    for (int s = 0; s < 4; ++s) {
                        acc2 = __builtin_amdgcn_mfma_f64_16x16x4f64(mat[(q * 2 + 1) * 256 + s * 64 + lane], un[s], acc2, 0, 0, 0);
                        if (q + 1 < GS)
                            pn = __builtin_amdgcn_mfma_f64_16x16x4f64(mat[((q + 1) * 2) * 256 + s * 64 + lane],
                                                                      (double)cur.y[q + 1][s] + (double)cur.r[q + 1][s], pn, 0, 0, 0);
                    }
#pragma unroll
                    for (int s = 0; s < 4; ++s) {
                        const long row = (long)I * 16 + 4 * s + kq;
                        un[s] = pa[s] - acc2[s];
                        const float sv = (float)((double)cur.y[q][s] - un[s]);
                        S[row * p + j] = sv;
                        smax = max(smax, __float_as_uint(fabsf(sv)));
                    }
                    pa = pn;
                }
            } else {
#pragma unroll
            for (int q = 0; q < GS; ++q) {
                const int I = nbk - 1 - (k * GS + q);
                doublex4 acc = {0.0, 0.0, 0.0, 0.0}, acc2 = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
                for (int s = 0; s < 4; ++s) {
                    const double yhs = (double)cur.y[q][s] + (double)cur.r[q][s];
                    acc = __builtin_amdgcn_mfma_f64_16x16x4f64(mat[(q * 2) * 256 + s * 64 + lane], yhs, acc, 0, 0, 0);
                    acc2 = __builtin_amdgcn_mfma_f64_16x16x4f64(mat[(q * 2 + 1) * 256 + s * 64 + lane], un[s], acc2, 0, 0, 0);
                }
#pragma unroll
                for (int s = 0; s < 4; ++s) {
                    const long row = (long)I * 16 + 4 * s + kq;
                    un[s] = acc[s] - acc2[s];
                    const float sv = (float)((double)cur.y[q][s] - un[s]);
                    if (jok && I >= 0 && row < n) {
                        S[row * p + j] = sv;
                        smax = max(smax, __float_as_uint(fabsf(sv)));
                    }
                }
            }
            }
            if (k + 1 < nst) sw.deposit(k + 1, nxt);
            lds_barrier();
        };
        sw.request(0, RA);
        if (nst > 1) sw.request(1, RB);
        sw.deposit(0, RA);
        lds_barrier();
        for (int k = 0; k < nst; k += 3) {
            stage(k, RA, RB, RC);
            if (k + 1 < nst) stage(k + 1, RB, RC, RA);
            if (k + 2 < nst) stage(k + 2, RC, RA, RB);
        }
    }
    if (amax_out) {
        // for the split-fp16 products: the largest |S| of the whole solve (most waves find a value at least as
        // large already there and skip the atomic)
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) smax = max(smax, (unsigned)__shfl_xor((int)smax, o));
        if (lane == 0 && smax > __atomic_load_n(amax_out, __ATOMIC_RELAXED)) atomicMax(amax_out, smax);
    }
}

}  // namespace

size_t admmq_band_factor_doubles(int64_t n, int count) {
    const size_t nbk = ((size_t)n + BW - 1) / BW;
    return (size_t)count * nbk * 3 * 256;
}

// Block-elimination factors of Bd + rho_t I for `count` penalties; fac: admmq_band_factor_doubles(n, count) doubles.
admmq_status admmq_k_band_factor(admmq_ctx *ctx, const double *bd, int64_t n, const double *rhos_dev, int count,
                                 double *fac) {
    const long npad = ((long)n + BW - 1) / BW * BW;
    hipLaunchKernelGGL(band_factor_kernel, dim3((unsigned)count), dim3(256), 0, ctx->stream, bd, npad, (int)(npad / BW),
                       rhos_dev, count, fac);
    ADMMQ_HIP(hipGetLastError());
    return ADMMQ_OK;
}

// S = (Bd + rho I)^-1 Bd Y for the penalty whose factors start at `fac` (one penalty's slice of the array above).
// Y, S: fp32 [n][p]; S must not be Y (it holds the forward sweep's intermediate before it holds the result).
admmq_status admmq_k_band_apply(admmq_ctx *ctx, const double *fac, int64_t n, int64_t p, const float *Y, float *S,
                                unsigned *amax_out) {
    if ((const float *)S == Y) return ADMMQ_ERR_PARAM;
    const int nbk = (int)((n + BW - 1) / BW);
    static int wpb = 0;
    if (wpb == 0) {
        const char *e = getenv("ADMMQ_BAND_WAVES");
        wpb = e ? atoi(e) : 2;              // measured at 12288 x 4096: 0.66 ms with two strips per block, 0.72 ms with four
        if (wpb != 2 && wpb != 4) wpb = 2;
    }
    const long strips = (p + 15) / 16;
    const bool full = n % BW == 0 && nbk % GS == 0 && p % (16 * wpb) == 0;
#define ADMMQ_BAND_LAUNCH(W, F)                                                                                          \
    hipLaunchKernelGGL((band_apply_kernel<W, F>), dim3((unsigned)((strips + W - 1) / W)), dim3(64 * W), 0, ctx->stream, fac, \
                       nbk, (long)n, (long)p, Y, S, amax_out)
    if (wpb == 2) {
        if (full) ADMMQ_BAND_LAUNCH(2, true); else ADMMQ_BAND_LAUNCH(2, false);
    } else {
        if (full) ADMMQ_BAND_LAUNCH(4, true); else ADMMQ_BAND_LAUNCH(4, false);
    }
#undef ADMMQ_BAND_LAUNCH
    ADMMQ_HIP(hipGetLastError());
    return ADMMQ_OK;
}
