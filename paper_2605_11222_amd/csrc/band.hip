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
constexpr int BSL = 4;           // block rows per segment of the split sweeps
constexpr int BMATS = 5;         // matrices per block row and penalty: F, rho Delta^-1, G, Pf, Pb

// position of M[i][j] in the order of the matrix core's first operand, lane by lane: lane l = (j & 3) * 16 + i holds
// M[l % 16][4 s + l / 16] for the k-step s = j >> 2, and a lane's four values lie side by side (one 32-byte load)
__device__ inline int a_operand_index(int i, int j) { return ((j & 3) * 16 + i) * 4 + (j >> 2); }

// One block (256 threads, thread = entry (i, j)) per penalty; block rows in sequence.
// bd[t][c] = Bd[c + t][c], t = 0 .. 16, c < npad.  fac[((t * nbk + I) * 5 + w) * 256 + ..]: w = 0: F_I, 1: rho Delta_I^-1,
// 2: G_I, and the propagators of the two recurrences inside the segments of BSL block rows (I0 = first, I1 = last
// block row of I's segment): 3: Pf_I = (-F_I)(-F_{I-1}) ... (-F_{I0}), 4: Pb_I = (-G_I)(-G_{I+1}) ... (-G_{I1}).
__global__ __launch_bounds__(256) void band_factor_kernel(const double *__restrict__ bd, long npad, int nbk,
                                                          const double *__restrict__ rhos, int count,
                                                          double *__restrict__ fac) {
    __shared__ double Dl[16][17], Ep[16][17], En[16][17], Fm[16][17], Inv[16][17], Pp[16][17];
    const int t = blockIdx.x;
    if (t >= count) return;
    const int tid = threadIdx.x, i = tid >> 4, j = tid & 15;
    const double rho = rhos[t];
    double *out = fac + (long)t * nbk * BMATS * 256;
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
        // Pf_I = -F_I Pf_{I-1}, restarting at the first block row of a segment
        double pf = -f;
        if (I % BSL != 0) {
            pf = 0.0;
#pragma unroll
            for (int k = 0; k < 16; ++k) pf -= Fm[i][k] * Pp[k][j];
        }
        double *o = out + (long)I * BMATS * 256;
        const int idx = a_operand_index(i, j);
        o[idx] = f;
        o[256 + idx] = rho * Inv[i][j];
        o[512 + idx] = g;
        o[768 + idx] = pf;
        __syncthreads();
        Ep[i][j] = e;
        Pp[i][j] = pf;
        __syncthreads();
    }
    // Pb_I = -G_I Pb_{I+1}, from the last block row up, restarting at the last block row of a segment
    for (int I = nbk - 1; I >= 0; --I) {
        double *o = out + (long)I * BMATS * 256;
        const int idx = a_operand_index(i, j);
        const double g = o[512 + idx];               // (written by this thread above)
        Fm[i][j] = g;
        __syncthreads();
        double pb = -g;
        if (I % BSL != BSL - 1 && I != nbk - 1) {
            pb = 0.0;
#pragma unroll
            for (int k = 0; k < 16; ++k) pb -= Fm[i][k] * Pp[k][j];
        }
        o[1024 + idx] = pb;
        __syncthreads();
        Pp[i][j] = pb;
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
            if (FULL || (I >= 0 && I < nbk)) z = *(const doublex4 *)(fac + ((long)I * BMATS + (BACKWARD ? 1 + w : 0)) * 256 + i);
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
                    acc = __builtin_amdgcn_mfma_f64_16x16x4f64(mat[q * 256 + lane * 4 + s], yh[s], acc, 0, 0, 0);
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
                    pa = __builtin_amdgcn_mfma_f64_16x16x4f64(mat[lane * 4 + s], (double)cur.y[0][s] + (double)cur.r[0][s], pa, 0, 0, 0);
#pragma unroll
                for (int q = 0; q < GS; ++q) {
                    const int I = nbk - 1 - (k * GS + q);
                    doublex4 acc2 = {0.0, 0.0, 0.0, 0.0}, pn = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
                    for (int s = 0; s < 4; ++s) {
                        acc2 = __builtin_amdgcn_mfma_f64_16x16x4f64(mat[(q * 2 + 1) * 256 + lane * 4 + s], un[s], acc2, 0, 0, 0);
                        if (q + 1 < GS)
                            pn = __builtin_amdgcn_mfma_f64_16x16x4f64(mat[((q + 1) * 2) * 256 + lane * 4 + s],
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
                    acc = __builtin_amdgcn_mfma_f64_16x16x4f64(mat[(q * 2) * 256 + lane * 4 + s], yhs, acc, 0, 0, 0);
                    acc2 = __builtin_amdgcn_mfma_f64_16x16x4f64(mat[(q * 2 + 1) * 256 + lane * 4 + s], un[s], acc2, 0, 0, 0);
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

// ---- the same solve with both recurrences split into segments ------------------------------------------------------
// A linear recurrence with matrix coefficients splits exactly like a scalar one: over a segment of block rows
// I0 .. I1 with the value c entering it,
//     yh_I = yt_I + Pf_I c,    yt = the recurrence started from zero,  Pf_I = (-F_I) ... (-F_{I0})    (forward)
//     u_I  = ut_I + Pb_I c',   c' = u_{I1 + 1},                        Pb_I = (-G_I) ... (-G_{I1})    (backward)
// and the propagators depend on the penalty only (band_factor_kernel forms them with the other matrices).
// A block owns one strip of 16 columns and walks the block rows in tiles of SW segments of BSL block rows; wave w
// runs segment w: the local recurrence (BSL dependent products instead of SW * BSL), the segment ends through LDS,
// the chain over the ends of the segments before it (w short steps), then the correction, whose BSL products do not
// depend on one another.  A dependent 16 x 16 x 16 product costs four matrix-core instructions of about 97 cycles
// each on this chip: the chain of dependent products per sweep falls from n / 16 to (n / 16) (BSL + SW) / (BSL SW),
// and SW waves per compute unit share the matrix cores instead of one.
// Between the sweeps r_I = yh_I - y_I is kept in fp32 in the output array, as in the unsplit kernel.
// Every matrix a phase needs is requested before the phase's first product (in the order of use: the loads of a
// wave return in order), the rows of Y and r of the next tile after them: a request in front of its product would
// cost the cache's latency once per product.
// FULL: n a multiple of 16, the number of block rows a multiple of the tile and p a multiple of 16: no access needs
// a guard (a guard per load is an exec-mask dance on the scalar unit that the block's waves share).
template <int SW, bool FULL>
__global__ __launch_bounds__(64 * SW) void band_apply_split_kernel(const double *__restrict__ fac, int nbk, long n, long p,
                                                                    const float *__restrict__ Y, float *__restrict__ S,
                                                                    unsigned *__restrict__ amax_out) {
    constexpr int TB = SW * BSL;                                   // block rows per tile
    __shared__ __align__(32) double ends[SW][256];                 // a segment's end value, in operand order
    __shared__ __align__(32) double carry[256];                    // the value entering the tile
    __shared__ __align__(32) double chm[SW][256];                  // the tile's chain matrices: the propagator over each segment
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int col = lane & 15, kq = lane >> 4;
    // blocks whose ids are congruent mod 8 run on the same XCD: they get neighbouring strips, so that the two halves
    // of a 128-byte line of Y (two strips' worth of a row) are asked for by the same L2
    long strip = blockIdx.x;
    if ((gridDim.x & 7) == 0) strip = (long)(blockIdx.x & 7) * (gridDim.x >> 3) + (blockIdx.x >> 3);
    const long j = strip * 16 + col;
    const bool jok = j < p;
    const int ntile = (nbk + TB - 1) / TB;
    unsigned smax = 0;
    auto lds_barrier = [&]() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); };
    // matrix w of block row I as the matrix core's first operand (zero beyond the last block row)
    auto load_mat = [&](int I, int w, double *m) {
        doublex4 v = {0.0, 0.0, 0.0, 0.0};
        if (FULL || I < nbk) v = *(const doublex4 *)(fac + ((long)I * BMATS + w) * 256 + lane * 4);
#pragma unroll
        for (int s = 0; s < 4; ++s) m[s] = v[s];
    };
    // acc = M x, x in operand order (lane holds rows 4 s + kq of its column)
    auto product = [&](const double *m, const double *x) {
        doublex4 acc = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
        for (int s = 0; s < 4; ++s) acc = __builtin_amdgcn_mfma_f64_16x16x4f64(m[s], x[s], acc, 0, 0, 0);
        return acc;
    };
    auto load_rows = [&](const float *src, int I0, float (*dst)[4]) {
#pragma unroll
        for (int q = 0; q < BSL; ++q)
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const long row = (long)(I0 + q) * 16 + 4 * s + kq;
                if (FULL) dst[q][s] = src[row * p + j];
                else dst[q][s] = (jok && I0 + q >= 0 && I0 + q < nbk && row < n) ? src[row * p + j] : 0.f;
            }
    };

    // ---- forward: r_I = yh_I - y_I, yh_I = y_I - F_I yh_{I-1} ---------------------------------------------------------
    if (tid < 256) carry[tid] = 0.0;
    float y[BSL][4], yn[BSL][4];
    load_rows(Y, wave * BSL, y);
    lds_barrier();
    for (int t = 0; t < ntile; ++t) {
        const int I0 = t * TB + wave * BSL;
        double mloc[BSL][4], mine[4];
#pragma unroll
        for (int q = 1; q < BSL; ++q) load_mat(I0 + q, 0, mloc[q]);
        load_mat(I0 + BSL - 1, 3, mine);                 // this segment's propagator, for the waves after this one
        if (!FULL || t + 1 < ntile) load_rows(Y, I0 + TB, yn);
        // the local recurrence from zero: d_q = yt_q - y_q = -F_q yt_{q-1}
        double d[BSL][4], prev[4];
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            d[0][s] = 0.0;
            prev[s] = (double)y[0][s];
        }
#pragma unroll
        for (int q = 1; q < BSL; ++q) {
            const doublex4 acc = product(mloc[q], prev);
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                d[q][s] = -acc[s];
                prev[s] = (double)y[q][s] + d[q][s];
            }
        }
#pragma unroll
        for (int q = 0; q < BSL; ++q) load_mat(I0 + q, 3, mloc[q]);          // the correction's propagators
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            ends[wave][lane * 4 + s] = prev[s];
            chm[wave][lane * 4 + s] = mine[s];
        }
        lds_barrier();
        // the value entering this segment: the tile's carry through the segments before it
        double c[4];
#pragma unroll
        for (int s = 0; s < 4; ++s) c[s] = carry[lane * 4 + s];
        for (int w = 0; w < wave; ++w) {
            double m[4];
#pragma unroll
            for (int s = 0; s < 4; ++s) m[s] = chm[w][lane * 4 + s];
            const doublex4 acc = product(m, c);
#pragma unroll
            for (int s = 0; s < 4; ++s) c[s] = ends[w][lane * 4 + s] + acc[s];
        }
        // correction and hand-over: r_q = d_q + Pf_q c
        double cend[4];
#pragma unroll
        for (int q = 0; q < BSL; ++q) {
            const doublex4 acc = product(mloc[q], c);
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const long row = (long)(I0 + q) * 16 + 4 * s + kq;
                const float r = (float)(d[q][s] + acc[s]);
                if (FULL || (jok && I0 + q < nbk && row < n)) S[row * p + j] = r;
                if (q == BSL - 1) cend[s] = (double)y[q][s] + (d[q][s] + acc[s]);
            }
        }
        lds_barrier();                                   // every wave has read the carry and the ends
        if (wave == SW - 1) {
#pragma unroll
            for (int s = 0; s < 4; ++s) carry[lane * 4 + s] = cend[s];
        }
#pragma unroll
        for (int q = 0; q < BSL; ++q)
#pragma unroll
            for (int s = 0; s < 4; ++s) y[q][s] = yn[q][s];
        lds_barrier();
    }

    // ---- backward: u_I = (rho Delta_I^-1) yh_I - G_I u_{I+1}, S_I = y_I - u_I ----------------------------------------
    // (every thread reads back exactly the entries of r it has written itself)
    if (tid < 256) carry[tid] = 0.0;
    float r[BSL][4], rn[BSL][4];
    load_rows(Y, (ntile - 1) * TB + wave * BSL, y);
    load_rows(S, (ntile - 1) * TB + wave * BSL, r);
    lds_barrier();
    for (int t = ntile - 1; t >= 0; --t) {
        const int I0 = t * TB + wave * BSL;
        double mz[BSL][4], mg[BSL][4], mine[4];
#pragma unroll
        for (int q = BSL - 1; q >= 0; --q) {
            load_mat(I0 + q, 1, mz[q]);
            if (q < BSL - 1) load_mat(I0 + q, 2, mg[q]);
        }
        load_mat(I0, 4, mine);                           // this segment's propagator, for the waves before this one
        if (!FULL || t > 0) {
            load_rows(Y, I0 - TB, yn);
            load_rows(S, I0 - TB, rn);
        }
        // z_q = (rho Delta_q^-1) yh_q, then the local recurrence from zero, from the segment's last block row up
        double u[BSL][4], next[4] = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
        for (int q = BSL - 1; q >= 0; --q) {
            double yh[4];
#pragma unroll
            for (int s = 0; s < 4; ++s) yh[s] = (double)y[q][s] + (double)r[q][s];
            doublex4 acc = product(mz[q], yh);
            if (q < BSL - 1) {
                const doublex4 acc2 = product(mg[q], next);
#pragma unroll
                for (int s = 0; s < 4; ++s) acc[s] -= acc2[s];
            }
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                u[q][s] = acc[s];
                next[s] = acc[s];
            }
        }
#pragma unroll
        for (int q = 0; q < BSL; ++q) load_mat(I0 + q, 4, mz[q]);            // the correction's propagators
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            ends[wave][lane * 4 + s] = next[s];
            chm[wave][lane * 4 + s] = mine[s];
        }
        lds_barrier();
        double c[4];
#pragma unroll
        for (int s = 0; s < 4; ++s) c[s] = carry[lane * 4 + s];
        for (int w = SW - 1; w > wave; --w) {
            double m[4];
#pragma unroll
            for (int s = 0; s < 4; ++s) m[s] = chm[w][lane * 4 + s];
            const doublex4 acc = product(m, c);
#pragma unroll
            for (int s = 0; s < 4; ++s) c[s] = ends[w][lane * 4 + s] + acc[s];
        }
        double cend[4];
#pragma unroll
        for (int q = 0; q < BSL; ++q) {
            const doublex4 acc = product(mz[q], c);
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const long row = (long)(I0 + q) * 16 + 4 * s + kq;
                const double uu = u[q][s] + acc[s];
                if (q == 0) cend[s] = uu;
                const float sv = (float)((double)y[q][s] - uu);
                if (FULL || (jok && I0 + q < nbk && row < n)) {
                    S[row * p + j] = sv;
                    smax = max(smax, __float_as_uint(fabsf(sv)));
                }
            }
        }
        lds_barrier();
        if (wave == 0) {
#pragma unroll
            for (int s = 0; s < 4; ++s) carry[lane * 4 + s] = cend[s];
        }
#pragma unroll
        for (int q = 0; q < BSL; ++q)
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                y[q][s] = yn[q][s];
                r[q][s] = rn[q][s];
            }
        lds_barrier();
    }
    if (amax_out) {
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) smax = max(smax, (unsigned)__shfl_xor((int)smax, o));
        if (lane == 0 && smax > __atomic_load_n(amax_out, __ATOMIC_RELAXED)) atomicMax(amax_out, smax);
    }
}

}  // namespace

size_t admmq_band_factor_doubles(int64_t n, int count) {
    const size_t nbk = ((size_t)n + BW - 1) / BW;
    return (size_t)count * nbk * BMATS * 256;
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
    // the split sweeps (eight segments per tile; sixteen, in blocks of 1024 threads with half the registers each, are
    // slower: 0.19 against 0.15 ms at 4096 x 4096); ADMMQ_BAND_SOLVE=chain: the unsplit ones, one wave per strip
    // (read at every call).  A block of the split sweeps fills a compute unit's registers, so its strips go in rounds
    // of one per unit; with more strips than units (25600 x 5120: 320 against 256) the unsplit sweeps, whose blocks
    // are small, are a little faster (1.47 against 1.56 ms).  The split ones are used all the same: a column's
    // result must not depend on how many columns share the call (several matrices on one Hessian).
    const char *solve_env = getenv("ADMMQ_BAND_SOLVE");
    const bool split = !(solve_env && solve_env[0] == 'c');
    if (split) {
        constexpr int SW = 8;
        const unsigned blocks = (unsigned)((p + 15) / 16);
        const bool whole = n % BW == 0 && p % 16 == 0 && nbk % (SW * BSL) == 0;
        if (whole)
            hipLaunchKernelGGL((band_apply_split_kernel<SW, true>), dim3(blocks), dim3(64 * SW), 0, ctx->stream, fac, nbk,
                               (long)n, (long)p, Y, S, amax_out);
        else
            hipLaunchKernelGGL((band_apply_split_kernel<SW, false>), dim3(blocks), dim3(64 * SW), 0, ctx->stream, fac, nbk,
                               (long)n, (long)p, Y, S, amax_out);
        ADMMQ_HIP(hipGetLastError());
        return ADMMQ_OK;
    }
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
