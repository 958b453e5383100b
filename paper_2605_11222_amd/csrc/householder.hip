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
#include <stdlib.h>

#include "common.h"

namespace {

constexpr int NB = 32;

typedef double doublex4 __attribute__((ext_vector_type(4)));

// Sum over the 64 lanes, left in every lane, without a trip through LDS: the two halves and the 16-lane rows are
// folded with the gfx950 lane-swap instructions, the rows with DPP rotations by 8, 4, 2, 1 (a fixed order).
template <int N>
__device__ inline double row_ror_add(double v) {
    const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(v), 0x120 + N, 0xF, 0xF, true);
    const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(v), 0x120 + N, 0xF, 0xF, true);
    return v + __hiloint2double(hi, lo);
}
__device__ inline double swap_fold32(double a) {
    const auto lo = __builtin_amdgcn_permlane32_swap((unsigned)__double2loint(a), (unsigned)__double2loint(a), false, false);
    const auto hi = __builtin_amdgcn_permlane32_swap((unsigned)__double2hiint(a), (unsigned)__double2hiint(a), false, false);
    return __hiloint2double((int)hi[0], (int)lo[0]) + __hiloint2double((int)hi[1], (int)lo[1]);
}
__device__ inline double swap_fold16(double a) {
    const auto lo = __builtin_amdgcn_permlane16_swap((unsigned)__double2loint(a), (unsigned)__double2loint(a), false, false);
    const auto hi = __builtin_amdgcn_permlane16_swap((unsigned)__double2hiint(a), (unsigned)__double2hiint(a), false, false);
    return __hiloint2double((int)hi[0], (int)lo[0]) + __hiloint2double((int)hi[1], (int)lo[1]);
}
__device__ inline double wave_sum(double v) {
    v = swap_fold32(v);
    v = swap_fold16(v);
    v = row_ror_add<8>(v);
    v = row_ror_add<4>(v);
    v = row_ror_add<2>(v);
    v = row_ror_add<1>(v);
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
constexpr int PART_W = 2 * NB + 4;   // partials per block: squared norm + 2 dots per slot (+ 3 values of block 0)
constexpr int PX_DIAG = 2 * NB + 1, PX_LEAD = 2 * NB + 2, PX_WLEAD = 2 * NB + 3;

// One butterfly step of a two-slot reduction over the lane halves (32) or alternating 16-lane rows (16): on return
// the lanes of the lower half / even rows hold a + (a from the partner lane), the others b + (b from the partner).
__device__ inline double swap_add32(double a, double b) {
    const unsigned alo = (unsigned)__double2loint(a), ahi = (unsigned)__double2hiint(a);
    const unsigned blo = (unsigned)__double2loint(b), bhi = (unsigned)__double2hiint(b);
    const auto lo = __builtin_amdgcn_permlane32_swap(alo, blo, false, false);
    const auto hi = __builtin_amdgcn_permlane32_swap(ahi, bhi, false, false);
    return __hiloint2double((int)hi[0], (int)lo[0]) + __hiloint2double((int)hi[1], (int)lo[1]);
}
__device__ inline double swap_add16(double a, double b) {
    const unsigned alo = (unsigned)__double2loint(a), ahi = (unsigned)__double2hiint(a);
    const unsigned blo = (unsigned)__double2loint(b), bhi = (unsigned)__double2hiint(b);
    const auto lo = __builtin_amdgcn_permlane16_swap(alo, blo, false, false);
    const auto hi = __builtin_amdgcn_permlane16_swap(ahi, bhi, false, false);
    return __hiloint2double((int)hi[0], (int)lo[0]) + __hiloint2double((int)hi[1], (int)lo[1]);
}

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
                                                      const double *__restrict__ part2, int nparts2, int sym,
                                                      int finalise) {
    __shared__ double vk[NB], wk[NB];
    __shared__ double xs[4];
    __shared__ double red[4][PART_W];
    __shared__ double tot[PART_W];
    __shared__ double scale_sh;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const long j = k + (long)blockIdx.x * ROW_CHUNK + tid;
    const bool ok = j < n;
    const long jj = ok ? j : n - 1;              // clamped index: loads stay in bounds, results unused
    const int cf = c - 1;                        // the slot that do_finish completes
    // ---- every load that depends on nothing computed here is issued first: one round trip, not four ----------
    double ds = 0.0;
    if (do_finish)
        for (int b = tid; b < nparts2; b += 256) ds += part2[b];
    double tp = 0.0, pj = 0.0, vpj = 0.0, pk = 0.0, vpk = 0.0;
    if (do_finish) {
        tp = tau[k - 1];
        pj = pbuf[jj];
        vpj = Vp[(long)cf * n + jj];
        pk = pbuf[k];
        vpk = Vp[(long)cf * n + k];
    }
    double vk_raw = 0.0, wk_raw = 0.0, w_lead = 0.0, v_lead = 0.0;
    double wq[NB], vq[NB];
    double x = 0.0;
    if (do_start) {
        if (tid < c) {
            vk_raw = Vp[(long)tid * n + k];
            v_lead = Vp[(long)tid * n + k + 1];
            if (!(do_finish && tid == cf)) {     // that slot's W is being written by this launch
                wk_raw = Wp[(long)tid * n + k];
                w_lead = Wp[(long)tid * n + k + 1];
            }
        }
        // this element's entries of every earlier slot serve both the row update and the dots below;
        // slots >= c are predicated off (c is uniform)
#pragma unroll
        for (int q = 0; q < NB; ++q) {
            wq[q] = (q < c && !(do_finish && q == cf)) ? Wp[(long)q * n + jj] : 0.0;
            vq[q] = q < c ? Vp[(long)q * n + jj] : 0.0;
        }
        // with only the lower triangle of the trailing matrix kept up to date, row k is read as column k
        x = ok ? (sym ? A[j * n + k] : A[k * n + j]) : 0.0;
    }
    // ---- finish column k-1 ---------------------------------------------------------------------------------
    double wnew = 0.0, wk_last = 0.0;
    if (do_finish) {
        // p'.v of column k-1: the block partials of its product kernel, added in a fixed order
        ds = wave_sum(ds);
        if (lane == 0) xs[wave] = ds;
        __syncthreads();
        const double pdotv = (xs[0] + xs[1]) + (xs[2] + xs[3]);
        const double cc = 0.5 * tp * tp * pdotv;
        if (ok) {
            wnew = tp * pj - cc * vpj;
            Wp[(long)cf * n + j] = wnew;
        }
        wk_last = tp * pk - cc * vpk;
    }
    if (!do_start) return;
    if (tid < c) {
        vk[tid] = vk_raw;
        wk[tid] = (do_finish && tid == cf) ? wk_last : wk_raw;
    }
#pragma unroll
    for (int q = 0; q < NB; ++q)
        if (do_finish && q == cf) wq[q] = wnew;
    __syncthreads();
#pragma unroll
    for (int q = 0; q < NB; ++q)
        if (q < c) x -= vk[q] * wq[q] + wk[q] * vq[q];
    if (ok) xbuf[j] = x;
    const double xt = (ok && j >= k + 2) ? x : 0.0;      // the reflector's tail
    // block partials: [0] squared tail norm, [1+2q] W_q . x_tail, [2+2q] V_q . x_tail; block 0 adds
    // [PX_DIAG] x[k], [PX_LEAD] x[k+1], [PX_WLEAD] the W entry at k+1 of the slot completed above
    const int nred = 1 + 2 * c;
    {
        const double s0 = wave_sum(xt * xt);
        if (lane == 0) red[wave][0] = s0;
    }
    // The 2 NB dots of the wave are reduced together: at the step with lane distance h every lane keeps the half
    // of its values whose slot has bit h equal to its own lane bit and hands the other half to its partner, so
    // after six steps lane L holds the complete sum of slot L.  63 exchanges instead of 6 per dot, no branches
    // (slots >= c hold zeros), the same pairwise order every time.
    {
        double v[2 * NB];
#pragma unroll
        for (int q = 0; q < NB; ++q) {
            v[2 * q] = wq[q] * xt;
            v[2 * q + 1] = vq[q] * xt;
        }
        // lane distances 32 and 16: the gfx950 lane-swap instructions do the exchange and the selection in one
        // step (checked on the device: permlane32_swap(a, b) returns (a_low, b_low) and (a_high, b_high) over the
        // two halves of the wave; permlane16_swap the same over alternating rows of 16 lanes)
#pragma unroll
        for (int i = 0; i < NB; ++i) v[i] = swap_add32(v[i], v[i + NB]);
#pragma unroll
        for (int i = 0; i < NB / 2; ++i) v[i] = swap_add16(v[i], v[i + NB / 2]);
#pragma unroll
        for (int h = NB / 4; h >= 1; h >>= 1) {
            const bool up = (lane & h) != 0;
            // all exchanges of a level are issued before the first sum waits for one of them (the scheduling
            // barrier keeps the compiler from pairing every exchange with its own wait)
            double recv[NB / 4];
#pragma unroll
            for (int i = 0; i < h; ++i) recv[i] = __shfl_xor(up ? v[i] : v[i + h], h, 64);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < h; ++i) v[i] = (up ? v[i + h] : v[i]) + recv[i];
            __builtin_amdgcn_sched_barrier(0);
        }
        red[wave][1 + lane] = v[0];
    }
    __syncthreads();
    if (tid < nred)
        part[(long)blockIdx.x * PART_W + tid] = (red[0][tid] + red[1][tid]) + (red[2][tid] + red[3][tid]);
    if (blockIdx.x == 0) {
        if (tid == 0) part[PX_DIAG] = x;
        if (tid == 1) {
            part[PX_LEAD] = x;
            part[PX_WLEAD] = wnew;
        }
    }
    // without `finalise` the product kernel that follows adds the partials up itself, while its first loads are
    // in flight: the fence, the counter and a second pass over the partials drop out of the column's critical path
    if (!finalise) return;
    if (!last_block_done(counter, gridDim.x)) return;
    // add the block partials in block order: thread r owns partial r; eight blocks' worth of its loads are in
    // flight at a time, the additions stay in index order
    double run = 0.0;
    if (tid < nred) {
        const double *src = part + tid;
        unsigned b0 = 0;
        for (; b0 + 8 <= gridDim.x; b0 += 8) {
            double v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = coherent_load(src + (long)(b0 + u) * PART_W);
#pragma unroll
            for (int u = 0; u < 8; ++u) run += v[u];
        }
        for (; b0 < gridDim.x; ++b0) run += coherent_load(src + (long)b0 * PART_W);
    } else if (tid >= PX_DIAG && tid < PART_W) {
        run = coherent_load(part + tid);         // block 0's three plain values
    }
    if (tid < PART_W) tot[tid] = run;
    __syncthreads();
    if (tid == 0) {
        const double sig = tot[0];
        const double alpha = tot[PX_LEAD];
        double beta, tk, scale;
        if (sig == 0.0) {
            beta = alpha; tk = 0.0; scale = 0.0;
        } else {
            const double nrm = sqrt(alpha * alpha + sig);
            beta = alpha >= 0.0 ? -nrm : nrm;
            tk = (beta - alpha) / beta;
            scale = 1.0 / (alpha - beta);
        }
        ta[k] = tot[PX_DIAG];
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
        const double wl = (do_finish && tid == cf) ? tot[PX_WLEAD] : w_lead;
        sc[SC_DOTS + 2 * tid] = scale * tot[1 + 2 * tid] + wl;
        sc[SC_DOTS + 2 * tid + 1] = scale * tot[2 + 2 * tid] + v_lead;
    }
}

// p'[i] = sum_{j >= k+1} A[i][j] v[j] - sum_q (V_q[i] (W_q.v) + W_q[i] (V_q.v)) for i >= k+1, with
// v = (1, scale * xbuf).  A is only read below row k; the normalised v is stored in panel slot c and in row k
// of A (its permanent home).  One wave per row, 4 rows per block.
// The reflector's scalars are formed here, by every block for itself, from the block partials that
// tri_row_kernel left (nparts1 of them, added in block order): the loads of the partials and of the matrix rows
// are in flight together, and the row dots are taken with the unscaled xbuf and scaled afterwards
// (p'[i] = A[i][k+1] + scale * sum_{j > k+1} A[i][j] xbuf[j]), so nothing waits for the scalars.  Block 0 records
// T's entries, tau and the scale.
__global__ __launch_bounds__(256) void tri_mat_kernel(double *__restrict__ A, long n, long k, int c,
                                                      double *__restrict__ Vp, const double *__restrict__ Wp,
                                                      const double *__restrict__ xbuf, double *__restrict__ pbuf,
                                                      double *__restrict__ sc, double *__restrict__ part,
                                                      const double *__restrict__ part1, int nparts1,
                                                      double *__restrict__ tau, double *__restrict__ ta,
                                                      double *__restrict__ tb) {
    __shared__ double ad[NB], bd[NB];
    __shared__ double tot[PART_W];
    __shared__ double wsum[4];
    __shared__ double scale_sh;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nred = 1 + 2 * c;
    // ---- requests first: this thread's partial column, the leading entries, the matrix row -----------------
    double run = 0.0;
    if (tid < nred) {
        const double *src = part1 + tid;
        int b0 = 0;
        for (; b0 + 8 <= nparts1; b0 += 8) {
            double v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = src[(long)(b0 + u) * PART_W];
#pragma unroll
            for (int u = 0; u < 8; ++u) run += v[u];
        }
        for (; b0 < nparts1; ++b0) run += src[(long)b0 * PART_W];
    }
    double w_lead = 0.0, v_lead = 0.0;
    if (tid < c) {
        w_lead = Wp[(long)tid * n + k + 1];
        v_lead = Vp[(long)tid * n + k + 1];
    }
    const double x_diag = xbuf[k], alpha = xbuf[k + 1];
    const long i = k + 1 + (long)blockIdx.x * 4 + wave;
    double a0 = 0.0, a1 = 0.0, lead = 0.0, xi = 0.0, vcorr = 0.0, wcorr = 0.0;
    if (i < n) {
        const double *row = A + i * n;
        long j = k + 1 + lane;
        if (lane == 0) {                     // v[k+1] = 1
            lead = row[j];
            j += 64;
        }
        for (; j + 64 < n; j += 128) {
            a0 += row[j] * xbuf[j];
            a1 += row[j + 64] * xbuf[j + 64];
        }
        if (j < n) a0 += row[j] * xbuf[j];
        if (lane < c) {
            vcorr = Vp[(long)lane * n + i];
            wcorr = Wp[(long)lane * n + i];
        }
        xi = xbuf[i];
    }
    // ---- the reflector's scalars --------------------------------------------------------------------------------
    if (tid < nred) tot[tid] = run;
    __syncthreads();
    if (tid == 0) {
        const double sig = tot[0];
        double beta, tk, scale;
        if (sig == 0.0) {
            beta = alpha; tk = 0.0; scale = 0.0;
        } else {
            const double nrm = sqrt(alpha * alpha + sig);
            beta = alpha >= 0.0 ? -nrm : nrm;
            tk = (beta - alpha) / beta;
            scale = 1.0 / (alpha - beta);
        }
        scale_sh = scale;
        if (blockIdx.x == 0) {
            ta[k] = x_diag;
            tb[k] = beta;
            tau[k] = tk;
            sc[SC_SCALE] = scale;
        }
    }
    __syncthreads();
    const double scale = scale_sh;
    if (tid < c) {
        // v = (1, scale * x_tail): dots with the earlier slots, the leading 1 sits at index k+1
        ad[tid] = scale * tot[1 + 2 * tid] + w_lead;
        bd[tid] = scale * tot[2 + 2 * tid] + v_lead;
    }
    __syncthreads();
    double wdot = 0.0;
    if (i < n) {
        double t = lead + scale * (a0 + a1);
        if (lane < c) t -= vcorr * ad[lane] + wcorr * bd[lane];
        t = wave_sum(t);
        if (lane == 0) {
            const double vi = (i == k + 1) ? 1.0 : xi * scale;
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

// ---- the same product from the lower triangle alone (large trailing matrices) ---------------------------------
// While the trailing matrix is too large for the caches the product is bound by reading it; a symmetric matrix
// needs only its lower triangle read: tile (I, J), J <= I, of 64 x 64 entries adds A_IJ v_J to rows I and
// A_IJ^T v_I to rows J.  Every tile writes its two pieces to slots of their own, Pb[T][S][64] (T = the tile row
// the piece belongs to, S = the other tile index), and tri_symv_finish_kernel adds the slots of a row in index
// order: no atomics, a fixed order.  In this mode only entries with i >= j of the trailing matrix are kept up to
// date (tri_update_kernel skips the strictly upper tiles, tri_row_kernel reads column k for row k).
// Tiles are anchored at multiples of 64 of the global index; t0 = (k+1)/64 is the first tile, nt their number.
constexpr int ST = 64;

__device__ inline void tri_tile_of(int id, int &ti, int &tj) {
    ti = (int)((sqrtf(8.f * (float)id + 1.f) - 1.f) * 0.5f);
    while ((long)(ti + 1) * (ti + 2) / 2 <= id) ++ti;
    while ((long)ti * (ti + 1) / 2 > id) --ti;
    tj = id - ti * (ti + 1) / 2;
}

// grid nt (nt + 1) / 2 blocks of 256 threads, one per tile on or below the diagonal; thread (ty, tx) owns rows
// ty*4.., columns tx*4.. of it.  (Measured at n = 25600: two or four tiles per block, or a square grid whose
// upper blocks leave at once, are 3 to 10 % slower.)
constexpr int SG = 1;
__global__ __launch_bounds__(256) void tri_symv_tile_kernel(const double *__restrict__ A, long n, long k,
                                                            const double *__restrict__ xbuf,
                                                            const double *__restrict__ sc, double *__restrict__ Pb,
                                                            int t0, int nt) {
    __shared__ double rs[SG][ST], cs[SG][4][ST];
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4, wave = tid >> 6;
    int ti, tj0;
    tri_tile_of((int)blockIdx.x, ti, tj0);           // one block per tile of the lower triangle, none idle
    if (ti >= nt) return;                            // cannot happen with that grid; keeps indices in range
    const long i0 = ((long)t0 + ti) * ST + ty * 4;
    const double scale = sc[SC_SCALE];
    const long lead = k + 1;                         // v[lead] = 1, v = 0 before it
    double xr[4];
#pragma unroll
    for (int a = 0; a < 4; ++a) {
        const long i = i0 + a;
        xr[a] = (i < lead || i >= n) ? 0.0 : (i == lead ? 1.0 : xbuf[i] * scale);
    }
    // a tile strictly below the diagonal and wholly inside the trailing block, rows 32-byte aligned: four
    // 32-byte loads per thread, no masks (the block decides as one)
    doublex4 rowv[SG][4];
    bool whole[SG];
#pragma unroll
    for (int u = 0; u < SG; ++u) {
        const int tj = tj0 + u;
        whole[u] = tj < ti && ((long)t0 + tj) * ST >= lead && ((long)t0 + ti + 1) * ST <= n && (n & 3) == 0;
        if (whole[u]) {
            const long j0 = ((long)t0 + tj) * ST + tx * 4;
#pragma unroll
            for (int a = 0; a < 4; ++a) rowv[u][a] = *(const doublex4 *)(A + (i0 + a) * n + j0);
        }
    }
#pragma unroll
    for (int u = 0; u < SG; ++u) {
        const int tj = tj0 + u;
        if (tj > ti) break;
        const long j0 = ((long)t0 + tj) * ST + tx * 4;
        const bool diag = ti == tj;
        double xc[4];
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const long j = j0 + b;
            xc[b] = (j < lead || j >= n) ? 0.0 : (j == lead ? 1.0 : xbuf[j] * scale);
        }
        double rsum[4] = {0.0, 0.0, 0.0, 0.0}, csum[4] = {0.0, 0.0, 0.0, 0.0};
        if (whole[u]) {
#pragma unroll
            for (int a = 0; a < 4; ++a) {
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    rsum[a] += rowv[u][a][b] * xc[b];
                    csum[b] += rowv[u][a][b] * xr[a];
                }
            }
        } else {
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                const long i = i0 + a;
                double row[4];
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    const long j = j0 + b;
                    // entries outside the trailing block, and above the diagonal, are never read
                    row[b] = (i >= lead && i < n && j >= lead && j <= i) ? A[i * n + j] : 0.0;
                }
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    rsum[a] += row[b] * xc[b];
                    // the transposed piece: strictly below the diagonal only (the diagonal is in the row piece)
                    if (!diag || j0 + b < i) csum[b] += row[b] * xr[a];
                }
            }
        }
        // row pieces: add over the 16 tx lanes (adjacent lanes of one wave)
#pragma unroll
        for (int a = 0; a < 4; ++a) {
#pragma unroll
            for (int o = 1; o < 16; o <<= 1) rsum[a] += __shfl_xor(rsum[a], o, 64);
        }
        // column pieces: add over the ty groups of the wave, then over the four waves through LDS
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            csum[b] += __shfl_xor(csum[b], 16, 64);
            csum[b] += __shfl_xor(csum[b], 32, 64);
        }
        if (tx == 0) {
#pragma unroll
            for (int a = 0; a < 4; ++a) rs[u][ty * 4 + a] = rsum[a];
        }
        if ((tid & 63) < 16) {
#pragma unroll
            for (int b = 0; b < 4; ++b) cs[u][wave][tx * 4 + b] = csum[b];
        }
    }
    __syncthreads();
    {
        // thread (u, e): piece e of the group's tile u
        const int u = tid >> 6, e = tid & 63, tj = tj0 + u;
        if (u < SG && tj <= ti) {
            const double col = (cs[u][0][e] + cs[u][1][e]) + (cs[u][2][e] + cs[u][3][e]);
            if (tj == ti) {
                Pb[((long)ti * nt + ti) * ST + e] = rs[u][e] + col;
            } else {
                Pb[((long)ti * nt + tj) * ST + e] = rs[u][e];
                Pb[((long)tj * nt + ti) * ST + e] = col;
            }
        }
    }
}

// p'[i] = sum_S Pb[T][S][e] - sum_q (V_q[i] (W_q.v) + W_q[i] (V_q.v)); stores the normalised v in panel slot c and
// in row k of A, and the block partials of p'.v, exactly as tri_mat_kernel does.  Block = one tile row: wave w
// adds the slots S = w, w+4, ... (four loads in flight each), the four sums are combined in a fixed order.
__global__ __launch_bounds__(256) void tri_symv_finish_kernel(double *__restrict__ A, long n, long k, int c,
                                                              double *__restrict__ Vp,
                                                              const double *__restrict__ Wp,
                                                              const double *__restrict__ xbuf,
                                                              double *__restrict__ pbuf,
                                                              const double *__restrict__ sc,
                                                              const double *__restrict__ Pb, int t0, int nt,
                                                              double *__restrict__ part) {
    __shared__ double ad[NB], bd[NB];
    __shared__ double ys[4][ST];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const double scale = sc[SC_SCALE];
    if (tid < c) {
        ad[tid] = sc[SC_DOTS + 2 * tid];
        bd[tid] = sc[SC_DOTS + 2 * tid + 1];
    }
    const int T = (int)blockIdx.x;
    const double *src = Pb + (long)T * nt * ST + lane;
    double y0 = 0.0, y1 = 0.0, y2 = 0.0, y3 = 0.0;
    int S = wave;
    for (; S + 12 < nt; S += 16) {
        y0 += src[(long)S * ST];
        y1 += src[(long)(S + 4) * ST];
        y2 += src[(long)(S + 8) * ST];
        y3 += src[(long)(S + 12) * ST];
    }
    for (; S < nt; S += 4) y0 += src[(long)S * ST];
    ys[wave][lane] = (y0 + y1) + (y2 + y3);
    __syncthreads();
    const long i = ((long)t0 + T) * ST + lane;
    double wdot = 0.0;
    if (wave == 0) {
        if (i >= k + 1 && i < n) {
            double t = (ys[0][lane] + ys[1][lane]) + (ys[2][lane] + ys[3][lane]);
            for (int q = 0; q < c; ++q) t -= Vp[(long)q * n + i] * ad[q] + Wp[(long)q * n + i] * bd[q];
            const double vi = (i == k + 1) ? 1.0 : xbuf[i] * scale;
            pbuf[i] = t;
            Vp[(long)c * n + i] = vi;
            A[k * n + i] = vi;
            wdot = t * vi;
        }
        wdot = wave_sum(wdot);
        if (lane == 0) part[blockIdx.x] = wdot;
    }
}

// A[j][i] = A[i][j] for i > j >= r0: the upper triangle of the trailing block is brought up to date when the
// factorisation leaves the lower-triangle mode.  32 x 32 tiles through LDS; grid over tile pairs with ti >= tj.
__global__ void tri_mirror_kernel(double *__restrict__ A, long n, long r0) {
    __shared__ double tile[32][33];
    const int tx = threadIdx.x, ty = threadIdx.y;     // 32 x 8
    int ti, tj;
    tri_tile_of((int)blockIdx.x, ti, tj);
    const long i0 = r0 + (long)ti * 32, j0 = r0 + (long)tj * 32;
    for (int r = ty; r < 32; r += 8) {
        const long i = i0 + r, j = j0 + tx;
        tile[r][tx] = (i < n && j < n) ? A[i * n + j] : 0.0;
    }
    __syncthreads();
    for (int r = ty; r < 32; r += 8) {
        const long j = j0 + r, i = i0 + tx;           // writes A[j][i], contiguous in i
        if (i < n && j < n && i > j) A[j * n + i] = tile[tx][r];
    }
}

// A[i][j] -= sum_c V_c[i] W_c[j] + W_c[i] V_c[j] for i, j >= r0.  64 x 64 tile per block on the fp64 matrix
// cores: wave w owns rows 16w..16w+15, four 16-column blocks, two products per step of four panel slots.
// lower_only: tiles strictly above the diagonal are left alone (only entries with i >= j are kept up to date).
__global__ __launch_bounds__(256) void tri_update_kernel(double *__restrict__ A, long n, long r0, int nbc,
                                                         const double *__restrict__ Vp,
                                                         const double *__restrict__ Wp, int lower_only) {
    constexpr int CC = 16, LD = 80;      // row stride 640 B: the two k-rows a half-wave reads use disjoint banks
    __shared__ double Vi[CC][LD], Wi[CC][LD], Vj[CC][LD], Wj[CC][LD];
    if (lower_only && blockIdx.x > blockIdx.y) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l16 = lane & 15, lq = lane >> 4;
    const long i0 = r0 + (long)blockIdx.y * 64, j0 = r0 + (long)blockIdx.x * 64;
    // the tile's own entries are requested first
    double av[4][4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const long i = i0 + wave * 16 + 4 * r + lq;
#pragma unroll
        for (int bb = 0; bb < 4; ++bb) {
            const long j = j0 + bb * 16 + l16;
            av[r][bb] = (i < n && j < n) ? A[i * n + j] : 0.0;
        }
    }
    doublex4 acc[4];
#pragma unroll
    for (int bb = 0; bb < 4; ++bb) acc[bb] = doublex4{0.0, 0.0, 0.0, 0.0};
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
        for (int c = 0; c < CC; c += 4) {
            const double v = Vi[c + lq][wave * 16 + l16], w = Wi[c + lq][wave * 16 + l16];
#pragma unroll
            for (int bb = 0; bb < 4; ++bb) {
                acc[bb] = __builtin_amdgcn_mfma_f64_16x16x4f64(v, Wj[c + lq][bb * 16 + l16], acc[bb], 0, 0, 0);
                acc[bb] = __builtin_amdgcn_mfma_f64_16x16x4f64(w, Vj[c + lq][bb * 16 + l16], acc[bb], 0, 0, 0);
            }
        }
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const long i = i0 + wave * 16 + 4 * r + lq;
        if (i >= n) continue;
#pragma unroll
        for (int bb = 0; bb < 4; ++bb) {
            const long j = j0 + bb * 16 + l16;
            if (j < n) A[i * n + j] = av[r][bb] - acc[bb][r];
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

// The accumulation works on blocks of NBT reflectors: 32 beside the tridiagonal chain (one panel), 64 for the band
// form (four panels: R is read and written once per 64 reflectors instead of once per 32).
// Reflector k0+c is row k0+c of A on indices >= k0+c+off (leading 1 stored); off = 1 for the tridiagonal
// reduction, the band width for the reduction to band form.  S[c1][c2] = v_c1 . v_c2.
// grid (nbc, nbc), block 256; only c1 <= c2 is computed (and mirrored).
template <int NBT>
__global__ __launch_bounds__(256) void q_gram_kernel(const double *__restrict__ A, long n, long k0, int nbc,
                                                     double *__restrict__ S, int off) {
    __shared__ double sh[4];
    const int c1 = blockIdx.y, c2 = blockIdx.x;
    if (c1 > c2) return;
    const double *v1 = A + (k0 + c1) * n, *v2 = A + (k0 + c2) * n;
    double s = 0.0;
    for (long i = k0 + c2 + off + threadIdx.x; i < n; i += 256) s += v1[i] * v2[i];
    s = wave_sum(s);
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        const double t = (sh[0] + sh[1]) + (sh[2] + sh[3]);
        S[c1 * NBT + c2] = t;
        S[c2 * NBT + c1] = t;
    }
}

// T of the compact WY form (forward, column-wise): T[c][c] = tau_c,
// T[0:c, c] = -tau_c T[0:c, 0:c] S[0:c, c].  One block of NBT threads (thread r owns row r); the Gram matrix is kept
// as its packed upper triangle (two full 64 x 64 arrays of doubles would not fit the static LDS limit).
template <int NBT>
__global__ void q_tfactor_kernel(const double *__restrict__ S, const double *__restrict__ tau, long k0, int nbc,
                                 double *__restrict__ T) {
    __shared__ double Ts[NBT][NBT + 1];
    __shared__ double Sp[NBT * (NBT + 1) / 2];          // S[q][c], q <= c, at c (c + 1) / 2 + q
    __shared__ double taus[NBT];
    const int r = threadIdx.x;
    for (int c = 0; c < NBT; ++c) {
        Ts[r][c] = 0.0;
        if (r <= c) Sp[c * (c + 1) / 2 + r] = S[r * NBT + c];      // the Gram matrix and the taus are fetched once, up front
    }
    taus[r] = r < nbc ? tau[k0 + r] : 0.0;
    __syncthreads();
    for (int c = 0; c < nbc; ++c) {
        const double tc = taus[c];
        if (r < c) {
            double s = 0.0;
            for (int q = r; q < c; ++q) s += Ts[r][q] * Sp[c * (c + 1) / 2 + q];
            Ts[r][c] = -tc * s;
        } else if (r == c) {
            Ts[r][c] = tc;
        }
        __syncthreads();
    }
    for (int c = 0; c < NBT; ++c) T[r * NBT + c] = Ts[r][c];
}

// Gp[s][j][c] = sum over slice s of i of R[j][i] v_c[i]  for rows j >= jstart (the slices of the
// contraction index give the chip enough blocks; they are added in a fixed order by the consumer).
// Block: 64 rows x NBT columns on the fp64 matrix cores (v_mfma_f64_16x16x4), one 16-row strip per wave.
// grid: any number of blocks up to row_tiles * ks.
constexpr int WY_KS_MAX = 16;
template <int NBT>
__global__ __launch_bounds__(256) void q_wy_g_kernel(const double *__restrict__ R, const double *__restrict__ A,
                                                     long n, long k0, int nbc, long chunk,
                                                     double *__restrict__ Gp, long jstart, int row_tiles, int ks,
                                                     int off) {
    constexpr int KC = 32;
    __shared__ double Rs[64][KC + 1];
    __shared__ double Vs[NBT][KC + 1];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l16 = lane & 15, lq = lane >> 4;
    // (row block, slice) pairs are walked with the grid's stride: a launch with few blocks leaves the rest of the
    // chip to the stream it runs beside
    for (long id = blockIdx.x; id < (long)row_tiles * ks; id += gridDim.x) {
        const long bx = id % row_tiles, by = id / row_tiles;
        const long j0 = jstart + bx * 64;           // first row of the block (rows jstart .. n-1)
        const long ibeg = k0 + off + by * chunk;
        const long iend = min(n, ibeg + chunk);
        // wave w owns rows 16w..16w+15 of the block, all NBT columns: NBT / 16 accumulators of 16 x 16
        doublex4 acc[NBT / 16];
#pragma unroll
        for (int b = 0; b < NBT / 16; ++b) acc[b] = doublex4{0.0, 0.0, 0.0, 0.0};
        for (long i0 = ibeg; i0 < iend; i0 += KC) {
            __syncthreads();
            for (int e = tid; e < 64 * KC; e += 256) {
                const int r = e / KC, q = e % KC;
                const long j = j0 + r, i = i0 + q;
                Rs[r][q] = (j < n && i < iend) ? R[j * n + i] : 0.0;
            }
            for (int e = tid; e < NBT * KC; e += 256) {
                const int c = e / KC, q = e % KC;
                const long i = i0 + q;
                Vs[c][q] = (c < nbc && i < iend && i >= k0 + c + off) ? A[(k0 + c) * n + i] : 0.0;
            }
            __syncthreads();
#pragma unroll
            for (int q = 0; q < KC; q += 4) {
                // matrix-core operands: A[row = lane%16][k = lane/16], B[k = lane/16][col = lane%16]
                const double a = Rs[wave * 16 + l16][q + lq];
#pragma unroll
                for (int b = 0; b < NBT / 16; ++b)
                    acc[b] = __builtin_amdgcn_mfma_f64_16x16x4f64(a, Vs[16 * b + l16][q + lq], acc[b], 0, 0, 0);
            }
        }
        // accumulator register r of lane l holds row 4r + l/16, column l%16 of its 16 x 16 block
        double *out = Gp + by * n * NBT;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const long j = j0 + wave * 16 + 4 * r + lq;
            if (j < n) {
#pragma unroll
                for (int b = 0; b < NBT / 16; ++b) out[j * NBT + 16 * b + l16] = acc[b][r];
            }
        }
    }
}

// G2[j][c] = sum_q (sum_s Gp[s][j][q]) T[c][q] for rows j >= jstart: the slices of the contraction are added in
// index order and the small triangular factor applied once per row (not once per tile of the update).
// One thread per (row, c); block 256 = 256 / NBT rows.
template <int NBT>
__global__ __launch_bounds__(256) void q_wy_g2_kernel(const double *__restrict__ Gp, const double *__restrict__ T,
                                                      long n, long k0, int nbc, int ks,
                                                      double *__restrict__ G2, long jstart, int forward) {
    constexpr int RPB = 256 / NBT;
    __shared__ double Ts[NBT][NBT + 1];
    __shared__ double Gs[RPB][NBT + 1];
    const int tid = threadIdx.x, c = tid & (NBT - 1), r = tid / NBT;
    for (int e = tid; e < NBT * NBT; e += 256) Ts[e / NBT][e % NBT] = T[e];
    const long j = jstart + (long)blockIdx.x * RPB + r;
    double g = 0.0;
    if (j < n && c < nbc)
        for (int s = 0; s < ks; ++s) g += Gp[((long)s * n + j) * NBT + c];
    Gs[r][c] = g;
    __syncthreads();
    if (j < n) {
        double t = 0.0;
        if (forward) {
            for (int q = 0; q <= c && q < nbc; ++q) t += Gs[r][q] * Ts[q][c];      // (G T)[c]
        } else {
            for (int q = c; q < nbc; ++q) t += Gs[r][q] * Ts[c][q];      // (G T^T)[c]; T is upper triangular
        }
        G2[j * NBT + c] = t;
    }
}

// R[j][i] -= sum_c G2[j][c] v_c[i]  for j >= jstart, i >= k0+off.  64 x 64 tile per block; the product runs on the fp64
// matrix cores: wave w owns rows 16w..16w+15 of the tile, four 16-column blocks; the reflectors go through LDS 32 at
// a time.
template <int NBT>
__global__ __launch_bounds__(256) void q_wy_update_kernel(double *__restrict__ R, const double *__restrict__ A,
                                                          long n, long k0, int nbc,
                                                          const double *__restrict__ G2, long jstart, int col_tiles,
                                                          int row_tiles, int off) {
    constexpr int CH = 32;
    __shared__ double G2s[64][CH + 1];
    __shared__ double Vs[CH][80];          // row stride 640 B: the two k-rows a half-wave reads use disjoint banks
    const int tid = threadIdx.x;
    for (long id = blockIdx.x; id < (long)col_tiles * row_tiles; id += gridDim.x) {
        const long bx = id % col_tiles, by = id / col_tiles;
        const long j0 = jstart + by * 64, i0 = k0 + off + bx * 64;
        const int lane = tid & 63, wave = tid >> 6, l16 = lane & 15, lq = lane >> 4;
        // the tile's own entries are requested before the operands are waited for
        double rv[4][4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const long j = j0 + wave * 16 + 4 * r + lq;
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                const long i = i0 + b * 16 + l16;
                rv[r][b] = (j < n && i < n) ? R[j * n + i] : 0.0;
            }
        }
        doublex4 acc[4];
#pragma unroll
        for (int b = 0; b < 4; ++b) acc[b] = doublex4{0.0, 0.0, 0.0, 0.0};
        for (int cb = 0; cb < NBT; cb += CH) {
            if (cb > 0) __syncthreads();           // the chunk before has been read
            for (int e = tid; e < 64 * CH; e += 256) {
                const int r = e / CH, c = e % CH;
                const long j = j0 + r;
                G2s[r][c] = (j < n && cb + c < nbc) ? G2[j * NBT + cb + c] : 0.0;
            }
            for (int e = tid; e < CH * 64; e += 256) {
                const int c = e >> 6, o = e & 63;
                const long i = i0 + o;
                Vs[c][o] = (cb + c < nbc && i < n && i >= k0 + cb + c + off) ? A[(k0 + cb + c) * n + i] : 0.0;
            }
            __syncthreads();
#pragma unroll
            for (int c = 0; c < CH; c += 4) {
                const double g = G2s[wave * 16 + l16][c + lq];
#pragma unroll
                for (int b = 0; b < 4; ++b)
                    acc[b] = __builtin_amdgcn_mfma_f64_16x16x4f64(g, Vs[c + lq][b * 16 + l16], acc[b], 0, 0, 0);
            }
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const long j = j0 + wave * 16 + 4 * r + lq;
            if (j >= n) continue;
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                const long i = i0 + b * 16 + l16;
                if (i < n) R[j * n + i] = rv[r][b] - acc[b][r];
            }
        }
        __syncthreads();                   // the next tile refills the two LDS arrays
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

// ---- reduction to band form (block reflectors) -------------------------------------------------------------------
// Hs = Q Bd Q^T with Bd of half-bandwidth BW.  Per panel of BW columns c0 .. c0+BW-1 (r0 = c0 + BW, m = n - r0):
//   factor : the m x BW block below the band, P = A[r0:, c0:c0+BW], gets its QR factorisation from two rounds of
//            Cholesky-QR (Gram matrix over all rows on the matrix cores, 16 x 16 Cholesky, P R^-1), which costs three
//            passes over P by the whole chip instead of BW dependent column steps; the Householder form
//            I - Y T Y^T of the orthonormal factor is then rebuilt from an LU factorisation of its top BW x BW block
//            (signs chosen so that every pivot is at least 1) and one triangular solve per row below it
//   symm   : X = A[r0:, r0:] Y on the fp64 matrix cores, the contraction cut into slices
//   finish : K = Y^T X, S = T^T K T, W = X T - 1/2 Y S
//   update : A[r0:, r0:] -= Y W^T + W Y^T                       (the rank-2 BW kernel of the tridiagonal path)
// so every panel costs one read and one read+write of the trailing matrix, against one read per COLUMN for the
// one-stage tridiagonalisation, and no step depends on a single column's reduction.
// A panel whose Gram matrix is not safely positive definite (a rank-deficient block), and the last panels (fewer
// than 64 rows), take plain Householder steps in one block instead.
constexpr int BW = 16;
constexpr int QB = 64;           // reflectors per block of the accumulation of Q (four panels)
enum { BS_R1 = 0, BS_R1INV = 256, BS_Z = 512, BS_Y1 = 768, BS_T = 1024, BS_S2 = 1280, BS_FLAG = 1536, BS_COUNT = 1600 };

// entry `tid` of the per-block partial sums, added in block order; sixteen loads are in flight at a time (one load
// per trip would pay the memory latency once per block)
__device__ inline double sum_block_partials(const double *part, unsigned nb, int tid) {
    double g = 0.0;
    unsigned b = 0;
    for (; b + 16 <= nb; b += 16) {
        double v[16];
#pragma unroll
        for (int u = 0; u < 16; ++u) v[u] = coherent_load(part + (long)(b + u) * 256 + tid);
#pragma unroll
        for (int u = 0; u < 16; ++u) g += v[u];
    }
    for (; b < nb; ++b) g += coherent_load(part + (long)b * 256 + tid);
    return g;
}

// 16 x 16 factorisations in the registers of one wave.  "Column layout": lane j < 16 holds column j of the matrix,
// a[i] = M[i][j]; an entry another lane needs comes by v_readlane (the loops are fully unrolled, so every source
// lane is a constant).  Lanes 16 .. 63 run along on zeros; nothing of theirs is ever read.
__device__ inline double lane_bcast(double v, int src) {
    const int lo = __builtin_amdgcn_readlane(__double2loint(v), src), hi = __builtin_amdgcn_readlane(__double2hiint(v), src);
    return __hiloint2double(hi, lo);
}
// G = R^T R: in a = G (symmetric), out a = upper R (zeros below the diagonal).  False when a pivot is not safely
// positive (below 1e-12 of its diagonal entry: the panel's columns are close to dependent).
__device__ inline bool chol16_cols(double (&a)[16], int lane) {
    bool ok = true;
#pragma unroll
    for (int k = 0; k < 16; ++k) {
        const double g0 = lane_bcast(a[k], k);
        double acc = g0;                               // G[k][k] - sum_{i<k} R[i][k]^2, left-looking on the diagonal
#pragma unroll
        for (int i = 0; i < k; ++i) {
            const double rik = lane_bcast(a[i], k);
            acc -= rik * rik;
        }
        if (!(acc > 1e-12 * g0)) ok = false;
        const double inv = 1.0 / sqrt(acc > 0.0 ? acc : 1.0);
        // row k: R[k][j] = (G[k][j] - sum_{i<k} R[i][k] R[i][j]) / R[k][k] for j >= k
        double s = a[k];
#pragma unroll
        for (int i = 0; i < k; ++i) s -= lane_bcast(a[i], k) * a[i];
        a[k] = lane >= k ? s * inv : 0.0;
    }
    return ok;
}
// inverse of an upper triangular matrix, column layout in and out (x[i] = (R^-1)[i][lane])
__device__ inline void triu_inverse16_cols(const double (&a)[16], double (&x)[16], int lane) {
#pragma unroll
    for (int i = 15; i >= 0; --i) {
        double s = lane == i ? 1.0 : 0.0;
#pragma unroll
        for (int k = i + 1; k < 16; ++k) s -= lane_bcast(a[i], k) * x[k];       // R[i][k] sits in lane k
        x[i] = lane >= i ? s / lane_bcast(a[i], i) : 0.0;
    }
}
// LU without pivoting of Q - S, S = diag(sg) chosen against the sign of each pivot as it comes up, so that every
// pivot is at least 1 in size: a = Q in, out a = U on and above the diagonal, the multipliers (Y1 without its unit
// diagonal) below it.
__device__ inline void lu16_signed_cols(double (&a)[16], double (&sg)[16], int lane) {
#pragma unroll
    for (int k = 0; k < 16; ++k) {
        const double p0 = lane_bcast(a[k], k);
        sg[k] = p0 >= 0.0 ? -1.0 : 1.0;
        const double inv = 1.0 / (p0 - sg[k]);
        if (lane == k) {
            a[k] -= sg[k];
#pragma unroll
            for (int i = k + 1; i < 16; ++i) a[i] *= inv;
        }
#pragma unroll
        for (int i = k + 1; i < 16; ++i) {
            const double lik = lane_bcast(a[i], k);
            if (lane > k) a[i] -= lik * a[k];
        }
    }
}

// Gram matrix of a row panel (PASS 1: P = A[r0:, c0:c0+16]; PASS 2: Q1 = P R1^-1, which is also written to Pq
// [m][16]) as per-block partials, 64 rows per block (thread = row, four columns); the block that finishes last adds
// them in block order, factorises and leaves in `small`
//   PASS 1: R1, R1^-1
//   PASS 2: with R2 the factor of the second round and Q = Q1 R2^-1 (orthonormal columns, P = Q R, R = R2 R1): the
//           Householder form of Q from its top 16 x 16 block.  With S = diag(+-1) chosen against the sign of each
//           pivot, Q - [S; 0] = Y U (LU without pivoting, Y unit lower trapezoidal, every pivot at least 1 in size),
//           T = -U S Y1^-T, and (I - Y T Y^T)^T P = [S R; 0].  Left behind: Z = R2^-1 U^-1 (so that the rows below
//           the top block are Y = Q1 Z), Y1, T, tau = diag T, and the block S R in the band array;
// or raises small[BS_FLAG].  PASS 1 also writes the panel's diagonal block into the band array.  Needs m >= 16.
template <int PASS>
__global__ __launch_bounds__(256) void band_gram_kernel(const double *__restrict__ A, long n, long c0, long m,
                                                        double *__restrict__ Pq, double *__restrict__ small,
                                                        double *__restrict__ part, unsigned *__restrict__ counter,
                                                        double *__restrict__ bd, long npad,
                                                        double *__restrict__ tau) {
    __shared__ double tile[64][17];
    __shared__ double Ms[16][17], Rs[16][17], Ri[16][17], Lu[16][17], Ts[16][17];
    __shared__ double red[4][256];
    __shared__ double sg[16];
    __shared__ int flag_sh;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l16 = lane & 15, lq = lane >> 4;
    const long r0 = c0 + BW;
    if (PASS == 2 && small[BS_FLAG] != 0.0) return;
    if (PASS == 1 && blockIdx.x == 0) {
        const int s = tid >> 4, u = tid & 15;
        if (s >= u && c0 + s < n) bd[(long)(s - u) * npad + c0 + u] = A[(c0 + s) * n + c0 + u];
    }
    if (PASS == 2) Ms[tid >> 4][tid & 15] = small[BS_R1INV + tid];
    const int rr = tid >> 2, cq = (tid & 3) * 4;
    const long row = (long)blockIdx.x * 64 + rr;
#pragma unroll
    for (int e = 0; e < 4; ++e) tile[rr][cq + e] = row < m ? A[(r0 + row) * n + c0 + cq + e] : 0.0;
    __syncthreads();
    if (PASS == 2) {
        double q[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int t = cq + e;
            double s = 0.0;
            for (int u = 0; u <= t; ++u) s += tile[rr][u] * Ms[u][t];
            q[e] = s;
        }
        __syncthreads();
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            tile[rr][cq + e] = q[e];
            if (row < m) Pq[row * 16 + cq + e] = q[e];
        }
        __syncthreads();
    }
    doublex4 acc = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        const double x = tile[16 * wave + 4 * s + lq][l16];
        acc = __builtin_amdgcn_mfma_f64_16x16x4f64(x, x, acc, 0, 0, 0);
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) red[wave][(4 * r + lq) * 16 + l16] = acc[r];
    __syncthreads();
    part[(long)blockIdx.x * 256 + tid] = (red[0][tid] + red[1][tid]) + (red[2][tid] + red[3][tid]);
    if (!last_block_done(counter, gridDim.x)) return;
    const double g = sum_block_partials(part, gridDim.x, tid);
    Ms[tid >> 4][tid & 15] = g;
    if (tid == 0) {
        *counter = 0u;
        flag_sh = 0;
    }
    __syncthreads();
    const int i = tid >> 4, j = tid & 15;
    // the serial part, by the first wave in registers: Cholesky, R^-1 and (PASS 2) the signed LU of the top block of
    // Q, T and U^-1; the small products around it by all threads through LDS
    if (wave == 0) {
        double a[16], x[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) a[r] = lane < 16 ? Ms[r][lane] : 0.0;
        const bool ok = chol16_cols(a, lane);
        if (__any(lane < 16 && !ok)) flag_sh = 1;
        triu_inverse16_cols(a, x, lane);
        if (lane < 16) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                Rs[r][lane] = a[r];
                Ri[r][lane] = x[r];
            }
        }
    }
    __syncthreads();
    if (flag_sh) {
        if (tid == 0) small[BS_FLAG] = 1.0;
        return;
    }
    if (PASS == 1) {
        small[BS_R1 + tid] = Rs[i][j];
        small[BS_R1INV + tid] = Ri[i][j];
        return;
    }
    // top block of Q = Q1 R2^-1 (the rows another block has just written are read past the caches)
    {
        double pq[16];
#pragma unroll
        for (int u = 0; u < 16; ++u) pq[u] = coherent_load(Pq + (long)i * 16 + u);
        double q = 0.0;
#pragma unroll
        for (int u = 0; u < 16; ++u)
            if (u <= j) q += pq[u] * Ri[u][j];
        Lu[i][j] = q;
    }
    __syncthreads();
    if (wave == 0) {
        double a[16], sgn[16], x[16], u[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) a[r] = lane < 16 ? Lu[r][lane] : (r == 0 ? 1.0 : 0.0);
        lu16_signed_cols(a, sgn, lane);
#pragma unroll
        for (int r = 0; r < 16; ++r) u[r] = (lane < 16 && r <= lane) ? a[r] : (lane >= 16 && r == 0 ? 1.0 : 0.0);
        if (lane < 16) {
#pragma unroll
            for (int r = 0; r < 16; ++r) Lu[r][lane] = a[r];
            sg[lane] = 0.0;
#pragma unroll
            for (int r = 0; r < 16; ++r)
                if (r == lane) sg[lane] = sgn[r];
        }
        // T = -U S Y1^-T, lane r = row r: t[c] = -U[r][c] s_c - sum_{k<c} t[k] Y1[c][k]   (Y1[c][k]: lane k, entry c)
        double t[16];
        const int rl = lane & 15;
#pragma unroll
        for (int c = 0; c < 16; ++c) {
            double sacc = c >= rl ? -Lu[rl][c] * sgn[c] : 0.0;      // (LDS written above by this wave: same wave, in order)
#pragma unroll
            for (int k = 0; k < c; ++k) sacc -= t[k] * lane_bcast(a[c], k);
            t[c] = sacc;
        }
        triu_inverse16_cols(u, x, lane);
        if (lane < 16) {
#pragma unroll
            for (int c = 0; c < 16; ++c) {
                Ts[lane][c] = t[c];
                Ms[c][lane] = x[c];                   // U^-1
            }
        }
    }
    __syncthreads();
    {
        double z = 0.0, rfull = 0.0;
        for (int k = i; k <= j; ++k) {
            z += Ri[i][k] * Ms[k][j];                               // Z = R2^-1 U^-1
            rfull += Rs[i][k] * small[BS_R1 + k * 16 + j];           // R = R2 R1
        }
        small[BS_Z + tid] = z;
        small[BS_Y1 + tid] = i > j ? Lu[i][j] : (i == j ? 1.0 : 0.0);
        small[BS_T + tid] = Ts[i][j];
        if (i <= j) bd[(long)(16 + i - j) * npad + c0 + j] = sg[i] * rfull;
    }
    if (tid < 16) tau[c0 + tid] = Ts[tid][tid];
}

// Plain Householder QR of the panel P = A[r0:, c0:c0+16] by one block (256 threads), in a row-major copy Pq [m][16]:
// the path of the last panels and of panels the Cholesky-QR route gave up on.  Leaves the same results as
// band_yt_kernel: Y in Vp[c][r0 + i] and in row c0+c of A (from its leading 1 on), tau[c0 + c], T in
// small[BS_T], and the new block below the band (R) in the band array.
__device__ void band_house_panel(double *__restrict__ A, long n, long c0, long m, double *__restrict__ Pq,
                                 double *__restrict__ small, double *__restrict__ Vp, double *__restrict__ tau,
                                 double *__restrict__ bd, long npad) {
    __shared__ double w_sh[4][16];
    __shared__ double sc_sh[4];
    __shared__ double Ts[16][17], Gv[16][17], taus[16];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const long r0 = c0 + BW;
    for (long e = tid; e < m * 16; e += 256) Pq[e] = A[(r0 + e / 16) * n + c0 + (e & 15)];
    if (tid < 16) taus[tid] = 0.0;
    __syncthreads();
    const int nr = (int)(m - 1 < 16 ? (m - 1 > 0 ? m - 1 : 0) : 16);
    for (int t = 0; t < nr; ++t) {
        double ssq = 0.0;
        for (long i = t + 1 + tid; i < m; i += 256) {
            const double x = Pq[i * 16 + t];
            ssq += x * x;
        }
        ssq = wave_sum(ssq);
        if (lane == 0) sc_sh[wave] = ssq;
        __syncthreads();
        ssq = (sc_sh[0] + sc_sh[1]) + (sc_sh[2] + sc_sh[3]);
        const double alpha = Pq[(long)t * 16 + t];
        __syncthreads();
        if (ssq == 0.0) continue;                    // nothing below the diagonal: H = I, tau = 0 (uniform branch)
        const double beta = -copysign(sqrt(alpha * alpha + ssq), alpha);
        const double tq = (beta - alpha) / beta, scale = 1.0 / (alpha - beta);
        // v = (1, P[t+1:, t] * scale); w_u = v . P[t:, u] for u > t
        double w[16];
#pragma unroll
        for (int u = 0; u < 16; ++u) w[u] = 0.0;
        for (long i = t + tid; i < m; i += 256) {
            const double v = i == t ? 1.0 : Pq[i * 16 + t] * scale;
#pragma unroll
            for (int u = 0; u < 16; ++u)
                if (u > t) w[u] += v * Pq[i * 16 + u];
        }
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            const double s = wave_sum(w[u]);
            if (lane == 0) w_sh[wave][u] = s;
        }
        __syncthreads();
        for (long i = t + tid; i < m; i += 256) {
            const double v = i == t ? 1.0 : Pq[i * 16 + t] * scale;
#pragma unroll
            for (int u = 0; u < 16; ++u)
                if (u > t) {
                    const double wu = (w_sh[0][u] + w_sh[1][u]) + (w_sh[2][u] + w_sh[3][u]);
                    Pq[i * 16 + u] -= tq * wu * v;
                }
            Pq[i * 16 + t] = i == t ? beta : v;
        }
        if (tid == 0) taus[t] = tq;
        __syncthreads();
    }
    // Gram matrix of the reflectors (unit diagonal, zeros above it), then T column by column
    for (int a = 0; a < 16; ++a)
        for (int b = a; b < 16; ++b) {
            double s = 0.0;
            for (long i = b + tid; i < m; i += 256) {
                const double va = i == a ? 1.0 : (i > a ? Pq[i * 16 + a] : 0.0);
                const double vb = i == b ? 1.0 : Pq[i * 16 + b];
                s += va * vb;
            }
            s = wave_sum(s);
            if (lane == 0) sc_sh[wave] = s;
            __syncthreads();
            if (tid == 0) Gv[a][b] = (sc_sh[0] + sc_sh[1]) + (sc_sh[2] + sc_sh[3]);
            __syncthreads();
        }
    if (tid < 16) {
        const int r = tid;
        for (int c = 0; c < 16; ++c) Ts[r][c] = 0.0;
    }
    __syncthreads();
    for (int c = 0; c < 16; ++c) {
        if (tid < 16) {
            const int r = tid;
            if (r < c) {
                double s = 0.0;
                for (int q = r; q < c; ++q) s += Ts[r][q] * Gv[q][c];
                Ts[r][c] = -taus[c] * s;
            } else if (r == c) {
                Ts[r][c] = taus[c];
            }
        }
        __syncthreads();
    }
    small[BS_T + tid] = Ts[tid >> 4][tid & 15];
    if (tid < 16 && c0 + tid < n) tau[c0 + tid] = taus[tid];
    {
        const int s = tid >> 4, u = tid & 15;          // the block below the band: R[s][u], s <= u
        if (s <= u && s < m) bd[(long)(16 + s - u) * npad + c0 + u] = Pq[(long)s * 16 + u];
    }
    for (long e = tid; e < m * 16; e += 256) {
        const long i = e / 16;
        const int c = (int)(e & 15);
        const double y = i == c ? 1.0 : (i > c && c < nr ? Pq[e] : 0.0);
        Vp[(long)c * n + r0 + i] = y;
        if (i >= c) A[(c0 + c) * n + r0 + i] = y;
    }
}

__global__ __launch_bounds__(256) void band_house_kernel(double *__restrict__ A, long n, long c0, long m,
                                                         double *__restrict__ Pq, double *__restrict__ small,
                                                         double *__restrict__ Vp, double *__restrict__ tau,
                                                         double *__restrict__ bd, long npad) {
    {
        const int s = threadIdx.x >> 4, u = threadIdx.x & 15;       // the panel's diagonal block
        if (s >= u && c0 + s < n) bd[(long)(s - u) * npad + c0 + u] = A[(c0 + s) * n + c0 + u];
    }
    band_house_panel(A, n, c0, m, Pq, small, Vp, tau, bd, npad);
}

// The reflectors of a panel from what the second Gram pass left: Y = Q1 Z below the top 16 x 16 block, Y1 in it;
// written to Vp[c][r0 + i] and to row c0+c of A (from its leading 1 on).  64 rows per block, thread = row, four
// columns.  A flagged panel (Cholesky-QR gave up) is done by the first block with plain Householder steps.
__global__ __launch_bounds__(256) void band_yt_kernel(double *__restrict__ A, long n, long c0, long m,
                                                      double *__restrict__ Pq, double *__restrict__ small,
                                                      double *__restrict__ Vp, double *__restrict__ tau,
                                                      double *__restrict__ bd, long npad) {
    __shared__ double Zs[16][17], tile[64][17];
    const int tid = threadIdx.x;
    const long r0 = c0 + BW;
    if (small[BS_FLAG] != 0.0) {
        if (blockIdx.x != 0) return;
        band_house_panel(A, n, c0, m, Pq, small, Vp, tau, bd, npad);
        __syncthreads();
        if (tid == 0) small[BS_FLAG] = 0.0;
        return;
    }
    Zs[tid >> 4][tid & 15] = small[BS_Z + tid];
    const int rr = tid >> 2, cq = (tid & 3) * 4;
    const long i = (long)blockIdx.x * 64 + rr;
#pragma unroll
    for (int e = 0; e < 4; ++e) tile[rr][cq + e] = i < m ? Pq[i * 16 + cq + e] : 0.0;
    __syncthreads();
    if (i >= m) return;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const int c = cq + e;
        double y = 0.0;
        if (i >= 16) {
            for (int u = 0; u <= c; ++u) y += tile[rr][u] * Zs[u][c];
        } else {
            y = small[BS_Y1 + (int)i * 16 + c];
        }
        Vp[(long)c * n + r0 + i] = y;
        if (i >= c) A[(c0 + c) * n + r0 + i] = y;
    }
}

// Xp[slice][i][c] = sum over the slice's k of A[r0+i][r0+k] Y[k][c]: 64 rows x 16 columns per block on the fp64
// matrix cores, one 16-row strip per wave; the slices of the contraction give the chip enough blocks.
constexpr int SYMM_KS_MAX = 16;      // slices of the full-square product
constexpr int SYMM_SLOTS_MAX = 64;   // slots of the lower-triangle product
__global__ __launch_bounds__(256) void band_symm_kernel(const double *__restrict__ A, long n, long r0, long m,
                                                        const double *__restrict__ Vp, long chunk,
                                                        double *__restrict__ Xp, int row_tiles, int ks) {
    constexpr int KC = 64;
    __shared__ double As[64][KC + 1];
    __shared__ double Vs[16][KC + 1];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l16 = lane & 15, lq = lane >> 4;
    for (long id = blockIdx.x; id < (long)row_tiles * ks; id += gridDim.x) {
        const long bx = id % row_tiles, by = id / row_tiles;
        const long i0 = bx * 64;
        const long kbeg = by * chunk, kend = min(m, kbeg + chunk);
        // a stage = 64 columns of the contraction; the next stage travels to registers while this one is multiplied
        double ra[16], rv[4];
        auto fetch = [&](long k0) {
#pragma unroll
            for (int u = 0; u < 16; ++u) {
                const int e = tid + 256 * u, r = e >> 6, q = e & 63;
                const long i = i0 + r, k = k0 + q;
                ra[u] = (i < m && k < kend) ? A[(r0 + i) * n + r0 + k] : 0.0;
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int e = tid + 256 * u, c = e >> 6, q = e & 63;
                const long k = k0 + q;
                rv[u] = k < kend ? Vp[(long)c * n + r0 + k] : 0.0;
            }
        };
        doublex4 acc = {0.0, 0.0, 0.0, 0.0};
        if (kbeg < kend) fetch(kbeg);
        for (long k0 = kbeg; k0 < kend; k0 += KC) {
            __syncthreads();                       // the stage before has been read
#pragma unroll
            for (int u = 0; u < 16; ++u) {
                const int e = tid + 256 * u;
                As[e >> 6][e & 63] = ra[u];
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int e = tid + 256 * u;
                Vs[e >> 6][e & 63] = rv[u];
            }
            __syncthreads();
            if (k0 + KC < kend) fetch(k0 + KC);
#pragma unroll
            for (int q = 0; q < KC; q += 4)
                acc = __builtin_amdgcn_mfma_f64_16x16x4f64(As[wave * 16 + l16][q + lq], Vs[l16][q + lq], acc, 0, 0, 0);
        }
        double *out = Xp + by * m * 16;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const long i = i0 + wave * 16 + 4 * r + lq;
            if (i < m) out[i * 16 + l16] = acc[r];
        }
    }
}

// The same product from the lower triangle alone, for trailing matrices too large for the caches (the pass is then
// bound by reading them): only entries A[i][j] with i >= j are read, and only those are kept up to date by the
// rank-32 update in this mode.  A block owns a square of TS x TS tiles of 64 x 64 on or below the diagonal, (P, Q)
// in units of that square; tile (ti, tj) below the diagonal adds A_t Y_cols to the rows of ti and A_t^T Y_rows to the
// rows of tj, a diagonal tile is made symmetric in LDS and used once.  The square's two results go to slots of
// their own, Xp[Q][rows of P] and Xp[P][rows of Q] (one slot when P == Q), so that every block of rows receives
// exactly one piece per slot 0 .. S-1 and band_k_kernel adds them in slot order: no atomics, a fixed order.
template <int TS>
__global__ __launch_bounds__(256) void band_symm_lower_kernel(const double *__restrict__ A, long n, long r0, long m,
                                                              const double *__restrict__ Vp, double *__restrict__ Xp) {
    __shared__ double As[64][65];
    __shared__ double Vc[16][65], Vr[16][65];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l16 = lane & 15, lq = lane >> 4;
    int P, Q;
    tri_tile_of((int)blockIdx.x, P, Q);
    const long ntile = (m + 63) / 64;
    doublex4 acc_n[TS], acc_t[TS];
#pragma unroll
    for (int t = 0; t < TS; ++t) {
        acc_n[t] = doublex4{0.0, 0.0, 0.0, 0.0};
        acc_t[t] = doublex4{0.0, 0.0, 0.0, 0.0};
    }
    double ra[16], rc[4], rr[4];
    auto valid = [&](int ti, int tj) {
        const long gi = (long)P * TS + ti, gj = (long)Q * TS + tj;
        return gi < ntile && gj <= gi;
    };
    auto fetch = [&](int ti, int tj) {
        const long i0 = ((long)P * TS + ti) * 64, j0 = ((long)Q * TS + tj) * 64;
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            const int e = tid + 256 * u, r = e >> 6, q = e & 63;
            const long i = i0 + r, j = j0 + q;
            ra[u] = (i < m && j <= i) ? A[(r0 + i) * n + r0 + j] : 0.0;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int e = tid + 256 * u, c = e >> 6, q = e & 63;
            rc[u] = j0 + q < m ? Vp[(long)c * n + r0 + j0 + q] : 0.0;
            rr[u] = i0 + q < m ? Vp[(long)c * n + r0 + i0 + q] : 0.0;
        }
    };
    // the valid tiles of the square in row-major order; the next one travels to registers while this one is multiplied
    int ti = 0, tj = 0;
    auto advance = [&](int &a, int &b) {          // next valid tile after (a, b), or a = TS
        do {
            if (++b == TS) {
                b = 0;
                ++a;
            }
        } while (a < TS && !valid(a, b));
    };
    if (!valid(0, 0)) advance(ti, tj);
    if (ti < TS) fetch(ti, tj);
    while (ti < TS) {
        __syncthreads();                       // the tile before has been read
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            const int e = tid + 256 * u;
            As[e >> 6][e & 63] = ra[u];
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int e = tid + 256 * u;
            Vc[e >> 6][e & 63] = rc[u];
            Vr[e >> 6][e & 63] = rr[u];
        }
        const bool diag = (long)P * TS + ti == (long)Q * TS + tj;
        __syncthreads();
        if (diag) {
            // the stored upper half of a diagonal tile may be stale: mirror the lower half
#pragma unroll
            for (int u = 0; u < 16; ++u) {
                const int e = tid + 256 * u, r = e >> 6, q = e & 63;
                if (q > r) As[r][q] = As[q][r];
            }
            __syncthreads();
        }
        const int ci = ti, cj = tj;
        advance(ti, tj);
        if (ti < TS) fetch(ti, tj);
#pragma unroll
        for (int t = 0; t < TS; ++t) {
            if (t == ci) {
#pragma unroll
                for (int q = 0; q < 64; q += 4)
                    acc_n[t] = __builtin_amdgcn_mfma_f64_16x16x4f64(As[wave * 16 + l16][q + lq], Vc[l16][q + lq], acc_n[t], 0, 0, 0);
            }
            if (t == cj && !diag) {
#pragma unroll
                for (int q = 0; q < 64; q += 4)
                    acc_t[t] = __builtin_amdgcn_mfma_f64_16x16x4f64(As[q + lq][wave * 16 + l16], Vr[l16][q + lq], acc_t[t], 0, 0, 0);
            }
        }
    }
    // results: rows of P into slot Q, rows of Q into slot P (summed into one piece when P == Q)
#pragma unroll
    for (int t = 0; t < TS; ++t) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const long in_n = ((long)P * TS + t) * 64 + wave * 16 + 4 * r + lq;
            const long in_t = ((long)Q * TS + t) * 64 + wave * 16 + 4 * r + lq;
            if (P == Q) {
                if (in_n < m) Xp[((long)Q * m + in_n) * 16 + l16] = acc_n[t][r] + acc_t[t][r];
            } else {
                if (in_n < m) Xp[((long)Q * m + in_n) * 16 + l16] = acc_n[t][r];
                if (in_t < m) Xp[((long)P * m + in_t) * 16 + l16] = acc_t[t][r];
            }
        }
    }
}

// X = sum of the slices (written to Xa [m][16]); K = Y^T X as per-block partials (64 rows per block); the last
// block adds them in block order and leaves S = T^T K T in small[BS_S2].
__global__ __launch_bounds__(256) void band_k_kernel(const double *__restrict__ Xp, int ks, long m, long n, long r0,
                                                     const double *__restrict__ Vp, double *__restrict__ Xa,
                                                     double *__restrict__ small, double *__restrict__ part,
                                                     unsigned *__restrict__ counter) {
    __shared__ double xt[64][17], vt[64][17];
    __shared__ double red[4][256];
    __shared__ double Ks[16][17], Ts[16][17], KT[16][17];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l16 = lane & 15, lq = lane >> 4;
    const int rr = tid >> 2, cq = (tid & 3) * 4;
    const long i = (long)blockIdx.x * 64 + rr;
    {
        double x[4] = {0.0, 0.0, 0.0, 0.0};
        if (i < m)
#pragma unroll 4
            for (int s = 0; s < ks; ++s) {
#pragma unroll
                for (int e = 0; e < 4; ++e) x[e] += Xp[((long)s * m + i) * 16 + cq + e];
            }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            xt[rr][cq + e] = x[e];
            if (i < m) Xa[i * 16 + cq + e] = x[e];
        }
        // Y[row][c] of the block's rows: thread = (column c = tid / 16, four rows)
        const int c = tid >> 4, r4 = (tid & 15) * 4;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const long ii = (long)blockIdx.x * 64 + r4 + e;
            vt[r4 + e][c] = ii < m ? Vp[(long)c * n + r0 + ii] : 0.0;
        }
    }
    __syncthreads();
    doublex4 acc = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        const int r = 16 * wave + 4 * s + lq;
        acc = __builtin_amdgcn_mfma_f64_16x16x4f64(vt[r][l16], xt[r][l16], acc, 0, 0, 0);      // K[a][b] += Y[r][a] X[r][b]
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) red[wave][(4 * r + lq) * 16 + l16] = acc[r];
    __syncthreads();
    part[(long)blockIdx.x * 256 + tid] = (red[0][tid] + red[1][tid]) + (red[2][tid] + red[3][tid]);
    if (!last_block_done(counter, gridDim.x)) return;
    const double g = sum_block_partials(part, gridDim.x, tid);
    const int a = tid >> 4, b = tid & 15;
    Ks[a][b] = g;
    Ts[a][b] = small[BS_T + tid];
    if (tid == 0) *counter = 0u;
    __syncthreads();
    double s = 0.0;
    for (int k = 0; k < 16; ++k) s += Ks[a][k] * Ts[k][b];
    KT[a][b] = s;
    __syncthreads();
    s = 0.0;
    for (int k = 0; k < 16; ++k) s += Ts[k][a] * KT[k][b];
    small[BS_S2 + tid] = s;
}

// W = X T - 1/2 Y S; written as Wp[c][r0 + i].  64 rows per block: thread = (column c, four rows).
__global__ __launch_bounds__(256) void band_w_kernel(const double *__restrict__ Xa, long m, long n, long r0,
                                                     const double *__restrict__ Vp, const double *__restrict__ small,
                                                     double *__restrict__ Wp) {
    __shared__ double Ts[16][17], Ss[16][17], xt[64][17], yt[64][17];
    const int tid = threadIdx.x;
    Ts[tid >> 4][tid & 15] = small[BS_T + tid];
    Ss[tid >> 4][tid & 15] = small[BS_S2 + tid];
    const long i0 = (long)blockIdx.x * 64;
    {
        const int rr = tid >> 2, cq = (tid & 3) * 4;
#pragma unroll
        for (int e = 0; e < 4; ++e) xt[rr][cq + e] = i0 + rr < m ? Xa[(i0 + rr) * 16 + cq + e] : 0.0;
    }
    const int c = tid >> 4, r4 = (tid & 15) * 4;
#pragma unroll
    for (int e = 0; e < 4; ++e) yt[r4 + e][c] = i0 + r4 + e < m ? Vp[(long)c * n + r0 + i0 + r4 + e] : 0.0;
    __syncthreads();
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const int r = r4 + e;
        if (i0 + r >= m) break;
        double s = 0.0, h = 0.0;
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            if (k <= c) s += xt[r][k] * Ts[k][c];         // T is upper triangular
            h += yt[r][k] * Ss[k][c];
        }
        Wp[(long)c * n + r0 + i0 + r] = s - 0.5 * h;
    }
}

// band array: zero, with a unit diagonal on the padded columns; then the last diagonal block
__global__ void band_init_kernel(double *__restrict__ bd, long n, long npad) {
    const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (BW + 1) * npad) return;
    const long t = idx / npad, j = idx - t * npad;
    bd[idx] = (t == 0 && j >= n) ? 1.0 : 0.0;
}
__global__ void band_tail_kernel(const double *__restrict__ A, long n, long c_end, double *__restrict__ bd,
                                 long npad) {
    for (int e = threadIdx.x; e < 32 * 32; e += blockDim.x) {
        const long s = e >> 5, u = e & 31;
        if (s >= u && s - u <= BW && c_end + s < n) bd[(s - u) * npad + c_end + u] = A[(c_end + s) * n + c_end + u];
    }
}

// One block of up to NBT reflectors applied to the accumulated matrix M (compact WY): M <- M (I - V T' V^T) on rows
// jstart .. n-1 and columns k0+off .. n-1; T' = T^T when R = Q^T is built from the last block to the first,
// T' = T when Q is built from the first block on.  cap > 0 bounds the blocks per launch of the two products.
// S, T: NBT x NBT doubles; Gp: WY_KS_MAX x N x NBT; G2: N x NBT.
template <int NBT>
static void wy_apply_block(hipStream_t s2, const double *A64, double *R64, long N, const double *tau, double *S,
                           double *T, double *Gp, double *G2, long k0, int nbc, long jstart, int forward, long cap,
                           int off) {
    hipLaunchKernelGGL(q_gram_kernel<NBT>, dim3(nbc, nbc), dim3(256), 0, s2, A64, N, k0, nbc, S, off);
    hipLaunchKernelGGL(q_tfactor_kernel<NBT>, dim3(1), dim3(NBT), 0, s2, S, tau, k0, nbc, T);
    const long m = N - k0 - off;               // length of the contraction
    const long rows = N - jstart;
    if (m < 1 || rows < 1) return;
    const unsigned row_tiles = blocks_for(rows, 64), col_tiles = blocks_for(m, 64);
    long ks = (2048 + (long)row_tiles - 1) / (long)row_tiles;      // eight blocks per compute unit or more
    if (ks > WY_KS_MAX) ks = WY_KS_MAX;
    if (ks > m / 256) ks = m / 256;
    if (ks < 1) ks = 1;
    long chunk = (m + ks - 1) / ks;
    chunk = (chunk + 31) / 32 * 32;
    const long g_blocks = (long)row_tiles * ks, u_blocks = (long)col_tiles * row_tiles;
    hipLaunchKernelGGL(q_wy_g_kernel<NBT>, dim3((unsigned)(cap > 0 && g_blocks > cap ? cap : g_blocks)), dim3(256), 0, s2,
                       R64, A64, N, k0, nbc, chunk, Gp, jstart, (int)row_tiles, (int)ks, off);
    hipLaunchKernelGGL(q_wy_g2_kernel<NBT>, dim3(blocks_for(rows, 256 / NBT)), dim3(256), 0, s2, Gp, T, N, k0, nbc, (int)ks,
                       G2, jstart, forward);
    hipLaunchKernelGGL(q_wy_update_kernel<NBT>, dim3((unsigned)(cap > 0 && u_blocks > cap ? cap : u_blocks)), dim3(256), 0,
                       s2, R64, A64, N, k0, nbc, G2, jstart, (int)col_tiles, (int)row_tiles, off);
}

}  // namespace

size_t admmq_householder_scratch_doubles(int64_t n) {
    const size_t N = (size_t)n;
    const size_t nt = N / ST + 2;                 // slots of the lower-triangle product: nt x nt pieces of ST
    return (3 + 2 * NB + WY_KS_MAX * NB + NB) * N + 2 * NB * NB + SC_COUNT + (N / ROW_CHUNK + 2) * PART_W + (N / 4 + 2) + 64 +
           nt * nt * ST;
}

// trailing size from which a panel runs in the lower-triangle mode (the matrix no longer fits the caches);
// ADMMQ_SYMV_MIN overrides it (read at every factorisation; values below 128 switch the mode off)
static long symv_min_size() {
    const char *e = getenv("ADMMQ_SYMV_MIN");
    long v = e ? atol(e) : 5120;
    return v < 128 ? (1L << 60) : v;
}

// A64: [n][n] scaled Hessian (destroyed: reflectors end up in its rows); R64: [n][n] scratch;
// vecs: admmq_householder_scratch_doubles(n) doubles.  Outputs: Q, Qt (fp32), ta, tb (fp64).
admmq_status admmq_k_householder(admmq_ctx *ctx, double *A64, int64_t n, double *R64, double *vecs, float *Q,
                                 float *Qt, double *ta, double *tb) {
    hipStream_t st = ctx->stream;
    const long N = (long)n;
    double *pbuf = vecs, *xbuf = vecs + N, *tau = vecs + 2 * N, *Vp = vecs + 3 * N, *Wp = Vp + (long)NB * N,
           *Gp = Wp + (long)NB * N, *S = Gp + (long)WY_KS_MAX * NB * N, *T = S + NB * NB, *sc = T + NB * NB,
           *part1 = sc + SC_COUNT, *part2 = part1 + (N / ROW_CHUNK + 2) * PART_W, *cnt = part2 + (N / 4 + 2),
           *G2 = cnt + 64, *Pb = G2 + (long)NB * N;
    unsigned *counters = (unsigned *)cnt;          // [0]: tri_row, [2]: tri_mat (8-byte slots)
    const long sym_min = symv_min_size();
    // One block of NB reflectors applied to the accumulated matrix M (compact WY): M <- M (I - V T' V^T) on rows
    // jstart .. n-1 and columns k0+1 .. n-1; T' = T^T when R = Q^T is built from the last block to the first,
    // T' = T when Q is built from the first block on.
    auto apply_block = [&](hipStream_t s2, long k0, int nbc, long jstart, int forward, long cap) {
        wy_apply_block<NB>(s2, A64, R64, N, tau, S, T, Gp, G2, k0, nbc, jstart, forward, cap, 1);
    };
    // While the trailing matrix fits the caches the panel chain above is bound by launch and memory latency and
    // leaves the chip mostly idle: Q = H_0 H_1 ... is then accumulated from the first block on (2 n^3 flop instead of
    // the (4/3) n^3 of the backward order), each block as soon as its panel is finished, on a stream of its own.
    // ADMMQ_Q_OVERLAP=0 keeps the backward order on the main stream.
    bool overlap = N >= 3 && N < sym_min;
    {
        const char *e = getenv("ADMMQ_Q_OVERLAP");
        if (e && atoi(e) == 0) overlap = false;
    }
    // blocks per side-stream launch of the two products: few enough to leave the panel chain its compute units
    long side_cap = 96;
    {
        const char *e = getenv("ADMMQ_Q_SIDE_BLOCKS");
        if (e && atol(e) > 0) side_cap = atol(e);
    }
    const long nblk_all = N >= 3 ? (N - 2 + NB - 1) / NB : 0;
    hipStream_t side = nullptr;
    if (overlap) {
        if (!ctx->side[0] && hipStreamCreateWithFlags(&ctx->side[0], hipStreamNonBlocking) != hipSuccess) overlap = false;
        side = ctx->side[0];
    }
    if (overlap && ctx->panel_event_count < nblk_all + 2) {
        const int want = (int)nblk_all + 2;
        hipEvent_t *grown = (hipEvent_t *)realloc(ctx->panel_events, (size_t)want * sizeof(hipEvent_t));
        if (!grown) overlap = false;
        else {
            ctx->panel_events = grown;
            while (ctx->panel_event_count < want) {
                if (hipEventCreateWithFlags(&ctx->panel_events[ctx->panel_event_count], hipEventDisableTiming) != hipSuccess) {
                    overlap = false;
                    break;
                }
                ++ctx->panel_event_count;
            }
        }
    }
    if (overlap) {
        // the side stream starts behind everything queued so far (R64 and the scratch may still be in use)
        ADMMQ_HIP(hipEventRecord(ctx->panel_events[nblk_all], st));
        ADMMQ_HIP(hipStreamWaitEvent(side, ctx->panel_events[nblk_all], 0));
        hipLaunchKernelGGL(identity_kernel, dim3(blocks_for(N * N, 256)), dim3(256), 0, side, R64, N);
    }
    bool was_sym = false;
    int parts_prev = 0;                            // block partials of p'.v left by the previous column's product
    ADMMQ_TRY(admmq_k_fill_bytes(ctx, cnt, 0, 32));
    ADMMQ_TRY(admmq_k_fill_bytes(ctx, sc, 0, SC_COUNT * 8));
    if (N <= 2) {
        hipLaunchKernelGGL(tri_tiny_kernel, dim3(1), dim3(64), 0, st, A64, N, ta, tb);
    } else {
        for (long k0 = 0; k0 <= N - 3; k0 += NB) {
            const int nbc = (int)((N - 2 - k0) < NB ? (N - 2 - k0) : NB);
            const bool sym = N - k0 >= sym_min;
            if (was_sym && !sym) {
                // leaving the lower-triangle mode: the upper triangle of the trailing block is stale
                const long t32 = (N - k0 + 31) / 32;
                hipLaunchKernelGGL(tri_mirror_kernel, dim3((unsigned)(t32 * (t32 + 1) / 2)), dim3(32, 8), 0, st, A64,
                                   N, k0);
            }
            was_sym = sym;
            for (int c = 0; c < nbc; ++c) {
                const long k = k0 + c;
                const unsigned row_blocks = blocks_for(N - k, ROW_CHUNK);
                hipLaunchKernelGGL(tri_row_kernel, dim3(row_blocks), dim3(256), 0, st, A64, N, k, c, c > 0 ? 1 : 0, 1,
                                   Vp, Wp, pbuf, xbuf, tau, ta, tb, sc, part1, counters, part2, parts_prev,
                                   sym ? 1 : 0, sym ? 1 : 0);
                if (sym) {
                    const int t0 = (int)((k + 1) / ST);
                    const int nt = (int)((N - 1) / ST) - t0 + 1;
                    hipLaunchKernelGGL(tri_symv_tile_kernel, dim3((unsigned)((long)nt * (nt + 1) / 2)), dim3(256), 0,
                                       st, A64, N, k, xbuf, sc, Pb, t0, nt);
                    parts_prev = nt;
                    hipLaunchKernelGGL(tri_symv_finish_kernel, dim3((unsigned)parts_prev), dim3(256), 0, st, A64, N, k,
                                       c, Vp, Wp, xbuf, pbuf, sc, Pb, t0, nt, part2);
                } else {
                    parts_prev = (int)blocks_for(N - k - 1, 4);
                    hipLaunchKernelGGL(tri_mat_kernel, dim3((unsigned)parts_prev), dim3(256), 0, st, A64, N, k, c, Vp,
                                       Wp, xbuf, pbuf, sc, part2, part1, (int)row_blocks, tau, ta, tb);
                }
            }
            // close the panel's last column, then apply the panel to the trailing matrix
            const long r0 = k0 + nbc;
            hipLaunchKernelGGL(tri_row_kernel, dim3(blocks_for(N - r0, ROW_CHUNK)), dim3(256), 0, st, A64, N, r0, nbc,
                               1, 0, Vp, Wp, pbuf, xbuf, tau, ta, tb, sc, part1, counters, part2, parts_prev,
                               sym ? 1 : 0, 1);
            if (overlap) {
                // the panel's reflectors (rows k0 .. r0-1 of A) and taus are final: its block joins Q
                const long b = k0 / NB;
                ADMMQ_HIP(hipEventRecord(ctx->panel_events[b], st));
                ADMMQ_HIP(hipStreamWaitEvent(side, ctx->panel_events[b], 0));
                apply_block(side, k0, nbc, 1, 1, side_cap);
            }
            const unsigned tiles = blocks_for(N - r0, 64);
            hipLaunchKernelGGL(tri_update_kernel, dim3(tiles, tiles), dim3(256), 0, st, A64, N, r0, nbc, Vp, Wp,
                               sym ? 1 : 0);
        }
        if (was_sym) {
            // (only when the override keeps the mode on to the end) the closing 2 x 2 block is read as stored
            hipLaunchKernelGGL(tri_mirror_kernel, dim3(1), dim3(32, 8), 0, st, A64, N, N - 2);
        }
        hipLaunchKernelGGL(tri_tail_kernel, dim3(1), dim3(64), 0, st, A64, N, ta, tb);
    }
    ADMMQ_HIP(hipGetLastError());
    dim3 tb32(32, 8), tg((unsigned)((N + 31) / 32), (unsigned)((N + 31) / 32));
    if (overlap) {
        // R64 holds Q: the main stream waits for the last block, then writes Q as stored and Q^T transposed
        ADMMQ_HIP(hipEventRecord(ctx->panel_events[nblk_all + 1], side));
        ADMMQ_HIP(hipStreamWaitEvent(st, ctx->panel_events[nblk_all + 1], 0));
        hipLaunchKernelGGL(emit_q_kernel, tg, tb32, 0, st, R64, N, Qt, Q);
    } else {
        hipLaunchKernelGGL(identity_kernel, dim3(blocks_for(N * N, 256)), dim3(256), 0, st, R64, N);
        if (N >= 3) {
            const long nref = N - 2;
            const long nblk = (nref + NB - 1) / NB;
            for (long b = nblk - 1; b >= 0; --b) {
                const long k0 = b * NB;
                const int nbc = (int)((nref - k0) < NB ? (nref - k0) : NB);
                apply_block(st, k0, nbc, k0 + 1, 0, 0);
            }
        }
        hipLaunchKernelGGL(emit_q_kernel, tg, tb32, 0, st, R64, N, Q, Qt);
    }
    ADMMQ_HIP(hipGetLastError());
    return ADMMQ_OK;
}

size_t admmq_band_scratch_doubles(int64_t n) {
    const size_t N = (size_t)n;
    return (1 + 2 * BW + SYMM_SLOTS_MAX * BW + 2 * BW + WY_KS_MAX * QB + QB) * N + 2 * (N / 64 + 2) * 256 + 2 * QB * QB + 4096;
}

// Hs = Q Bd Q^T with Bd symmetric of half-bandwidth 16.  A64: [n][n] scaled Hessian (destroyed: reflectors end up in its
// rows); R64: [n][n] scratch; vecs: admmq_band_scratch_doubles(n) doubles.  Outputs: Q, Qt (fp32 [n][n]) and the
// band bd[t][j] = Bd[j + t][j], t = 0 .. 16, j < npad = n rounded up to a multiple of 16 (unit diagonal beyond n).
admmq_status admmq_k_band_reduce(admmq_ctx *ctx, double *A64, int64_t n, double *R64, double *vecs, float *Q, float *Qt,
                                 double *bd) {
    hipStream_t st = ctx->stream;
    const long N = (long)n, npad = (N + BW - 1) / BW * BW;
    double *tau = vecs, *Vp = tau + N, *Wp = Vp + (long)BW * N, *Xp = Wp + (long)BW * N,
           *Xa = Xp + (long)SYMM_SLOTS_MAX * BW * N, *Pq = Xa + (long)BW * N, *Gp = Pq + (long)BW * N,
           *G2 = Gp + (long)WY_KS_MAX * QB * N, *part1 = G2 + (long)QB * N, *part2 = part1 + (N / 64 + 2) * 256,
           *S = part2 + (N / 64 + 2) * 256, *T = S + QB * QB, *small = T + QB * QB;
    unsigned *counters = (unsigned *)(small + BS_COUNT);      // [0]: Gram kernels, [2]: K kernel
    ADMMQ_TRY(admmq_k_fill_bytes(ctx, small, 0, 2048 * 8));
    ADMMQ_TRY(admmq_k_fill_bytes(ctx, tau, 0, (size_t)N * 8));
    hipLaunchKernelGGL(band_init_kernel, dim3(blocks_for((BW + 1) * npad, 256)), dim3(256), 0, st, bd, N, npad);
    const long nref = N > BW + 1 ? N - BW - 1 : 0;            // reflector g has its leading 1 at index g + 16 <= n - 2
    const long nblk_all = (nref + QB - 1) / QB;
    // The accumulation of Q: as in the tridiagonal reduction, from the first block on and on a stream of its own
    // while the matrix fits the caches (the panel chain is a string of short launches), else from the last block back
    // on the main stream afterwards.
    bool overlap = nref > 0 && N < symv_min_size();
    {
        const char *e = getenv("ADMMQ_Q_OVERLAP");
        if (e && atoi(e) == 0) overlap = false;
    }
    long side_cap = 0;
    {
        const char *e = getenv("ADMMQ_Q_SIDE_BLOCKS");
        if (e && atol(e) > 0) side_cap = atol(e);
    }
    hipStream_t side = nullptr;
    if (overlap) {
        if (!ctx->side[0] && hipStreamCreateWithFlags(&ctx->side[0], hipStreamNonBlocking) != hipSuccess) overlap = false;
        side = ctx->side[0];
    }
    if (overlap && ctx->panel_event_count < nblk_all + 2) {
        const int want = (int)nblk_all + 2;
        hipEvent_t *grown = (hipEvent_t *)realloc(ctx->panel_events, (size_t)want * sizeof(hipEvent_t));
        if (!grown) overlap = false;
        else {
            ctx->panel_events = grown;
            while (ctx->panel_event_count < want) {
                if (hipEventCreateWithFlags(&ctx->panel_events[ctx->panel_event_count], hipEventDisableTiming) != hipSuccess) {
                    overlap = false;
                    break;
                }
                ++ctx->panel_event_count;
            }
        }
    }
    if (overlap) {
        ADMMQ_HIP(hipEventRecord(ctx->panel_events[nblk_all], st));
        ADMMQ_HIP(hipStreamWaitEvent(side, ctx->panel_events[nblk_all], 0));
        hipLaunchKernelGGL(identity_kernel, dim3(blocks_for(N * N, 256)), dim3(256), 0, side, R64, N);
    }
    // trailing size from which the passes over the trailing matrix use its lower triangle only (ADMMQ_BAND_LOWER_MIN;
    // with 64 slots of 256 rows the mode ends at 16384, where squares of 512 rows begin)
    long lower_min = 6144;
    {
        const char *e = getenv("ADMMQ_BAND_LOWER_MIN");
        if (e) lower_min = atol(e) < 128 ? (1L << 60) : atol(e);
    }
    bool was_lower = false;
    for (long c0 = 0; c0 < nref; c0 += BW) {
        const long r0 = c0 + BW, m = N - r0;                  // m >= 2
        const unsigned rb = blocks_for(m, 64);
        if (m >= 64) {
            hipLaunchKernelGGL(band_gram_kernel<1>, dim3(rb), dim3(256), 0, st, A64, N, c0, m, Pq, small, part1, counters,
                               bd, npad, tau);
            hipLaunchKernelGGL(band_gram_kernel<2>, dim3(rb), dim3(256), 0, st, A64, N, c0, m, Pq, small, part1, counters,
                               bd, npad, tau);
            hipLaunchKernelGGL(band_yt_kernel, dim3(rb), dim3(256), 0, st, A64, N, c0, m, Pq, small, Vp, tau, bd, npad);
        } else {
            hipLaunchKernelGGL(band_house_kernel, dim3(1), dim3(256), 0, st, A64, N, c0, m, Pq, small, Vp, tau, bd, npad);
        }
        // While the trailing matrix is larger than the caches the two passes over it read and update its lower
        // triangle only; below that size the upper triangle is restored once and the full-square kernels take over.
        const int ts = m >= 16384 ? 8 : 4;                     // tiles per side of a block's square
        const long S2 = (m + 64 * ts - 1) / (64 * ts);
        const bool lower = m >= lower_min && S2 <= SYMM_SLOTS_MAX;
        if (was_lower && !lower) {
            const long t32 = (m + 31) / 32;
            hipLaunchKernelGGL(tri_mirror_kernel, dim3((unsigned)(t32 * (t32 + 1) / 2)), dim3(32, 8), 0, st, A64, N, r0);
        }
        was_lower = lower;
        long ks;
        if (lower) {
            ks = S2;
            if (ts == 8)
                hipLaunchKernelGGL(band_symm_lower_kernel<8>, dim3((unsigned)(S2 * (S2 + 1) / 2)), dim3(256), 0, st, A64, N, r0,
                                   m, Vp, Xp);
            else
                hipLaunchKernelGGL(band_symm_lower_kernel<4>, dim3((unsigned)(S2 * (S2 + 1) / 2)), dim3(256), 0, st, A64, N, r0,
                                   m, Vp, Xp);
        } else {
            const long row_tiles = (m + 63) / 64;
            ks = (1024 + row_tiles - 1) / row_tiles;
            if (ks > SYMM_KS_MAX) ks = SYMM_KS_MAX;
            if (ks > m / 256) ks = m / 256;
            if (ks < 1) ks = 1;
            long chunk = (m + ks - 1) / ks;
            chunk = (chunk + 63) / 64 * 64;
            hipLaunchKernelGGL(band_symm_kernel, dim3((unsigned)(row_tiles * ks)), dim3(256), 0, st, A64, N, r0, m, Vp, chunk,
                               Xp, (int)row_tiles, (int)ks);
        }
        hipLaunchKernelGGL(band_k_kernel, dim3(rb), dim3(256), 0, st, Xp, (int)ks, m, N, r0, Vp, Xa, small, part2,
                           counters + 2);
        hipLaunchKernelGGL(band_w_kernel, dim3(rb), dim3(256), 0, st, Xa, m, N, r0, Vp, small, Wp);
        const unsigned tiles = blocks_for(m, 64);
        hipLaunchKernelGGL(tri_update_kernel, dim3(tiles, tiles), dim3(256), 0, st, A64, N, r0, BW, Vp, Wp, lower ? 1 : 0);
        const long done = c0 + BW < nref ? c0 + BW : nref;     // reflectors finished so far
        if (overlap && (done % QB == 0 || done == nref)) {
            const long b = (done - 1) / QB, k0 = b * QB;
            ADMMQ_HIP(hipEventRecord(ctx->panel_events[b], st));
            ADMMQ_HIP(hipStreamWaitEvent(side, ctx->panel_events[b], 0));
            wy_apply_block<QB>(side, A64, R64, N, tau, S, T, Gp, G2, k0, (int)(done - k0), BW, 1, side_cap, BW);
        }
    }
    {
        const long c_end = (nref + BW - 1) / BW * BW;
        hipLaunchKernelGGL(band_tail_kernel, dim3(1), dim3(256), 0, st, A64, N, c_end, bd, npad);
    }
    ADMMQ_HIP(hipGetLastError());
    dim3 tb32(32, 8), tg((unsigned)((N + 31) / 32), (unsigned)((N + 31) / 32));
    if (overlap) {
        ADMMQ_HIP(hipEventRecord(ctx->panel_events[nblk_all + 1], side));
        ADMMQ_HIP(hipStreamWaitEvent(st, ctx->panel_events[nblk_all + 1], 0));
        hipLaunchKernelGGL(emit_q_kernel, tg, tb32, 0, st, R64, N, Qt, Q);
    } else {
        hipLaunchKernelGGL(identity_kernel, dim3(blocks_for(N * N, 256)), dim3(256), 0, st, R64, N);
        for (long b = nblk_all - 1; b >= 0; --b) {
            const long k0 = b * QB;
            const int nbc = (int)((nref - k0) < QB ? (nref - k0) : QB);
            wy_apply_block<QB>(st, A64, R64, N, tau, S, T, Gp, G2, k0, nbc, k0 + BW, 0, 0, BW);
        }
        hipLaunchKernelGGL(emit_q_kernel, tg, tb32, 0, st, R64, N, Q, Qt);
    }
    ADMMQ_HIP(hipGetLastError());
    return ADMMQ_OK;
}
