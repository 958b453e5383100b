// Pair-swap local search kernels (Sec. 3.5, eq. 11), in the unscaled space on H' = H + lambda I.
//
// Per batch of candidate row pairs:
//   evaluate : one block per (pair, column chunk); every column takes the best feasible sign
//              combination of (+-delta_i1, +-delta_i2) by eq. 11 if it lowers the loss; the chunk's
//              summed gain goes to partial[pair][chunk]
//   plan     : every block sums the chunks in a fixed order and picks the largest total (lowest slot
//              on ties) - the same winner in every block - then writes, for its own columns, the new
//              codes and the applied steps of the winner into slot (batch mod K) of a pending list
//   flush    : every K batches G is streamed ONCE for all pending pairs:
//              G[i][j] -= sum_k H'[i][a_k] d1_k[j] + H'[i][b_k] d2_k[j]          (rank-2K correction)
// Between flushes the two gradient rows a candidate pair needs are corrected on the fly from the
// pending list, so every evaluation sees the gradient of the current codes (Sec. 3.5 step (v)) while
// the n x p array is read and written once per K applied pairs instead of once per pair.
#include "common.h"

typedef float floatx4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int LS_CHUNK = 256;    // columns per evaluate block (one per thread)

struct PairEval {
    float gain;   // -dL of the chosen combination, 0 if none improves
    int combo;    // 0..3 in the order (+,+),(+,-),(-,+),(-,-), or -1
};

// eq. 11 for one column.  a = delta of row i1's group, b = delta of row i2's group.
__device__ inline PairEval eval_column(float g1, float g2, int k1, int k2, float a, float b, float h11, float h22,
                                       float h12, int levels) {
    PairEval r;
    r.gain = 0.f;
    r.combo = -1;
    if (a == 0.f || b == 0.f) return r;        // a degenerate group cannot move
    float best = 0.f;
    const float qa = a * a * h11, qb = b * b * h22, cross = 2.f * a * b * h12;
    const float la = 2.f * a * g1, lb = 2.f * b * g2;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        const int s1 = (c & 2) ? -1 : 1, s2 = (c & 1) ? -1 : 1;
        const int n1 = k1 + s1, n2 = k2 + s2;
        if (n1 < 0 || n1 > levels || n2 < 0 || n2 > levels) continue;
        // dL = -2 d1 G1 + d1^2 H11 - 2 d2 G2 + d2^2 H22 + 2 d1 d2 H12,  d1 = s1 a, d2 = s2 b
        const float dL = -(float)s1 * la + qa - (float)s2 * lb + qb + (float)(s1 * s2) * cross;
        if (dL < best) {
            best = dL;
            r.combo = c;
        }
    }
    r.gain = -best;
    return r;
}

__device__ inline float wave_sum_f(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o, 64);
    return v;
}

constexpr int LS_K = 16;          // pending pairs between two passes over G

// coefficients of the pending corrections for gradient rows i1 and i2:
//   coef[k][0..3] = H'[i1][a_k], H'[i1][b_k], H'[i2][a_k], H'[i2][b_k]   (0 for an empty slot)
__device__ inline void load_pending_coef(const float *__restrict__ H, float lambda, long n, long i1, long i2,
                                         const int32_t *__restrict__ pend_idx, int npend, float (*coef)[4]) {
    for (int e = threadIdx.x; e < npend * 4; e += blockDim.x) {
        const int k = e >> 2, w = e & 3;
        const long row = (w & 2) ? i2 : i1;
        const long col = pend_idx[2 * k + (w & 1)];
        float h = 0.f;
        if (pend_idx[2 * k] >= 0) {
            h = H[row * n + col];
            if (row == col) h += lambda;
        }
        coef[k][w] = h;
    }
}

// gradient entries of rows i1, i2 at column j for the CURRENT codes
__device__ inline void current_g(const float *__restrict__ G, long p, long i1, long i2, long j,
                                 const float *__restrict__ pend_d, int npend, const float (*coef)[4], float &g1,
                                 float &g2) {
    g1 = G[i1 * p + j];
    g2 = G[i2 * p + j];
    // four pending slots per trip, so that their loads are in flight together
    for (int k0 = 0; k0 < npend; k0 += 4) {
        float d1[4], d2[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int k = min(k0 + u, npend - 1);
            d1[u] = pend_d[(long)(2 * k) * p + j];
            d2[u] = pend_d[(long)(2 * k + 1) * p + j];
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (k0 + u < npend) {
                g1 -= coef[k0 + u][0] * d1[u] + coef[k0 + u][1] * d2[u];
                g2 -= coef[k0 + u][2] * d1[u] + coef[k0 + u][3] * d2[u];
            }
        }
    }
}

// grid (chunks, npairs), block 256
__global__ __launch_bounds__(256) void ls_evaluate_kernel(const float *__restrict__ H, float lambda,
                                                          const float *__restrict__ G,
                                                          const uint8_t *__restrict__ codes, long n, long p,
                                                          int levels, long g, const float *__restrict__ scales,
                                                          const int32_t *__restrict__ pairs,
                                                          const int32_t *__restrict__ pend_idx,
                                                          const float *__restrict__ pend_d, int npend,
                                                          float *__restrict__ partial, int chunks) {
    __shared__ float sh[4];
    __shared__ float coef[LS_K][4];
    const int pr = blockIdx.y;
    const long i1 = pairs[2 * pr], i2 = pairs[2 * pr + 1];
    if (i1 < 0 || i2 < 0 || i1 >= n || i2 >= n || i1 == i2) {      // not a row pair: contributes nothing
        if (threadIdx.x == 0) partial[(long)pr * chunks + blockIdx.x] = 0.f;
        return;
    }
    load_pending_coef(H, lambda, n, i1, i2, pend_idx, npend, coef);
    __syncthreads();
    const float h11 = H[i1 * n + i1] + lambda, h22 = H[i2 * n + i2] + lambda, h12 = H[i1 * n + i2];
    const float *s1 = scales + (i1 / g) * p, *s2 = scales + (i2 / g) * p;
    float sum = 0.f;
    const long j = (long)blockIdx.x * LS_CHUNK + threadIdx.x;
    if (j < p) {
        float g1, g2;
        current_g(G, p, i1, i2, j, pend_d, npend, coef, g1, g2);
        PairEval e = eval_column(g1, g2, codes[i1 * p + j], codes[i2 * p + j], s1[j], s2[j], h11, h22, h12, levels);
        sum = e.gain;
    }
    sum = wave_sum_f(sum);
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    if (lane == 0) sh[w] = sum;
    __syncthreads();
    if (threadIdx.x == 0) partial[(long)pr * chunks + blockIdx.x] = (sh[0] + sh[1]) + (sh[2] + sh[3]);
}

// grid ceil(p/256), block 256.  Every block finds the same winner; block 0 records it.
__global__ __launch_bounds__(256) void ls_plan_kernel(const float *__restrict__ H, float lambda,
                                                      const float *__restrict__ G, uint8_t *__restrict__ codes,
                                                      long n, long p, int levels, long g,
                                                      const float *__restrict__ scales,
                                                      const int32_t *__restrict__ pairs, int npairs,
                                                      const float *__restrict__ partial, int chunks,
                                                      int32_t *__restrict__ pend_idx, float *__restrict__ pend_d,
                                                      int slot, int32_t *__restrict__ choice,
                                                      int *__restrict__ moves, double *__restrict__ drop) {
    __shared__ float stot[256];
    __shared__ int sidx[256];
    __shared__ float coef[LS_K][4];
    const int tid = threadIdx.x;
    float best = 0.f;
    int bidx = -1;
    for (int pr = tid; pr < npairs; pr += 256) {
        float t = 0.f;
        for (int c = 0; c < chunks; ++c) t += partial[(long)pr * chunks + c];
        if (t > best) {            // strictly larger: within a thread slots come in increasing order
            best = t;
            bidx = pr;
        }
    }
    stot[tid] = best;
    sidx[tid] = bidx;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
        if (tid < s) {
            const float o = stot[tid + s];
            const int oi = sidx[tid + s];
            // larger total wins; equal totals: the lower slot wins
            if (oi >= 0 && (o > stot[tid] || (o == stot[tid] && (sidx[tid] < 0 || oi < sidx[tid])))) {
                stot[tid] = o;
                sidx[tid] = oi;
            }
        }
        __syncthreads();
    }
    const int win = sidx[0];
    const float wtot = stot[0];
    if (blockIdx.x == 0 && tid == 0) {
        choice[0] = win;
        choice[1] = win >= 0 ? pairs[2 * win] : -1;
        choice[2] = win >= 0 ? pairs[2 * win + 1] : -1;
        pend_idx[2 * slot] = win >= 0 ? pairs[2 * win] : -1;
        pend_idx[2 * slot + 1] = win >= 0 ? pairs[2 * win + 1] : -1;
        if (win >= 0) {
            *moves += 1;
            *drop += (double)wtot;
        }
    }
    if (win < 0) {
        // empty slot: zero steps, so that a later on-the-fly correction reads finite values
        const long j = (long)blockIdx.x * 256 + tid;
        if (j < p) {
            pend_d[(long)(2 * slot) * p + j] = 0.f;
            pend_d[(long)(2 * slot + 1) * p + j] = 0.f;
        }
        return;
    }
    const long i1 = pairs[2 * win], i2 = pairs[2 * win + 1];
    load_pending_coef(H, lambda, n, i1, i2, pend_idx, slot, coef);     // slots before this one
    __syncthreads();
    const long j = (long)blockIdx.x * 256 + tid;
    if (j >= p) return;
    const float h11 = H[i1 * n + i1] + lambda, h22 = H[i2 * n + i2] + lambda, h12 = H[i1 * n + i2];
    const float sc1 = scales[(i1 / g) * p + j], sc2 = scales[(i2 / g) * p + j];
    const int k1 = codes[i1 * p + j], k2 = codes[i2 * p + j];
    float g1, g2;
    current_g(G, p, i1, i2, j, pend_d, slot, coef, g1, g2);
    PairEval e = eval_column(g1, g2, k1, k2, sc1, sc2, h11, h22, h12, levels);
    float d1 = 0.f, d2 = 0.f;
    if (e.combo >= 0) {
        const int sg1 = (e.combo & 2) ? -1 : 1, sg2 = (e.combo & 1) ? -1 : 1;
        d1 = (float)sg1 * sc1;
        d2 = (float)sg2 * sc2;
        codes[i1 * p + j] = (uint8_t)(k1 + sg1);
        codes[i2 * p + j] = (uint8_t)(k2 + sg2);
    }
    pend_d[(long)(2 * slot) * p + j] = d1;
    pend_d[(long)(2 * slot + 1) * p + j] = d2;
}

// grid (ceil(p/1024), ceil(n/8)), block 256: each thread 4 columns x 8 rows; applies `count` slots
__global__ __launch_bounds__(256) void ls_flush_kernel(const float *__restrict__ H, float lambda,
                                                       float *__restrict__ G, long n, long p,
                                                       const int32_t *__restrict__ pend_idx,
                                                       const float *__restrict__ pend_d, int count) {
    // coefficients of this block's 8 rows for every pending slot: coef[k][0][rr] = H'[r0+rr][a_k],
    // coef[k][1][rr] = H'[r0+rr][b_k] (column a of the symmetric H' read as row a); an empty slot gives 0
    __shared__ float coef[LS_K][2][8];
    __shared__ int any_sh;
    const long r0 = (long)blockIdx.y * 8;
    if (threadIdx.x == 0) any_sh = 0;
    __syncthreads();
    for (int e = threadIdx.x; e < count * 16; e += 256) {
        const int k = e >> 4, w = (e >> 3) & 1, rr = e & 7;
        const long src = pend_idx[2 * k + w];
        const long i = r0 + rr;
        float h = 0.f;
        if (pend_idx[2 * k] >= 0 && i < n) {
            h = H[src * n + i];
            if (i == src) h += lambda;
            any_sh = 1;
        }
        coef[k][w][rr] = h;
    }
    __syncthreads();
    const bool any = any_sh != 0;
    const long j0 = ((long)blockIdx.x * 256 + threadIdx.x) * 4;
    if (j0 >= p || !any) return;
    float acc[8][4];
#pragma unroll
    for (int rr = 0; rr < 8; ++rr)
#pragma unroll
        for (int c = 0; c < 4; ++c) acc[rr][c] = 0.f;
    const bool vecd = (p % 4 == 0);
    for (int k = 0; k < count; ++k) {
        if (pend_idx[2 * k] < 0) continue;
        float d1[4], d2[4];
        if (vecd) {
            const floatx4 t1 = *(const floatx4 *)(pend_d + (long)(2 * k) * p + j0);
            const floatx4 t2 = *(const floatx4 *)(pend_d + (long)(2 * k + 1) * p + j0);
            d1[0] = t1.x; d1[1] = t1.y; d1[2] = t1.z; d1[3] = t1.w;
            d2[0] = t2.x; d2[1] = t2.y; d2[2] = t2.z; d2[3] = t2.w;
        } else {
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                d1[c] = j0 + c < p ? pend_d[(long)(2 * k) * p + j0 + c] : 0.f;
                d2[c] = j0 + c < p ? pend_d[(long)(2 * k + 1) * p + j0 + c] : 0.f;
            }
        }
#pragma unroll
        for (int rr = 0; rr < 8; ++rr) {
            const float c1 = coef[k][0][rr], c2 = coef[k][1][rr];
#pragma unroll
            for (int c = 0; c < 4; ++c) acc[rr][c] += c1 * d1[c] + c2 * d2[c];
        }
    }
    const bool vec = (p % 4 == 0);
#pragma unroll
    for (int rr = 0; rr < 8; ++rr) {
        const long i = r0 + rr;
        if (i >= n) break;
        float *row = G + i * p + j0;
        if (vec) {
            floatx4 gq = *(floatx4 *)row;
            gq.x -= acc[rr][0]; gq.y -= acc[rr][1]; gq.z -= acc[rr][2]; gq.w -= acc[rr][3];
            *(floatx4 *)row = gq;
        } else {
#pragma unroll
            for (int c = 0; c < 4; ++c)
                if (j0 + c < p) row[c] -= acc[rr][c];
        }
    }
}

}  // namespace

int admmq_ls_chunks(int64_t p) { return (int)((p + LS_CHUNK - 1) / LS_CHUNK); }
int admmq_ls_defer() { return LS_K; }

// One batch: evaluate the candidate pairs against the current codes, then (if `apply`) record the best
// one in pending slot `slot` (= batch index mod K).  The caller flushes after slot K-1 and at the end.
admmq_status admmq_k_ls_batch(admmq_ctx *ctx, const float *H, float lambda, float *G, uint8_t *codes, int64_t n,
                              int64_t p, int bits, int64_t g, const float *scales, const int32_t *pairs,
                              int npairs, float *partial, int32_t *pend_idx, float *pend_d, int slot,
                              int32_t *choice, int *dev_moves, double *dev_drop, int apply) {
    const int chunks = admmq_ls_chunks(p);
    const int levels = (1 << bits) - 1;
    hipLaunchKernelGGL(ls_evaluate_kernel, dim3((unsigned)chunks, (unsigned)npairs), dim3(256), 0, ctx->stream, H,
                       lambda, G, codes, (long)n, (long)p, levels, (long)g, scales, pairs, pend_idx, pend_d, slot,
                       partial, chunks);
    if (apply) {
        hipLaunchKernelGGL(ls_plan_kernel, dim3((unsigned)((p + 255) / 256)), dim3(256), 0, ctx->stream, H, lambda, G,
                           codes, (long)n, (long)p, levels, (long)g, scales, pairs, npairs, partial, chunks, pend_idx,
                           pend_d, slot, choice, dev_moves, dev_drop);
    }
    ADMMQ_HIP(hipGetLastError());
    return ADMMQ_OK;
}

admmq_status admmq_k_ls_flush(admmq_ctx *ctx, const float *H, float lambda, float *G, int64_t n, int64_t p,
                              const int32_t *pend_idx, const float *pend_d, int count) {
    if (count <= 0) return ADMMQ_OK;
    dim3 grid((unsigned)((p + 1023) / 1024), (unsigned)((n + 7) / 8));
    const int sp = admmq_prof_begin(ctx, ADMMQ_TAG_LS_APPLY);
    hipLaunchKernelGGL(ls_flush_kernel, grid, dim3(256), 0, ctx->stream, H, lambda, G, (long)n, (long)p, pend_idx,
                       pend_d, count);
    admmq_prof_end(ctx, sp);
    ADMMQ_HIP(hipGetLastError());
    return ADMMQ_OK;
}

// totals[pr] = sum of the chunk partials (fixed order); used by the single-step entry point
__global__ void ls_totals_kernel(const float *__restrict__ partial, int chunks, int npairs,
                                 float *__restrict__ totals) {
    int pr = blockIdx.x * blockDim.x + threadIdx.x;
    if (pr >= npairs) return;
    float t = 0.f;
    for (int c = 0; c < chunks; ++c) t += partial[(long)pr * chunks + c];
    totals[pr] = t;
}

admmq_status admmq_k_ls_totals(admmq_ctx *ctx, const float *partial, int chunks, int npairs, float *totals) {
    hipLaunchKernelGGL(ls_totals_kernel, dim3((unsigned)((npairs + 63) / 64)), dim3(64), 0, ctx->stream, partial,
                       chunks, npairs, totals);
    ADMMQ_HIP(hipGetLastError());
    return ADMMQ_OK;
}
