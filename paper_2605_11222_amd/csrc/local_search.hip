// Pair-swap local search kernels (Sec. 3.5, eq. 11), in the unscaled space on H' = H + lambda I.
//
// Per batch of candidate row pairs:
//   evaluate : one block per (pair, column chunk); every column takes the best feasible sign
//              combination of (+-delta_i1, +-delta_i2) by eq. 11 if it lowers the loss; the chunk's
//              summed gain goes to partial[pair][chunk]
//   select   : one block; sums the chunks in a fixed order, picks the largest total (lowest slot on
//              ties), and for the winner writes the per-column steps dstep[2][p] and the new codes
//   apply    : streams G once:  G[i][j] -= H'[i][i1] dstep1[j] + H'[i][i2] dstep2[j]
// Nothing is applied when the best total is not positive (the apply kernel returns at once).
#include "common.h"

typedef float floatx4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int LS_CHUNK = 1024;   // columns per evaluate block (256 threads x 4)

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

// grid (chunks, npairs), block 256
__global__ __launch_bounds__(256) void ls_evaluate_kernel(const float *__restrict__ H, float lambda,
                                                          const float *__restrict__ G,
                                                          const uint8_t *__restrict__ codes, long n, long p,
                                                          int levels, long g, const float *__restrict__ scales,
                                                          const int32_t *__restrict__ pairs,
                                                          float *__restrict__ partial, int chunks) {
    __shared__ float sh[4];
    const int pr = blockIdx.y;
    const long i1 = pairs[2 * pr], i2 = pairs[2 * pr + 1];
    if (i1 < 0 || i2 < 0 || i1 >= n || i2 >= n || i1 == i2) {      // not a row pair: contributes nothing
        if (threadIdx.x == 0) partial[(long)pr * chunks + blockIdx.x] = 0.f;
        return;
    }
    const float h11 = H[i1 * n + i1] + lambda, h22 = H[i2 * n + i2] + lambda, h12 = H[i1 * n + i2];
    const float *s1 = scales + (i1 / g) * p, *s2 = scales + (i2 / g) * p;
    float sum = 0.f;
    const long jbase = (long)blockIdx.x * LS_CHUNK;
    for (int q = 0; q < 4; ++q) {
        const long j = jbase + q * 256 + threadIdx.x;
        if (j < p) {
            PairEval e = eval_column(G[i1 * p + j], G[i2 * p + j], codes[i1 * p + j], codes[i2 * p + j], s1[j],
                                     s2[j], h11, h22, h12, levels);
            sum += e.gain;
        }
    }
    sum = wave_sum_f(sum);
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    if (lane == 0) sh[w] = sum;
    __syncthreads();
    if (threadIdx.x == 0) partial[(long)pr * chunks + blockIdx.x] = (sh[0] + sh[1]) + (sh[2] + sh[3]);
}

// one block of 256 threads
__global__ __launch_bounds__(256) void ls_select_kernel(const float *__restrict__ H, float lambda,
                                                        const float *__restrict__ G, uint8_t *__restrict__ codes,
                                                        long n, long p, int levels, long g,
                                                        const float *__restrict__ scales,
                                                        const int32_t *__restrict__ pairs, int npairs,
                                                        const float *__restrict__ partial, int chunks,
                                                        float *__restrict__ totals, int32_t *__restrict__ choice,
                                                        float *__restrict__ dstep, int *__restrict__ moves,
                                                        double *__restrict__ drop) {
    __shared__ float stot[256];
    __shared__ int sidx[256];
    const int tid = threadIdx.x;
    float best = 0.f;
    int bidx = -1;
    for (int pr = tid; pr < npairs; pr += 256) {
        float t = 0.f;
        for (int c = 0; c < chunks; ++c) t += partial[(long)pr * chunks + c];
        if (totals) totals[pr] = t;
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
    if (tid == 0) {
        choice[0] = win;
        choice[1] = win >= 0 ? pairs[2 * win] : -1;
        choice[2] = win >= 0 ? pairs[2 * win + 1] : -1;
        if (win >= 0) {
            *moves += 1;
            *drop += (double)wtot;
        }
    }
    if (win < 0) return;
    const long i1 = pairs[2 * win], i2 = pairs[2 * win + 1];
    const float h11 = H[i1 * n + i1] + lambda, h22 = H[i2 * n + i2] + lambda, h12 = H[i1 * n + i2];
    const float *s1 = scales + (i1 / g) * p, *s2 = scales + (i2 / g) * p;
    for (long j = tid; j < p; j += 256) {
        const int k1 = codes[i1 * p + j], k2 = codes[i2 * p + j];
        PairEval e = eval_column(G[i1 * p + j], G[i2 * p + j], k1, k2, s1[j], s2[j], h11, h22, h12, levels);
        float d1 = 0.f, d2 = 0.f;
        if (e.combo >= 0) {
            const int sg1 = (e.combo & 2) ? -1 : 1, sg2 = (e.combo & 1) ? -1 : 1;
            d1 = (float)sg1 * s1[j];
            d2 = (float)sg2 * s2[j];
            codes[i1 * p + j] = (uint8_t)(k1 + sg1);
            codes[i2 * p + j] = (uint8_t)(k2 + sg2);
        }
        dstep[j] = d1;
        dstep[p + j] = d2;
    }
}

// grid (ceil(p/1024), ceil(n/8)), block 256: each thread 4 columns x 8 rows
__global__ __launch_bounds__(256) void ls_apply_kernel(const float *__restrict__ H, float lambda,
                                                       float *__restrict__ G, long n, long p,
                                                       const int32_t *__restrict__ choice,
                                                       const float *__restrict__ dstep) {
    if (choice[0] < 0) return;
    const long i1 = choice[1], i2 = choice[2];
    const long j0 = ((long)blockIdx.x * 256 + threadIdx.x) * 4;
    if (j0 >= p) return;
    float d1[4], d2[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        d1[c] = j0 + c < p ? dstep[j0 + c] : 0.f;
        d2[c] = j0 + c < p ? dstep[p + j0 + c] : 0.f;
    }
    const bool vec = (p % 4 == 0);
    const long r0 = (long)blockIdx.y * 8;
#pragma unroll
    for (int rr = 0; rr < 8; ++rr) {
        const long i = r0 + rr;
        if (i >= n) break;
        // column i1 of the symmetric H' read as row i1
        float c1 = H[i1 * n + i], c2 = H[i2 * n + i];
        if (i == i1) c1 += lambda;
        if (i == i2) c2 += lambda;
        float *row = G + i * p + j0;
        if (vec) {
            floatx4 gq = *(floatx4 *)row;
            gq.x -= c1 * d1[0] + c2 * d2[0];
            gq.y -= c1 * d1[1] + c2 * d2[1];
            gq.z -= c1 * d1[2] + c2 * d2[2];
            gq.w -= c1 * d1[3] + c2 * d2[3];
            *(floatx4 *)row = gq;
        } else {
#pragma unroll
            for (int c = 0; c < 4; ++c)
                if (j0 + c < p) row[c] -= c1 * d1[c] + c2 * d2[c];
        }
    }
}

}  // namespace

int admmq_ls_chunks(int64_t p) { return (int)((p + LS_CHUNK - 1) / LS_CHUNK); }

admmq_status admmq_k_ls_batch(admmq_ctx *ctx, const float *H, float lambda, float *G, uint8_t *codes, int64_t n,
                              int64_t p, int bits, int64_t g, const float *scales, const int32_t *pairs,
                              int npairs, float *partial, float *totals_or_null, int32_t *choice, float *dstep,
                              int *dev_moves, double *dev_drop, int apply) {
    const int chunks = admmq_ls_chunks(p);
    const int levels = (1 << bits) - 1;
    hipLaunchKernelGGL(ls_evaluate_kernel, dim3((unsigned)chunks, (unsigned)npairs), dim3(256), 0, ctx->stream, H,
                       lambda, G, codes, (long)n, (long)p, levels, (long)g, scales, pairs, partial, chunks);
    if (apply) {
        hipLaunchKernelGGL(ls_select_kernel, dim3(1), dim3(256), 0, ctx->stream, H, lambda, G, codes, (long)n,
                           (long)p, levels, (long)g, scales, pairs, npairs, partial, chunks, totals_or_null, choice,
                           dstep, dev_moves, dev_drop);
        dim3 grid((unsigned)((p + 1023) / 1024), (unsigned)((n + 7) / 8));
        const int sp = admmq_prof_begin(ctx, ADMMQ_TAG_LS_APPLY);
        hipLaunchKernelGGL(ls_apply_kernel, grid, dim3(256), 0, ctx->stream, H, lambda, G, (long)n, (long)p, choice,
                           dstep);
        admmq_prof_end(ctx, sp);
    }
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
