// Pair-swap local search kernels (Sec. 3.5, eq. 11), in the unscaled space on H' = H + lambda I.
//
// Per batch of candidate row pairs:
//   evaluate : one block per (pair, column chunk); every column takes the best feasible sign
//              combination of (+-delta_i1, +-delta_i2) by eq. 11 if it lowers the loss; the chunk's
//              summed gain goes to partial[pair][chunk]
//   plan     : every block sums the chunks in a fixed order and picks the largest total (lowest slot
//              on ties) - the same winner in every block - and takes, for its own column, the winner's
//              move from the byte its evaluation left: slot (batch mod K) of a pending list
//   (the plan of batch m and the evaluation of batch m+1 share ONE launch, ls_step_kernel)
//   flush    : every K batches G is streamed ONCE for all pending pairs:
//              G[i][j] -= sum_k H'[i][a_k] d1_k[j] + H'[i][b_k] d2_k[j]          (rank-2K correction)
//              and the stored codes of the pending rows take their moves
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

// Wave-wide reductions without a trip through LDS: the halves of the wave and the 16-lane rows are folded with the
// gfx950 lane-swap instructions (permlane32_swap(x, x) hands every lane its own half's value and the other
// half's), the rows with DPP rotations by 8, 4, 2, 1.  The result is left in every lane; the order is fixed.
template <int N>
__device__ inline unsigned row_ror(unsigned x) {
    return (unsigned)__builtin_amdgcn_update_dpp(0, (int)x, 0x120 + N, 0xF, 0xF, true);
}
__device__ inline float wave_sum_f(float v) {
    auto a = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    v = __uint_as_float(a[0]) + __uint_as_float(a[1]);
    a = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    v = __uint_as_float(a[0]) + __uint_as_float(a[1]);
    v += __uint_as_float(row_ror<8>(__float_as_uint(v)));
    v += __uint_as_float(row_ror<4>(__float_as_uint(v)));
    v += __uint_as_float(row_ror<2>(__float_as_uint(v)));
    v += __uint_as_float(row_ror<1>(__float_as_uint(v)));
    return v;
}

constexpr int LS_K = 16;          // pending pairs between two passes over G (cfg2 on MI355X: 8 -> 0.132 s,
                                  // 16 -> 0.120 s, 32 -> 0.181 s for the whole search)

__device__ inline int step_sign(float d) { return (d > 0.f) - (d < 0.f); }

// the pending steps of column j, all slots, in registers (zero beyond npend): the same values serve the
// winner's rows and the block's own pair
struct PendCol {
    float d1[LS_K], d2[LS_K];
};

__device__ inline void load_pending_col(const float *__restrict__ pend_d, long p, long j, int npend, PendCol &pc) {
#pragma unroll
    for (int k = 0; k < LS_K; ++k) {
        const bool on = k < npend;
        pc.d1[k] = on ? pend_d[(long)(2 * k) * p + j] : 0.f;
        pc.d2[k] = on ? pend_d[(long)(2 * k + 1) * p + j] : 0.f;
    }
}

// One applied pair's steps (d1, d2) onto the gradient entries of a row pair: g -= H'[row][a] d1 + H'[row][b] d2,
// co = H'[i1][a], H'[i1][b], H'[i2][a], H'[i2][b].  Fused multiply-adds in a fixed order: half the vector
// instructions of separate products and sums, and the one place where both forms of the search (one launch per
// batch, one launch per group) take this step, so that they round alike.
__device__ inline void pending_onto(float &g1, float &g2, const float *co, float d1, float d2) {
    g1 = __fmaf_rn(-co[1], d2, __fmaf_rn(-co[0], d1, g1));
    g2 = __fmaf_rn(-co[3], d2, __fmaf_rn(-co[2], d1, g2));
}

// stored gradient entries and codes of a row pair at one column -> those of the CURRENT codes: the pending
// moves are added (codes and G are both brought up to date by the flush)
__device__ inline void apply_pending(const PendCol &pc, int npend, const float (*coef)[4], const int *which,
                                     float &g1, float &g2, int &k1, int &k2) {
#pragma unroll
    for (int k = 0; k < LS_K; ++k) {
        if (k < npend) {
            pending_onto(g1, g2, coef[k], pc.d1[k], pc.d2[k]);
            const int wh = which[k];
            if (wh) {
                const int s1 = step_sign(pc.d1[k]), s2 = step_sign(pc.d2[k]);
                k1 += ((wh & 1) ? s1 : 0) + ((wh & 2) ? s2 : 0);
                k2 += ((wh & 4) ? s1 : 0) + ((wh & 8) ? s2 : 0);
            }
        }
    }
}

// larger total wins; equal totals: the lower slot wins; slot -1 = no candidate
__device__ inline void better(float &t, int &i, float ot, int oi) {
    if (oi >= 0 && (ot > t || (ot == t && (i < 0 || oi < i)))) {
        t = ot;
        i = oi;
    }
}

constexpr int LS_FAST_PAIRS = 64;      // candidate pairs per batch up to which the winner's data is prefetched

// the best (total, slot) of the wave, in every lane (same folding as wave_sum_f; `better` is commutative)
__device__ inline void wave_best(float &t, int &i) {
    {
        const auto a = __builtin_amdgcn_permlane32_swap(__float_as_uint(t), __float_as_uint(t), false, false);
        const auto b = __builtin_amdgcn_permlane32_swap((unsigned)i, (unsigned)i, false, false);
        t = __uint_as_float(a[0]);
        i = (int)b[0];
        better(t, i, __uint_as_float(a[1]), (int)b[1]);
    }
    {
        const auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(t), __float_as_uint(t), false, false);
        const auto b = __builtin_amdgcn_permlane16_swap((unsigned)i, (unsigned)i, false, false);
        t = __uint_as_float(a[0]);
        i = (int)b[0];
        better(t, i, __uint_as_float(a[1]), (int)b[1]);
    }
    better(t, i, __uint_as_float(row_ror<8>(__float_as_uint(t))), (int)row_ror<8>((unsigned)i));
    better(t, i, __uint_as_float(row_ror<4>(__float_as_uint(t))), (int)row_ror<4>((unsigned)i));
    better(t, i, __uint_as_float(row_ror<2>(__float_as_uint(t))), (int)row_ror<2>((unsigned)i));
    better(t, i, __uint_as_float(row_ror<1>(__float_as_uint(t))), (int)row_ror<1>((unsigned)i));
}

// The same choice from one 64-bit key per lane: a positive total's bit pattern orders like the total, and below it
// 2^32 - 1 - slot makes the lower slot the larger key; 0 = no candidate.  One compare and two selects per folding
// step instead of the half dozen of `better` (the group kernel's sixteen waves each run this once per batch).
__device__ inline unsigned long long best_key(float t, int i) {
    return (i >= 0 && t > 0.f) ? (((unsigned long long)__float_as_uint(t) << 32) | (unsigned long long)(0xFFFFFFFFu - (unsigned)i)) : 0ull;
}
__device__ inline unsigned long long wave_max_key(unsigned long long k) {
    unsigned lo = (unsigned)k, hi = (unsigned)(k >> 32);
    auto fold = [&](unsigned olo, unsigned ohi) {
        const unsigned long long o = ((unsigned long long)ohi << 32) | olo, m = ((unsigned long long)hi << 32) | lo;
        if (o > m) {
            lo = olo;
            hi = ohi;
        }
    };
    {
        const auto a = __builtin_amdgcn_permlane32_swap(lo, lo, false, false);
        const auto b = __builtin_amdgcn_permlane32_swap(hi, hi, false, false);
        lo = a[0];
        hi = b[0];
        fold(a[1], b[1]);
    }
    {
        const auto a = __builtin_amdgcn_permlane16_swap(lo, lo, false, false);
        const auto b = __builtin_amdgcn_permlane16_swap(hi, hi, false, false);
        lo = a[0];
        hi = b[0];
        fold(a[1], b[1]);
    }
    fold(row_ror<8>(lo), row_ror<8>(hi));
    fold(row_ror<4>(lo), row_ror<4>(hi));
    fold(row_ror<2>(lo), row_ror<2>(hi));
    fold(row_ror<1>(lo), row_ror<1>(hi));
    return ((unsigned long long)hi << 32) | lo;
}

// One step of the search, grid (chunks, npairs), block 256, one column per thread:
//   plan     (when a previous batch exists): every block adds that batch's chunk partials in a fixed order and
//            finds its winner (largest total, lowest slot on ties) - the same winner in every block.  The winner's
//            move at each column is the one its evaluation chose in the previous launch (kept as one byte per
//            pair and column); the blocks of pair 0 store the applied steps into pending slot `slot_prev`, the
//            blocks of pair 1 copy the two H' columns of the winner's rows into the slot's coefficient cache,
//            one thread records the pair;
//   evaluate (when a current batch exists): the block's own candidate pair at its column, against the codes and
//            the gradient AFTER the winner's move, which is taken from registers, never from memory that another
//            block may be writing; the chosen sign combination goes to the byte array of this batch.
// Nothing a block reads is written in the same launch: codes and G change only in the flush, slot `slot_prev`
// of the pending arrays is written here and first read by the next launch, the partials and the move bytes of
// the two batches live in buffers that trade places every step.
// npend = pending slots already in memory (== slot_prev whenever there is a previous batch).
// Latency is what this launch costs, so everything that does not depend on the winner is requested up front,
// including (for up to LS_FAST_PAIRS candidates) every candidate's move byte at this column and the four
// H' entries that couple the own pair with every candidate: after the selection no load from DRAM remains.
// hcol[(2k + w) n + r] = H'[r][row w of slot k]: coefficients of the pending corrections without a dependent
// look-up of the slot's rows; empty slots keep finite stale entries (their steps are zero).
__global__ __launch_bounds__(256) void ls_step_kernel(const float *__restrict__ H, float lambda,
                                                      const float *__restrict__ G, const uint8_t *__restrict__ codes,
                                                      long n, long p, int levels, long g,
                                                      const float *__restrict__ scales,
                                                      const int32_t *__restrict__ pairs_prev, int npairs_prev,
                                                      const float *__restrict__ partial_prev,
                                                      const uint8_t *__restrict__ mv_prev, int slot_prev,
                                                      const int32_t *__restrict__ pairs_cur, int npend,
                                                      int32_t *pend_idx, float *pend_d, float *hcol,
                                                      float *__restrict__ partial_cur, uint8_t *__restrict__ mv_cur,
                                                      int chunks, int32_t *__restrict__ choice,
                                                      int *__restrict__ moves, double *__restrict__ drop,
                                                      const int32_t *__restrict__ pairs_next, int npairs_next,
                                                      const float *__restrict__ exs_cur,
                                                      float *__restrict__ exs_next) {
    __shared__ float coef_o[LS_K][4];
    __shared__ int which_o[LS_K];
    __shared__ int cand[2 * LS_FAST_PAIRS];
    __shared__ float exs[LS_FAST_PAIRS][4];
    __shared__ __align__(16) uint8_t smv[LS_FAST_PAIRS][LS_CHUNK];
    __shared__ float wtot_sh[4];
    __shared__ int widx_sh[4];
    __shared__ float sh[4];
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const long j = (long)blockIdx.x * LS_CHUNK + tid;
    const bool first_block = blockIdx.x == 0 && blockIdx.y == 0;
    const bool in = j < p;
    const bool fast = npairs_prev <= LS_FAST_PAIRS;

    // ---- loads that need no winner: all of them are requested before the first one is used -------------
    long i1 = -1, i2 = -1;
    bool own = false;
    if (pairs_cur) {
        i1 = pairs_cur[2 * blockIdx.y];
        i2 = pairs_cur[2 * blockIdx.y + 1];
        own = !(i1 < 0 || i2 < 0 || i1 >= n || i2 >= n || i1 == i2);      // else: not a row pair
    }
    const bool prev_fast = npairs_prev > 0 && fast;
    const bool mv_vec = fast && (p & 15) == 0;
    // (1) the coupling entries of H' between the own pair and every candidate of the previous batch: gathered by
    // the previous launch into exs_cur (one plain load here); without it, the oldest request is the one a second
    // request depends on: candidate row -> coupling entry
    long ex_col = -1;
    const bool ex_on = prev_fast && own && tid < 4 * npairs_prev;
    float ex_ready = 0.f;
    if (ex_on) {
        if (exs_cur) ex_ready = exs_cur[((long)blockIdx.y * LS_FAST_PAIRS) * 4 + tid];
        else ex_col = pairs_prev[2 * (tid >> 2) + (tid & 1)];
    }
    // the same gather for the NEXT launch (own pairs of the next batch x candidates of this one): one entry per
    // thread in the first block column, requested here and stored at the very end, off this launch's critical path
    const bool gather = exs_next && pairs_next && pairs_cur && blockIdx.x == 0 && (int)blockIdx.y < npairs_next &&
                        (int)gridDim.y <= LS_FAST_PAIRS && npairs_next <= LS_FAST_PAIRS && tid < 4 * (int)gridDim.y;
    long g_row = -1, g_col = -1;
    if (gather) {
        g_row = pairs_next[2 * blockIdx.y + ((tid >> 1) & 1)];
        g_col = pairs_cur[2 * (tid >> 2) + (tid & 1)];
    }
    // (2) everything else
    int cand_r = 0;
    if (prev_fast && tid < 2 * npairs_prev) cand_r = pairs_prev[tid];
    long pa = -1, pb = -1;
    float coef_r = 0.f;
    if (own) {
        if (tid < npend) {
            pa = pend_idx[2 * tid];
            pb = pend_idx[2 * tid + 1];
        }
        if (tid < npend * 4) coef_r = hcol[(long)(2 * (tid >> 2) + (tid & 1)) * n + ((tid & 2) ? i2 : i1)];
    }
    PendCol pc;
    if (in) load_pending_col(pend_d, p, j, npend, pc);
    float og1 = 0.f, og2 = 0.f, oh11 = 0.f, oh22 = 0.f, oh12 = 0.f, osc1 = 0.f, osc2 = 0.f;
    int ok1 = 0, ok2 = 0;
    if (own && in) {
        og1 = G[i1 * p + j];
        og2 = G[i2 * p + j];
        ok1 = codes[i1 * p + j];
        ok2 = codes[i2 * p + j];
        osc1 = scales[(i1 / g) * p + j];
        osc2 = scales[(i2 / g) * p + j];
        oh11 = H[i1 * n + i1] + lambda;
        oh22 = H[i2 * n + i2] + lambda;
        oh12 = H[i1 * n + i2];
    }
    // with one group per column the winner's grid steps do not depend on its rows
    const bool one_group = g >= n;
    float sc_col = 0.f;
    if (one_group && in && npairs_prev > 0) sc_col = scales[j];
    // every candidate's move bytes for the block's 256 columns go through LDS: 16-byte loads, 16 threads to a
    // candidate's row segment (four loads per thread when there are 64 candidates)
    uint4 mvr[LS_FAST_PAIRS / 16];
    if (prev_fast && mv_vec) {
        const long c0 = (long)blockIdx.x * LS_CHUNK + (tid & 15) * 16;
#pragma unroll
        for (int r = 0; r < LS_FAST_PAIRS / 16; ++r) {
            const int q = (tid >> 4) + 16 * r;
            mvr[r] = (q < npairs_prev && c0 < p) ? *(const uint4 *)(mv_prev + (long)q * p + c0) : uint4{0u, 0u, 0u, 0u};
        }
    }
    // the candidates' chunk partials: sixteen are requested at a time (a loop of single loads would pay the cache
    // latency once per chunk) and added in chunk order; they come last so that nothing above waits for them
    float best = 0.f;
    int bidx = -1;
    if (npairs_prev > 0) {
        for (int pr = tid; pr < npairs_prev; pr += 256) {
            const float *src = partial_prev + (long)pr * chunks;
            float psum = 0.f;
            int c = 0;
            for (; c + 16 <= chunks; c += 16) {
                float v[16];
#pragma unroll
                for (int u = 0; u < 16; ++u) v[u] = src[c + u];
#pragma unroll
                for (int u = 0; u < 16; ++u) psum += v[u];
            }
            for (; c < chunks; ++c) psum += src[c];
            if (psum > best) {     // strictly larger: within a thread slots come in increasing order
                best = psum;
                bidx = pr;
            }
        }
    }
    // (3) the dependent request, then the hand-over to LDS
    float g_val = 0.f;
    if (gather && g_row >= 0 && g_row < n && g_col >= 0 && g_col < n)
        g_val = H[g_row * n + g_col] + (g_row == g_col ? lambda : 0.f);
    if (ex_on) {
        float h = ex_ready;
        if (!exs_cur) {
            const long row = (tid & 2) ? i2 : i1;
            h = 0.f;
            if (ex_col >= 0 && ex_col < n) h = H[row * n + ex_col] + (row == ex_col ? lambda : 0.f);
        }
        exs[tid >> 2][tid & 3] = h;
    }
    if (prev_fast && tid < 2 * npairs_prev) cand[tid] = cand_r;
    if (own) {
        if (tid < npend) which_o[tid] = pa < 0 ? 0 : ((pa == i1) | ((pb == i1) << 1) | ((pa == i2) << 2) | ((pb == i2) << 3));
        if (tid < npend * 4) coef_o[tid >> 2][tid & 3] = coef_r;
    }
    if (prev_fast && mv_vec) {
#pragma unroll
        for (int r = 0; r < LS_FAST_PAIRS / 16; ++r)
            *(uint4 *)(&smv[(tid >> 4) + 16 * r][(tid & 15) * 16]) = mvr[r];
    }
    // ---- the previous batch's winner ----------------------------------------------------------------------
    int win = -1;
    float wtot = 0.f;
    if (npairs_prev > 0) {
        wave_best(best, bidx);
        if (lane == 0) {
            wtot_sh[wv] = best;
            widx_sh[wv] = bidx;
        }
    }
    __syncthreads();                         // wave results, coef_o, which_o, cand, exs, smv
    if (npairs_prev > 0) {
        wtot = wtot_sh[0];
        win = widx_sh[0];
#pragma unroll
        for (int w = 1; w < 4; ++w) better(wtot, win, wtot_sh[w], widx_sh[w]);
    }
    // ---- the winner's move at column j --------------------------------------------------------------------
    long wi1 = -1, wi2 = -1;
    float nd1 = 0.f, nd2 = 0.f;
    int ws1 = 0, ws2 = 0;
    float ex[4] = {0.f, 0.f, 0.f, 0.f};
    if (win >= 0) {
        uint32_t mb = 0u;
        if (fast) {
            wi1 = cand[2 * win];
            wi2 = cand[2 * win + 1];
            if (mv_vec) mb = smv[win][tid];
            else if (in) mb = mv_prev[(long)win * p + j];
            if (own) {
#pragma unroll
                for (int w = 0; w < 4; ++w) ex[w] = exs[win][w];
            }
        } else {
            wi1 = pairs_prev[2 * win];
            wi2 = pairs_prev[2 * win + 1];
            if (in) mb = mv_prev[(long)win * p + j];
            if (own) {
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    const long row = (w & 2) ? i2 : i1, col = (w & 1) ? wi2 : wi1;
                    ex[w] = H[row * n + col] + (row == col ? lambda : 0.f);
                }
            }
        }
        if (in && mb != 0u) {
            const int combo = (int)mb - 1;
            ws1 = (combo & 2) ? -1 : 1;
            ws2 = (combo & 1) ? -1 : 1;
            nd1 = (float)ws1 * (one_group ? sc_col : scales[(wi1 / g) * p + j]);
            nd2 = (float)ws2 * (one_group ? sc_col : scales[(wi2 / g) * p + j]);
        }
    }
    if (npairs_prev > 0 && blockIdx.y == 0 && in) {
        pend_d[(long)(2 * slot_prev) * p + j] = nd1;        // zero steps for an empty slot
        pend_d[(long)(2 * slot_prev + 1) * p + j] = nd2;
    }
    if (win >= 0) {
        // coefficient cache of the new slot: the two H' columns (rows of the symmetric H) of the winner's rows.
        // The blocks of the pairs 1, 2, ... share the n entries out, one per thread (a loop in one row of blocks
        // would pay the memory latency once per trip); a launch without candidates has only row 0 and loops.
        if (gridDim.y > 1) {
            if (blockIdx.y >= 1) {
                const long r = (((long)blockIdx.y - 1) * gridDim.x + blockIdx.x) * LS_CHUNK + tid;
                const long cover = ((long)gridDim.y - 1) * gridDim.x * LS_CHUNK;
                for (long rr = r; rr < n; rr += cover) {
                    hcol[(long)(2 * slot_prev) * n + rr] = H[wi1 * n + rr] + (rr == wi1 ? lambda : 0.f);
                    hcol[(long)(2 * slot_prev + 1) * n + rr] = H[wi2 * n + rr] + (rr == wi2 ? lambda : 0.f);
                }
            }
        } else {
            for (long r = (long)blockIdx.x * LS_CHUNK + tid; r < n; r += (long)gridDim.x * LS_CHUNK) {
                hcol[(long)(2 * slot_prev) * n + r] = H[wi1 * n + r] + (r == wi1 ? lambda : 0.f);
                hcol[(long)(2 * slot_prev + 1) * n + r] = H[wi2 * n + r] + (r == wi2 ? lambda : 0.f);
            }
        }
    }
    if (npairs_prev > 0 && first_block && tid == 0) {
        choice[0] = win;
        choice[1] = (int32_t)wi1;
        choice[2] = (int32_t)wi2;
        pend_idx[2 * slot_prev] = (int32_t)wi1;
        pend_idx[2 * slot_prev + 1] = (int32_t)wi2;
        if (win >= 0) {
            *moves += 1;
            *drop += (double)wtot;
        }
    }
    if (gather) exs_next[((long)blockIdx.y * LS_FAST_PAIRS) * 4 + tid] = g_val;
    if (!pairs_cur) return;
    // ---- this block's candidate pair ----------------------------------------------------------------------
    float gain = 0.f;
    uint32_t mine = 0u;
    if (own && in) {
        apply_pending(pc, npend, coef_o, which_o, og1, og2, ok1, ok2);
        if (win >= 0) {
            // the move planned above changes the own pair's gradient rows by H'[i][wi1] nd1 + H'[i][wi2] nd2
            pending_onto(og1, og2, ex, nd1, nd2);
            ok1 += i1 == wi1 ? ws1 : (i1 == wi2 ? ws2 : 0);
            ok2 += i2 == wi1 ? ws1 : (i2 == wi2 ? ws2 : 0);
        }
        const PairEval e = eval_column(og1, og2, ok1, ok2, osc1, osc2, oh11, oh22, oh12, levels);
        gain = e.gain;
        mine = e.combo >= 0 ? (uint32_t)(e.combo + 1) : 0u;
    }
    if (in && mv_cur) mv_cur[(long)blockIdx.y * p + j] = (uint8_t)mine;
    gain = wave_sum_f(gain);
    if (lane == 0) sh[wv] = gain;
    __syncthreads();
    if (tid == 0) partial_cur[(long)blockIdx.y * chunks + blockIdx.x] = (sh[0] + sh[1]) + (sh[2] + sh[3]);
}

// ---- a whole group of up to LS_K batches in ONE launch ----------------------------------------------------------
// The batches of a group depend on one another only through the winner of the batch before (its move changes the
// gradient rows and codes the next candidates are evaluated against), and what the blocks of a batch owe one
// another is one number per candidate pair: its summed gain.  So the group runs as one kernel whose blocks stay
// on the chip and hand those sums to one another through a table in global memory:
//   grid (ceil(p / 256), ceil(npairs / (4 PP))), block 1024: wave w works on the pairs 4 PP y + 4 i + w/4, i < PP,
//   at the 64 columns 256 x + 64 (w%4) + lane.  PP = 1 (one candidate pair and one column per thread, as in the
//   launch-per-batch kernel) unless that would be more blocks than the chip holds at once.
//   Per batch: evaluate the own pair; the four wave sums of a pair add up to the block's 256-column sum, which
//   one thread stores into table[pair][x] together with the batch's sequence number (one 8-byte word, so a
//   reader that sees the number sees the value); every block reads the whole table, adds each pair's sums in
//   chunk order and finds the winner - the same sums in the same order as the launch-per-batch kernels, hence
//   the same winner everywhere.  The winner's steps at a block's 256 columns are not exchanged: four waves
//   evaluate the winning pair again from the same inputs in the same order, which gives the same bits.
//   Everything else a block needs is read-only during the group (H, G, codes, scales, the sampled pairs) or its
//   own (the steps applied so far at its columns, in LDS).
// Waiting is bounded: a poll that sees no progress for `spin_ticks` of the wall clock (or finds the abort word
// set by another block) makes its block leave, and the group then stays uncommitted: the flush that follows and
// all later group kernels check the commit counter and do nothing, and the host repeats the work from that group
// on with one launch per batch.  All blocks must be resident at once: the host picks PP from the occupancy the
// runtime reports for this kernel.
constexpr int LSG_TILE = 256;                          // columns per block
constexpr int LSG_PB_MAX = 8;                          // candidate pairs per block: 4 PP, PP = pairs per thread (1 or 2)
constexpr int LSG_MAX_CHUNKS = 32;
static_assert(LS_K == 16, "the group kernel's thread maps take sixteen slots per pair");

struct LsGroupArgs {
    const float *H;
    float lambda;
    const float *G;
    const uint8_t *codes;
    long n, p;
    int levels;
    long g;
    const float *scales;
    const int32_t *pairs;           // [cnt][npairs][2]: the group's batches
    int npairs, cnt;
    unsigned seq0;                  // sequence number of the group's first batch (>= 1, unique within the call)
    int group_seq;                  // how many groups must have been committed before this one
    unsigned long long *xch;        // [2][LS_FAST_PAIRS][chunks]: (sequence number << 32) | float bits, then
                                    // [2][chunks][LS_FAST_PAIRS][4][8]: (sequence number << 32) | the chosen sign
                                    // combinations of 8 columns (3 bits each: bit 0 = a move, bits 1-2 = which)
    const float *couple;            // [cnt - 1][LS_FAST_PAIRS][LS_FAST_PAIRS][4]: H' between the rows of pair a of
                                    // batch s + 1 and the rows of pair w of batch s (ls_couple_kernel)
    unsigned *fin;                  // [blocks]: group_seq + 1 once a block is through
    int *commit;                    // groups committed so far
    int *abort_word;
    long long spin_ticks;
    int32_t *pend_idx;              // out [2 cnt]
    float *pend_d;                  // out [2 cnt][p]
    int *moves;
    double *drop;
};

__device__ inline bool ls_wait_expired(long long t0, long long limit, const int *abort_word) {
    if (__hip_atomic_load(abort_word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) return true;
    return (long long)wall_clock64() - t0 > limit;
}

struct LsGroupLds {
    float pd[LS_K][2][LSG_TILE];                  // 32 KB: steps applied so far in this group, at my columns
    float tot[LS_FAST_PAIRS];                     // every candidate's summed gain
    int pairs_l[LS_K][LS_FAST_PAIRS][2];          //  8 KB: the group's batches
    float coef_own[LSG_PB_MAX][LS_K][4];          // H' between the own pairs and the rows of the applied slots
    int which_own[LSG_PB_MAX][LS_K];              // which rows of a slot are rows of the pair (4 bits)
    int prow[LS_K][2];                            // rows of the applied pairs, -1 = none
    float wsum[LSG_PB_MAX][4];
    unsigned combos[LS_FAST_PAIRS * 32];          //  8 KB: every candidate's sign combinations at my columns
    int bad;                                      // set by a thread whose wait ran out
};

// lane 0 of every 16-lane row: acc + v[lane 1] + v[lane 2] + ... + v[lane 15] of its row, added in that order
template <int N>
__device__ inline float row_lane(float v) {       // lane i <- lane i + N of the same row
    return __uint_as_float((unsigned)__builtin_amdgcn_update_dpp(0, (int)__float_as_uint(v), 0x100 + N, 0xF, 0xF, true));
}
__device__ inline float row_ordered_sum(float acc, float v, bool with_lane0) {
    if (with_lane0) acc += v;
    acc += row_lane<1>(v);  acc += row_lane<2>(v);  acc += row_lane<3>(v);  acc += row_lane<4>(v);
    acc += row_lane<5>(v);  acc += row_lane<6>(v);  acc += row_lane<7>(v);  acc += row_lane<8>(v);
    acc += row_lane<9>(v);  acc += row_lane<10>(v); acc += row_lane<11>(v); acc += row_lane<12>(v);
    acc += row_lane<13>(v); acc += row_lane<14>(v); acc += row_lane<15>(v);
    return acc;
}

// one pair at one column: the values read from memory, then brought up to date slot by slot.  Codes and diagonal
// entries stay as loaded (raw bytes, H without the damping) and what is done to them is kept beside them (dk, the
// damping added where the cell is evaluated): an operation on a loaded value at the place of the load would make
// the wave wait there for the whole trip to memory, which is what issuing the loads a step ahead is meant to hide.
struct LsCell {
    float g1, g2, sc1, sc2, h11, h22, h12;
    unsigned k1, k2;
    int dk1, dk2;
};

// vz: a zero the compiler cannot see through, in a vector register.  The three entries of H' have the same address
// in all lanes and would otherwise be fetched by the scalar unit, whose loads share a counter with the LDS: the
// next LDS read would then wait out their whole trip to memory.  As vector loads they are waited for where used.
__device__ inline void ls_cell_load(LsCell &c, const LsGroupArgs &a, int r1, int r2, long j, bool one_group,
                                    float sc_col, int vz) {
    const long i1 = r1, i2 = r2;
    const int g = (int)a.g;               // (rows and group size fit 32 bits: a 64-bit division per load would cost more
    c.g1 = a.G[i1 * a.p + j];             //  than the rest of the evaluation)
    c.g2 = a.G[i2 * a.p + j];
    c.k1 = a.codes[i1 * a.p + j];
    c.k2 = a.codes[i2 * a.p + j];
    if (one_group) {
        c.sc1 = c.sc2 = sc_col;
    } else {
        c.sc1 = a.scales[(long)(r1 / g) * a.p + j];
        c.sc2 = a.scales[(long)(r2 / g) * a.p + j];
    }
    c.h11 = a.H[i1 * a.n + i1 + vz];
    c.h22 = a.H[i2 * a.n + i2 + vz];
    c.h12 = a.H[i1 * a.n + i2 + vz];
}

// slot with steps (d1, d2) at this column, coefficients co = H'[i1][a], H'[i1][b], H'[i2][a], H'[i2][b] and row
// coincidences wh (bit 0: a == i1, 1: b == i1, 2: a == i2, 3: b == i2)
__device__ inline void ls_cell_apply(LsCell &c, const float *co, int wh, float d1, float d2) {
    pending_onto(c.g1, c.g2, co, d1, d2);
    // (a slot's rows are rows of this pair once in a few thousand slots, and for all lanes at once: a branch on
    // the scalar unit instead of a dozen vector instructions per slot)
    if (__builtin_amdgcn_readfirstlane(wh) != 0) {
        const int s1 = step_sign(d1), s2 = step_sign(d2);
        c.dk1 += ((wh & 1) ? s1 : 0) + ((wh & 2) ? s2 : 0);
        c.dk2 += ((wh & 4) ? s1 : 0) + ((wh & 8) ? s2 : 0);
    }
}

__device__ inline int ls_which(long pa, long pb, long i1, long i2) {
    return pa < 0 ? 0 : (int)((pa == i1) | ((pb == i1) << 1) | ((pa == i2) << 2) | ((pb == i2) << 3));
}

// the applied slots [0, count) onto a cell: coefficients and row coincidences from LDS (coef[k][4], which[k]; entries
// beyond the slots in use are zero), steps of this column from pd.  Four slots are read at a time before any is
// used, so that the LDS latency is paid once per four, not once per slot; the subtractions keep the slot order.
template <int NCELL>
__device__ inline void ls_apply_slots(LsCell *cells, const bool *on, const float (*const *coef)[4], const int *const *which,
                                      const float (*pd)[2][LSG_TILE], int col, int count) {
    constexpr int U = 4;
    for (int k0 = 0; k0 < count; k0 += U) {
        float d1[U], d2[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            d1[u] = pd[k0 + u][0][col];
            d2[u] = pd[k0 + u][1][col];
        }
#pragma unroll
        for (int i = 0; i < NCELL; ++i) {
            floatx4 c[U];
            int wh[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                c[u] = *(const floatx4 *)&coef[i][k0 + u][0];
                wh[u] = which[i][k0 + u];
            }
            if (on[i]) {
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const float co[4] = {c[u].x, c[u].y, c[u].z, c[u].w};
                    ls_cell_apply(cells[i], co, wh[u], d1[u], d2[u]);
                }
            }
        }
    }
}

// The coupling table of a run of batches: for every batch b of the run but the last,
//   X[b][a][w][k] = H'[row (k >> 1) of pair a of batch b + 1][row (k & 1) of pair w of batch b]
// (0 where a pair does not exist or is not a pair of two different rows of the matrix).  Whichever candidate of
// batch b wins, the entries that carry its move into the gradient rows of the next batch's candidates are then
// already there, 1 KB per next-batch pair, and no look-up of H' stands between a winner and the next evaluation.
// grid = batches of the run - 1, block 1024; pairs: [batches][npairs][2].
__global__ __launch_bounds__(1024) void ls_couple_kernel(const float *__restrict__ H, float lambda, long n,
                                                         const int32_t *__restrict__ pairs, int npairs,
                                                         float *__restrict__ X) {
    __shared__ int rows[2][LS_FAST_PAIRS][2];
    const int b = blockIdx.x, tid = threadIdx.x;
    if (tid < 4 * LS_FAST_PAIRS) {
        const int which = tid / (2 * LS_FAST_PAIRS), r = tid - which * 2 * LS_FAST_PAIRS, q = r >> 1;
        int v = -1;
        if (q < npairs) {
            const int32_t *pr = pairs + ((size_t)(b + which) * npairs + q) * 2;
            const int r1 = pr[0], r2 = pr[1];
            if (!(r1 < 0 || r2 < 0 || r1 >= n || r2 >= n || r1 == r2)) v = pr[r & 1];
        }
        rows[which][q][r & 1] = v;
    }
    __syncthreads();
    float *out = X + (size_t)b * (LS_FAST_PAIRS * LS_FAST_PAIRS * 4);
    for (int e = tid; e < LS_FAST_PAIRS * LS_FAST_PAIRS * 4; e += 1024) {
        const int a = e >> 8, w = (e >> 2) & (LS_FAST_PAIRS - 1), k = e & 3;
        const long row = rows[1][a][k >> 1], cr = rows[0][w][k & 1];
        float v = 0.f;
        if (row >= 0 && cr >= 0) v = H[row * n + cr] + (row == cr ? lambda : 0.f);
        out[e] = v;
    }
}

// the value lane `l` (the same in all lanes) holds, in every lane
__device__ inline float lane_value(float v, int l) {
    return __uint_as_float((unsigned)__builtin_amdgcn_readlane((int)__float_as_uint(v), l));
}

template <int PP>
__global__ __launch_bounds__(1024) void ls_group_kernel(LsGroupArgs a) {
    extern __shared__ __align__(16) unsigned char ls_group_lds[];
    LsGroupLds &L = *reinterpret_cast<LsGroupLds *>(ls_group_lds);
    if (*a.commit != a.group_seq) return;      // an earlier group did not complete; the host takes over from there
    // (the wave's index, the rows of its candidate pairs and everything derived from them are the same in all 64
    // lanes; taken through readfirstlane they live in scalar registers, and the address arithmetic on them - most
    // of the integer work of a step - goes to the scalar unit, which the block's sixteen waves do not queue for)
    const int tid = threadIdx.x, lane = tid & 63, wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int pl = wv >> 2, sub = wv & 3;                      // pair within the block, 64-column strip
    const int chunks = gridDim.x;
    const long n = a.n, p = a.p;
    const int col = sub * 64 + lane;
    const long j = (long)blockIdx.x * LSG_TILE + col;
    const bool in = j < p;
    const int npairs = a.npairs;
    constexpr int PB = 4 * PP;                                 // pairs per block
    const int q_base = (int)blockIdx.y * PB;                   // own pair i of this thread: q_base + 4 i + pl
    const int block_id = (int)(blockIdx.y * gridDim.x + blockIdx.x), nblocks = (int)(gridDim.x * gridDim.y);

    for (int e = tid; e < a.cnt * npairs * 2; e += 1024) {
        const int s = e / (2 * npairs), r = e - s * 2 * npairs;
        L.pairs_l[s][r >> 1][r & 1] = a.pairs[e];
    }
    // (zero steps, coefficients and coincidences for the slots not yet in use: the apply loops read whole fours)
    for (int e = tid; e < LS_K * 2 * LSG_TILE; e += 1024) (&L.pd[0][0][0])[e] = 0.f;
    for (int e = tid; e < LSG_PB_MAX * LS_K * 4; e += 1024) (&L.coef_own[0][0][0])[e] = 0.f;
    for (int e = tid; e < LSG_PB_MAX * LS_K; e += 1024) (&L.which_own[0][0])[e] = 0;
    if (tid < 2 * LS_K) (&L.prow[0][0])[tid] = -1;
    if (tid == 0) L.bad = 0;
    // A barrier that orders LDS traffic only.  __syncthreads() also waits for every global load and store the wave
    // has in flight - here the requests for the next batch and the words just published - which put a trip to
    // memory into every barrier of a step.  Global loads are waited for where their values are used, and the
    // published words validate themselves.
    auto lds_barrier = [&]() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); };
    int moves_l = 0;
    double drop_l = 0.0;
    if (tid == 0) {
        moves_l = *a.moves;
        drop_l = *a.drop;
    }
    __syncthreads();

    int vz;
    asm volatile("v_mov_b32 %0, 0" : "=v"(vz));
    // one grid per column: the step of every row is the column's, known from the start
    const bool one_group = a.g >= n;
    const float sc_col = (one_group && in) ? a.scales[j] : 0.f;
    LsCell own[PP], own_n[PP];             // the own pairs of the batch in hand, and of the next one (on their way)
    int i1[PP], i2[PP], i1n[PP], i2n[PP];
    bool has[PP], hasn[PP];
    auto load_cells = [&](int s, LsCell *cell, int *r1, int *r2, bool *ok) {
#pragma unroll
        for (int i = 0; i < PP; ++i) {
            const int q = q_base + 4 * i + pl;
            r1[i] = r2[i] = -1;
            if (q < npairs) {
                r1[i] = __builtin_amdgcn_readfirstlane(L.pairs_l[s][q][0]);
                r2[i] = __builtin_amdgcn_readfirstlane(L.pairs_l[s][q][1]);
            }
            const bool pair_ok = !(r1[i] < 0 || r2[i] < 0 || r1[i] >= n || r2[i] >= n || r1[i] == r2[i]);
            ok[i] = pair_ok && in;
            cell[i] = LsCell{0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0u, 0u, 0, 0};
            if (pair_ok) {
                if (in) ls_cell_load(cell[i], a, r1[i], r2[i], j, one_group, sc_col, vz);
            }
        }
    };
    const float (*coef_rows[PP])[4];
    const int *which_rows[PP];
#pragma unroll
    for (int i = 0; i < PP; ++i) {
        coef_rows[i] = L.coef_own[4 * i + pl];
        which_rows[i] = L.which_own[4 * i + pl];
    }

    load_cells(0, own, i1, i2, has);
    for (int s = 0; s <= a.cnt; ++s) {
        const bool nxt = s + 1 < a.cnt;
        float c_next = 0.f;                // one coefficient of the pairs of batch s+1 against the slots 0 .. s-1
        int c_pp = 0, c_k = 0, c_w = 0;
        bool c_on = false;
        if (s > 0) {
            // ---- the winner of batch s-1: everybody's sums, added in chunk order ---------------------------------------
            const unsigned seq = a.seq0 + (unsigned)(s - 1);
            const unsigned long long *tab = a.xch + (size_t)(seq & 1u) * LS_FAST_PAIRS * chunks;
            const unsigned long long *cmb = a.xch + (size_t)2 * LS_FAST_PAIRS * chunks +
                                            ((size_t)(seq & 1u) * chunks + blockIdx.x) * (LS_FAST_PAIRS * 32);
            // H' between the own pairs of batch s and every candidate of batch s-1 (a table of an earlier launch, so
            // an ordinary load): requested before the wait, there by the time the winner is known
            // (lane w of a wave holds the four entries of its pair against candidate w: the winner's are then one
            // lane's registers, read by all lanes without a pass through LDS)
            floatx4 xv[PP];
#pragma unroll
            for (int i = 0; i < PP; ++i) {
                xv[i] = floatx4{0.f, 0.f, 0.f, 0.f};
                const int q = q_base + 4 * i + pl;
                if (s < a.cnt && q < npairs)
                    xv[i] = *(const floatx4 *)(a.couple + ((size_t)(s - 1) * LS_FAST_PAIRS + q) * (LS_FAST_PAIRS * 4) + 4 * lane);
            }
            bool bad = a.spin_ticks < 0;          // a negative bound makes every block leave at its first wait
            {
                // sixteen lanes to a candidate: lane c of the row reads the sums of the chunks c and c + 16; chunks
                // beyond the last count as zero (so does a candidate beyond the last, whose total stays zero).  Every
                // thread also fetches two words of the candidates' sign combinations at this block's columns.
                const int q = tid >> 4, c0 = tid & 15;
                const unsigned long long *src[4] = {tab + (size_t)q * chunks + c0, tab + (size_t)q * chunks + c0 + 16,
                                                    cmb + tid, cmb + tid + 1024};
                const bool need[4] = {q < npairs && c0 < chunks, q < npairs && c0 + 16 < chunks, (tid >> 5) < npairs,
                                      ((tid + 1024) >> 5) < npairs};
                unsigned long long w[4] = {0ull, 0ull, 0ull, 0ull};
                if (!bad) {
                    const long long t0 = (long long)wall_clock64();
#pragma unroll
                    for (int h = 0; h < 4; ++h)
                        if (need[h]) w[h] = __hip_atomic_load(src[h], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
                    for (int h = 0; h < 4; ++h) {
                        if (!need[h] || bad) continue;
                        unsigned it = 0;
                        while ((unsigned)(w[h] >> 32) != seq) {
                            if ((it++ & 7u) == 0u && ls_wait_expired(t0, a.spin_ticks, a.abort_word)) {
                                bad = true;
                                break;
                            }
                            w[h] = __hip_atomic_load(src[h], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        }
                    }
                }
                const float v0 = need[0] && !bad ? __uint_as_float((unsigned)w[0]) : 0.f;
                const float v1 = need[1] && !bad ? __uint_as_float((unsigned)w[1]) : 0.f;
                // 0 + chunk 0 + chunk 1 + ... in index order, as the launch-per-batch kernel adds them
                float tot = row_ordered_sum(0.f, v0, true);
                if (chunks > 16) tot = row_ordered_sum(tot, v1, true);
                if (c0 == 0) L.tot[q] = tot;
                L.combos[tid] = need[2] ? (unsigned)w[2] : 0u;
                L.combos[tid + 1024] = need[3] ? (unsigned)w[3] : 0u;
            }
            if (bad) L.bad = 1;
            lds_barrier();
            if (L.bad) {
                if (tid == 0) __hip_atomic_store(a.abort_word, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                return;
            }
            // every wave finds the winner for itself: lane = candidate
            int win;
            float win_tot;
            {
                const unsigned long long key = wave_max_key(lane < npairs ? best_key(L.tot[lane], lane) : 0ull);
                const unsigned klo = __builtin_amdgcn_readfirstlane((unsigned)key);
                const unsigned khi = __builtin_amdgcn_readfirstlane((unsigned)(key >> 32));
                win = (klo | khi) ? (int)(0xFFFFFFFFu - klo) : -1;
                win_tot = __uint_as_float(khi);
            }
            const int wi1 = win >= 0 ? __builtin_amdgcn_readfirstlane(L.pairs_l[s - 1][win][0]) : -1;
            const int wi2 = win >= 0 ? __builtin_amdgcn_readfirstlane(L.pairs_l[s - 1][win][1]) : -1;
            if (tid == 0) {
                L.prow[s - 1][0] = wi1;
                L.prow[s - 1][1] = wi2;
                if (win >= 0) {
                    moves_l += 1;
                    drop_l += (double)win_tot;
                }
            }
            // ---- the winner's steps at my column: the sign combination its own block's evaluation chose (the same
            // bits a second evaluation from the same inputs would give), times the step of each row's group ----------
            float wsc1 = sc_col, wsc2 = sc_col;
            if (win >= 0 && in && !one_group) {
                const int g = (int)a.g;
                wsc1 = a.scales[(long)(wi1 / g) * p + j];
                wsc2 = a.scales[(long)(wi2 / g) * p + j];
            }
            // everything for batch s+1 (used after batch s has been evaluated and published)
            if (nxt) {
                load_cells(s + 1, own_n, i1n, i2n, hasn);
                if (tid >= 128 && tid < 128 + PB * 64 && ((tid >> 2) & 15) < s) {     // slots 0 .. s-1 of each own pair
                    const int e = tid - 128;
                    c_pp = e >> 6;
                    c_k = (e >> 2) & 15;
                    c_w = e & 3;
                    c_on = true;
                    const int q = q_base + c_pp;
                    const long src = c_k == s - 1 ? (c_w & 1 ? wi2 : wi1) : (long)L.prow[c_k][c_w & 1];
                    if (q < npairs && src >= 0) {
                        const long row = L.pairs_l[s + 1][q][c_w >> 1];
                        if (row >= 0 && row < n) c_next = a.H[src * n + row] + (row == src ? a.lambda : 0.f);
                    }
                }
            }
            if (win >= 0) {
                float st1 = 0.f, st2 = 0.f;
                const unsigned code = (L.combos[(win * 4 + sub) * 8 + (lane >> 3)] >> (3 * (lane & 7))) & 7u;
                if (in && (code & 1u)) {
                    st1 = (code & 4u) ? -wsc1 : wsc1;
                    st2 = (code & 2u) ? -wsc2 : wsc2;
                }
                if (pl == 0) {              // kept for the batches after the next (read behind a later barrier)
                    L.pd[s - 1][0][col] = st1;
                    L.pd[s - 1][1][col] = st2;
                }
#pragma unroll
                for (int i = 0; i < PP; ++i) {
                    const float eo[4] = {lane_value(xv[i].x, win), lane_value(xv[i].y, win), lane_value(xv[i].z, win),
                                         lane_value(xv[i].w, win)};
                    if (has[i] && s < a.cnt) ls_cell_apply(own[i], eo, ls_which(wi1, wi2, i1[i], i2[i]), st1, st2);
                }
            }
            if (s == a.cnt) break;
        } else if (nxt) {
            load_cells(1, own_n, i1n, i2n, hasn);
        }
        // ---- evaluate the own pairs of batch s and publish the block's 256-column sums ---------------------------------
        {
#pragma unroll
            for (int i = 0; i < PP; ++i) {
                float gain = 0.f;
                unsigned code = 0u;
                if (has[i]) {
                    const PairEval ev = eval_column(own[i].g1, own[i].g2, (int)(own[i].k1 & 0xFFu) + own[i].dk1,
                                                    (int)(own[i].k2 & 0xFFu) + own[i].dk2, own[i].sc1, own[i].sc2,
                                                    own[i].h11 + a.lambda, own[i].h22 + a.lambda, own[i].h12, a.levels);
                    gain = ev.gain;
                    if (ev.combo >= 0) code = 1u | ((unsigned)ev.combo << 1);
                }
                // the chosen combinations of 8 neighbouring columns in one word, published with the batch's number
                const int q = q_base + 4 * i + pl;
                unsigned bits = code << (3 * (lane & 7));
                bits |= (unsigned)__builtin_amdgcn_update_dpp(0, (int)bits, 0xB1, 0xF, 0xF, true);     // lanes ^ 1
                bits |= (unsigned)__builtin_amdgcn_update_dpp(0, (int)bits, 0x4E, 0xF, 0xF, true);     // lanes ^ 2
                bits |= (unsigned)__builtin_amdgcn_update_dpp(0, (int)bits, 0x141, 0xF, 0xF, true);    // 7 - lane
                if ((lane & 7) == 0 && q < npairs) {
                    const unsigned sq = a.seq0 + (unsigned)s;
                    unsigned long long *dst = a.xch + (size_t)2 * LS_FAST_PAIRS * chunks +
                                              ((size_t)(sq & 1u) * chunks + blockIdx.x) * (LS_FAST_PAIRS * 32) +
                                              ((size_t)q * 4 + sub) * 8 + (lane >> 3);
                    __hip_atomic_store(dst, ((unsigned long long)sq << 32) | (unsigned long long)bits, __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_AGENT);
                }
                gain = wave_sum_f(gain);
                if (lane == 0) L.wsum[4 * i + pl][sub] = gain;
            }
            lds_barrier();
            if (tid < PB && q_base + tid < npairs) {
                const unsigned seq = a.seq0 + (unsigned)s;
                unsigned long long *tab = a.xch + (size_t)(seq & 1u) * LS_FAST_PAIRS * chunks;
                const float tot = (L.wsum[tid][0] + L.wsum[tid][1]) + (L.wsum[tid][2] + L.wsum[tid][3]);
                __hip_atomic_store(tab + (size_t)(q_base + tid) * chunks + blockIdx.x,
                                   ((unsigned long long)seq << 32) | (unsigned long long)__float_as_uint(tot),
                                   __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
        // ---- the pairs of batch s+1 have arrived: bring them up to date with the slots 0 .. s-1 ------------------------
        if (nxt) {
#pragma unroll
            for (int i = 0; i < PP; ++i) {
                own[i] = own_n[i];
                i1[i] = i1n[i];
                i2[i] = i2n[i];
                has[i] = hasn[i];
            }
            if (c_on) L.coef_own[c_pp][c_k][c_w] = c_next;
            if (tid < PB * 16 && (tid & 15) < s) {
                const int pp = tid >> 4, k = tid & 15, q = q_base + pp;
                L.which_own[pp][k] = q < npairs ? ls_which(L.prow[k][0], L.prow[k][1], L.pairs_l[s + 1][q][0], L.pairs_l[s + 1][q][1]) : 0;
            }
            lds_barrier();
            ls_apply_slots<PP>(own, has, coef_rows, which_rows, L.pd, col, s);
        }
    }

    // ---- hand the group's moves to the flush -------------------------------------------------------------------------
    if (blockIdx.y == 0) {
        for (int e = tid; e < a.cnt * 2 * LSG_TILE; e += 1024) {
            const int kw = e / LSG_TILE, c = e - kw * LSG_TILE;
            const long jj = (long)blockIdx.x * LSG_TILE + c;
            if (jj < p) a.pend_d[(long)kw * p + jj] = (&L.pd[0][0][0])[e];
        }
        if (blockIdx.x == 0 && tid < 2 * a.cnt) a.pend_idx[tid] = (&L.prow[0][0])[tid];
    }
    // (what the blocks have written is read by later launches only, so no ordering is needed inside this one: the
    // words below just tell block 0 that nobody gave up)
    if (tid == 0)
        __hip_atomic_store(a.fin + block_id, (unsigned)(a.group_seq + 1), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (block_id != 0) return;
    // block 0 commits the group once every block is through
    bool bad = false;
    {
        const long long t0 = (long long)wall_clock64();
        for (int b = tid; b < nblocks && !bad; b += 1024) {
            unsigned it = 0;
            while (__hip_atomic_load(a.fin + b, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != (unsigned)(a.group_seq + 1)) {
                if ((it++ & 7u) == 0u && ls_wait_expired(t0, a.spin_ticks, a.abort_word)) {
                    bad = true;
                    break;
                }
            }
        }
    }
    if (__syncthreads_or(bad ? 1 : 0)) {
        if (tid == 0) __hip_atomic_store(a.abort_word, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return;
    }
    if (tid == 0) {
        *a.moves = moves_l;
        *a.drop = drop_l;
        *a.commit = a.group_seq + 1;
    }
}

// grid (ceil(p/1024), ceil(n/8)), block 256: each thread 4 columns x 8 rows; applies `count` slots
__global__ __launch_bounds__(256) void ls_flush_kernel(const float *__restrict__ H, float lambda,
                                                       float *__restrict__ G, uint8_t *__restrict__ codes, long n,
                                                       long p,
                                                       const int32_t *__restrict__ pend_idx,
                                                       const float *__restrict__ pend_d, int count,
                                                       const int *__restrict__ commit, int commit_needed) {
    // after a group kernel: apply its moves only if the group was committed
    if (commit && *commit != commit_needed) return;
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
        // the block that owns a pending row brings its stored codes up to date (one owner per row and
        // column, slots in order: a row may sit in several slots)
        const long a = pend_idx[2 * k], b = pend_idx[2 * k + 1];
        if (a >= r0 && a < r0 + 8) {
#pragma unroll
            for (int c = 0; c < 4; ++c)
                if (j0 + c < p && d1[c] != 0.f) codes[a * p + j0 + c] = (uint8_t)((int)codes[a * p + j0 + c] + step_sign(d1[c]));
        }
        if (b >= r0 && b < r0 + 8) {
#pragma unroll
            for (int c = 0; c < 4; ++c)
                if (j0 + c < p && d2[c] != 0.f) codes[b * p + j0 + c] = (uint8_t)((int)codes[b * p + j0 + c] + step_sign(d2[c]));
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

// The same pass for rows of whole 16-byte pieces (p a multiple of 4), organised around what is re-read: a thread
// keeps the steps of all slots at its four columns in registers (2 K x 4 values) and walks 32 rows of G with them,
// so the pending step rows come through the caches once per 32 rows of G instead of once per 8; the rows'
// coefficients sit in LDS (every lane reads the same word), the next eight rows of G are on their way while eight are
// worked on, and each slot enters a sum by two fused multiply-adds in slot order.
// grid (ceil(p/1024), ceil(n/LSF_ROWS)), block 256; LSF_ROWS = 32, or 16 or 8 where 32 would leave the chip short of
// blocks (narrow matrices).
template <int LSF_ROWS>
__global__ __launch_bounds__(256, 2) void ls_flush_rows_kernel(const float *__restrict__ H, float lambda,
                                                               float *__restrict__ G, uint8_t *__restrict__ codes,
                                                               long n, long p, const int32_t *__restrict__ pend_idx,
                                                               const float *__restrict__ pend_d, int count,
                                                               const int *__restrict__ commit, int commit_needed) {
    typedef floatx4 vec;
    constexpr int CPT = 4;                               // columns per thread
    if (commit && *commit != commit_needed) return;
    constexpr int R = LSF_ROWS, S2 = 2 * LS_K;
    __shared__ __align__(16) float coef[R][S2];          // coef[rr][2 k + w] = H'[r0 + rr][row w of slot k], 0 for an empty slot
    __shared__ int any_sh;
    const int tid = threadIdx.x;
    const long r0 = (long)blockIdx.y * R;
    const long j0 = ((long)blockIdx.x * 256 + tid) * CPT;
    if (tid == 0) any_sh = 0;
    __syncthreads();
    for (int e = tid; e < R * S2; e += 256) {
        const int kw = e / R, rr = e - kw * R, k = kw >> 1;          // neighbouring threads: neighbouring entries of a row of H'
        const long i = r0 + rr;
        float h = 0.f;
        if (k < count && pend_idx[2 * k] >= 0 && i < n) {
            const long src = pend_idx[kw];
            h = H[src * n + i];
            if (i == src) h += lambda;
            any_sh = 1;
        }
        coef[rr][kw] = h;
    }
    const bool cols = j0 < p;
    vec zero;
#pragma unroll
    for (int c = 0; c < CPT; ++c) zero[c] = 0.f;
    vec d[S2];
#pragma unroll
    for (int kw = 0; kw < S2; ++kw) {
        d[kw] = zero;
        if (cols && (kw >> 1) < count) d[kw] = *(const vec *)(pend_d + (long)kw * p + j0);
    }
    // (the first rows of G are asked for before the barrier: they travel while the coefficients are gathered)
    constexpr int PF = 8;
    vec g[2][PF];
#pragma unroll
    for (int u = 0; u < PF; ++u) g[0][u] = (cols && r0 + u < n) ? *(const vec *)(G + (r0 + u) * p + j0) : zero;
    __syncthreads();
    if (any_sh == 0 || !cols) return;
    // the block that owns a pending row brings its stored codes up to date (one owner per row and column, slots in
    // order: a row may sit in several slots)
    for (int k = 0; k < count; ++k) {
        const long a = pend_idx[2 * k], b = pend_idx[2 * k + 1];
        if (a < 0) continue;
#pragma unroll
        for (int w = 0; w < 2; ++w) {
            const long row = w ? b : a;
            if (row >= r0 && row < r0 + R) {
                vec dv = d[0];
#pragma unroll
                for (int kk = 0; kk < LS_K; ++kk)
                    if (kk == k) dv = d[2 * kk + w];                  // (register array: selected, not indexed)
#pragma unroll
                for (int c = 0; c < CPT; ++c)
                    if (dv[c] != 0.f) codes[row * p + j0 + c] = (uint8_t)((int)codes[row * p + j0 + c] + step_sign(dv[c]));
            }
        }
    }
#pragma unroll
    for (int c8 = 0; c8 < R / PF; ++c8) {
        const int cur = c8 & 1;
        if (c8 + 1 < R / PF) {
#pragma unroll
            for (int u = 0; u < PF; ++u) {
                const long i = r0 + (c8 + 1) * PF + u;
                g[cur ^ 1][u] = i < n ? *(const vec *)(G + i * p + j0) : zero;
            }
        }
#pragma unroll
        for (int u = 0; u < PF; ++u) {
            const int rr = c8 * PF + u;
            const long i = r0 + rr;
            if (i >= n) break;
            vec acc = zero;
#pragma unroll
            for (int q4 = 0; q4 < S2 / 4; ++q4) {
                const floatx4 cf = *(const floatx4 *)&coef[rr][4 * q4];
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const vec dv = d[4 * q4 + t];
#pragma unroll
                    for (int c = 0; c < CPT; ++c) acc[c] = __fmaf_rn(cf[t], dv[c], acc[c]);
                }
            }
            vec gq = g[cur][u];
#pragma unroll
            for (int c = 0; c < CPT; ++c) gq[c] -= acc[c];
            *(vec *)(G + i * p + j0) = gq;
        }
    }
}

}  // namespace

int admmq_ls_chunks(int64_t p) { return (int)((p + LS_CHUNK - 1) / LS_CHUNK); }
int admmq_ls_defer() { return LS_K; }
int admmq_ls_fast_pairs() { return LS_FAST_PAIRS; }

// One step: plan the previous batch (if npairs_prev > 0) into pending slot slot_prev, and evaluate the current
// batch (if pairs_cur) against the state after that move.  npend = pending slots already in memory, i.e. slots
// 0 .. npend-1 hold earlier moves of the current group (npend == slot_prev whenever there is a previous batch).
// mv_prev / mv_cur: [npairs][p] bytes, the sign combination each evaluation chose; hcol: [2 K][n] floats.
admmq_status admmq_k_ls_step(admmq_ctx *ctx, const float *H, float lambda, const float *G, const uint8_t *codes,
                             int64_t n, int64_t p, int bits, int64_t g, const float *scales,
                             const int32_t *pairs_prev, int npairs_prev, const float *partial_prev,
                             const uint8_t *mv_prev, int slot_prev, const int32_t *pairs_cur, int npairs_cur,
                             int npend, int32_t *pend_idx, float *pend_d, float *hcol, float *partial_cur,
                             uint8_t *mv_cur, int32_t *choice, int *dev_moves, double *dev_drop,
                             const int32_t *pairs_next, int npairs_next, const float *exs_cur, float *exs_next) {
    const int chunks = admmq_ls_chunks(p);
    const int levels = (1 << bits) - 1;
    const unsigned gy = (unsigned)(pairs_cur ? npairs_cur : 1);
    hipLaunchKernelGGL(ls_step_kernel, dim3((unsigned)chunks, gy), dim3(256), 0, ctx->stream, H, lambda, G, codes,
                       (long)n, (long)p, levels, (long)g, scales, pairs_prev, npairs_prev, partial_prev, mv_prev,
                       slot_prev, pairs_cur, npend, pend_idx, pend_d, hcol, partial_cur, mv_cur, chunks, choice,
                       dev_moves, dev_drop, pairs_next, npairs_next, exs_cur, exs_next);
    ADMMQ_HIP(hipGetLastError());
    return ADMMQ_OK;
}

admmq_status admmq_k_ls_flush(admmq_ctx *ctx, const float *H, float lambda, float *G, uint8_t *codes, int64_t n,
                              int64_t p, const int32_t *pend_idx, const float *pend_d, int count, const int *commit,
                              int commit_needed) {
    if (count <= 0) return ADMMQ_OK;
    const int sp = admmq_prof_begin(ctx, ADMMQ_TAG_LS_APPLY);
    if (p % 4 == 0) {
        // 32 rows per block where that still gives two blocks per compute unit, else 16, else 8
        const long cb = (p + 1023) / 1024;
        const int R = cb * ((n + 31) / 32) >= 512 ? 32 : (cb * ((n + 15) / 16) >= 512 ? 16 : 8);
        dim3 grid((unsigned)cb, (unsigned)((n + R - 1) / R));
        if (R == 32)
            hipLaunchKernelGGL(ls_flush_rows_kernel<32>, grid, dim3(256), 0, ctx->stream, H, lambda, G, codes, (long)n,
                               (long)p, pend_idx, pend_d, count, commit, commit_needed);
        else if (R == 16)
            hipLaunchKernelGGL(ls_flush_rows_kernel<16>, grid, dim3(256), 0, ctx->stream, H, lambda, G, codes, (long)n,
                               (long)p, pend_idx, pend_d, count, commit, commit_needed);
        else
            hipLaunchKernelGGL(ls_flush_rows_kernel<8>, grid, dim3(256), 0, ctx->stream, H, lambda, G, codes, (long)n,
                               (long)p, pend_idx, pend_d, count, commit, commit_needed);
    } else {
        dim3 grid((unsigned)((p + 1023) / 1024), (unsigned)((n + 7) / 8));
        hipLaunchKernelGGL(ls_flush_kernel, grid, dim3(256), 0, ctx->stream, H, lambda, G, codes, (long)n, (long)p,
                           pend_idx, pend_d, count, commit, commit_needed);
    }
    admmq_prof_end(ctx, sp);
    ADMMQ_HIP(hipGetLastError());
    return ADMMQ_OK;
}

// How a search of this shape runs its groups as single launches: candidate pairs per thread (1 or 2: the fewer
// for which all blocks are on the chip at once - blocks wait for one another), or 0 if it cannot.
static int ls_group_chunks(int64_t p) { return (int)((p + LSG_TILE - 1) / LSG_TILE); }
template <int PP>
static int ls_group_resident_blocks(int device) {
    static int cached[64];
    int &slot = cached[device & 63];
    if (slot == 0) {
        int per_cu = 0, cus = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, ls_group_kernel<PP>, 1024, sizeof(LsGroupLds)) != hipSuccess ||
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess) {
            (void)hipGetLastError();
            per_cu = 0;
        }
        slot = per_cu > 0 && cus > 0 ? per_cu * cus : -1;
    }
    return slot > 0 ? slot : 0;
}
int admmq_ls_group_pairs_per_thread(admmq_ctx *ctx, int64_t p, int npairs) {
    if (npairs < 1 || npairs > LS_FAST_PAIRS || ls_group_chunks(p) > LSG_MAX_CHUNKS) return 0;
    static unsigned long long lds_done[2] = {0, 0};
    const int chunks = ls_group_chunks(p);
    if (admmq_allow_lds((const void *)ls_group_kernel<1>, (int)sizeof(LsGroupLds), ctx->device, &lds_done[0]) != hipSuccess ||
        admmq_allow_lds((const void *)ls_group_kernel<2>, (int)sizeof(LsGroupLds), ctx->device, &lds_done[1]) != hipSuccess) {
        (void)hipGetLastError();
        return 0;
    }
    const int share = ctx->ls_side_by_side > 1 ? ctx->ls_side_by_side : 1;
    if (chunks * ((npairs + 3) / 4) * share <= ls_group_resident_blocks<1>(ctx->device)) return 1;
    if (chunks * ((npairs + 7) / 8) * share <= ls_group_resident_blocks<2>(ctx->device)) return 2;
    return 0;
}
int admmq_ls_group_max_blocks(int64_t p) { return ls_group_chunks(p) * (LS_FAST_PAIRS / 4); }
size_t admmq_ls_group_xch_words(int64_t p) { return 2 * (size_t)LS_FAST_PAIRS * ls_group_chunks(p) * (1 + 32); }

// One group of `cnt` <= LS_K batches (pairs: device [cnt][npairs][2]) as one launch; see ls_group_kernel.
// pairs_per_thread: from admmq_ls_group_pairs_per_thread.  couple: the coupling table of the group's batches
// (admmq_k_ls_couple on the same pairs).  xch: admmq_ls_group_xch_words(p) 8-byte words, fin: one
// 4-byte word per block, commit, abort_word: 4-byte words, all zero at the start of a search.
admmq_status admmq_k_ls_couple(admmq_ctx *ctx, const float *H, float lambda, int64_t n, const int32_t *pairs,
                               int npairs, int batches, float *X) {
    if (batches < 2) return ADMMQ_OK;
    if (npairs < 1 || npairs > LS_FAST_PAIRS) return ADMMQ_ERR_PARAM;
    hipLaunchKernelGGL(ls_couple_kernel, dim3((unsigned)(batches - 1)), dim3(1024), 0, ctx->stream, H, lambda, (long)n,
                       pairs, npairs, X);
    ADMMQ_HIP(hipGetLastError());
    return ADMMQ_OK;
}
size_t admmq_ls_couple_floats(int batches) {
    return batches > 1 ? (size_t)(batches - 1) * LS_FAST_PAIRS * LS_FAST_PAIRS * 4 : 0;
}

admmq_status admmq_k_ls_group(admmq_ctx *ctx, int pairs_per_thread, const float *H, float lambda, const float *G,
                              const uint8_t *codes, int64_t n, int64_t p, int bits, int64_t g, const float *scales,
                              const int32_t *pairs, int npairs, int cnt, unsigned seq0, int group_seq,
                              unsigned long long *xch, unsigned *fin, int *commit, int *abort_word,
                              long long spin_ticks, int32_t *pend_idx, float *pend_d, int *dev_moves,
                              double *dev_drop, const float *couple) {
    LsGroupArgs a;
    a.couple = couple;
    a.H = H; a.lambda = lambda; a.G = G; a.codes = codes; a.n = (long)n; a.p = (long)p;
    a.levels = (1 << bits) - 1; a.g = (long)g; a.scales = scales; a.pairs = pairs; a.npairs = npairs; a.cnt = cnt;
    a.seq0 = seq0; a.group_seq = group_seq; a.xch = xch; a.fin = fin; a.commit = commit; a.abort_word = abort_word;
    a.spin_ticks = spin_ticks; a.pend_idx = pend_idx; a.pend_d = pend_d; a.moves = dev_moves; a.drop = dev_drop;
    const int pb = 4 * pairs_per_thread;
    const dim3 grid((unsigned)ls_group_chunks(p), (unsigned)((npairs + pb - 1) / pb));
    if (pairs_per_thread == 1)
        hipLaunchKernelGGL(ls_group_kernel<1>, grid, dim3(1024), sizeof(LsGroupLds), ctx->stream, a);
    else if (pairs_per_thread == 2)
        hipLaunchKernelGGL(ls_group_kernel<2>, grid, dim3(1024), sizeof(LsGroupLds), ctx->stream, a);
    else
        return ADMMQ_ERR_PARAM;
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
