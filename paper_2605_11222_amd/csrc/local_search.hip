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

// stored gradient entries and codes of a row pair at one column -> those of the CURRENT codes: the pending
// moves are added (codes and G are both brought up to date by the flush)
__device__ inline void apply_pending(const PendCol &pc, int npend, const float (*coef)[4], const int *which,
                                     float &g1, float &g2, int &k1, int &k2) {
#pragma unroll
    for (int k = 0; k < LS_K; ++k) {
        if (k < npend) {
            g1 -= coef[k][0] * pc.d1[k] + coef[k][1] * pc.d2[k];
            g2 -= coef[k][2] * pc.d1[k] + coef[k][3] * pc.d2[k];
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
            og1 -= ex[0] * nd1 + ex[1] * nd2;
            og2 -= ex[2] * nd1 + ex[3] * nd2;
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

// grid (ceil(p/1024), ceil(n/8)), block 256: each thread 4 columns x 8 rows; applies `count` slots
__global__ __launch_bounds__(256) void ls_flush_kernel(const float *__restrict__ H, float lambda,
                                                       float *__restrict__ G, uint8_t *__restrict__ codes, long n,
                                                       long p,
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
                              int64_t p, const int32_t *pend_idx, const float *pend_d, int count) {
    if (count <= 0) return ADMMQ_OK;
    dim3 grid((unsigned)((p + 1023) / 1024), (unsigned)((n + 7) / 8));
    const int sp = admmq_prof_begin(ctx, ADMMQ_TAG_LS_APPLY);
    hipLaunchKernelGGL(ls_flush_kernel, grid, dim3(256), 0, ctx->stream, H, lambda, G, codes, (long)n, (long)p,
                       pend_idx, pend_d, count);
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
