// fp32 matrix-core GEMM family for gfx950:  out = alpha * A^T B + beta * Z.
//
// Both operands are k-major ([K][M] and [K][N], consecutive m / n contiguous), which is the natural
// layout of every dense contraction on the ADMM-Q path:
//   Hessian (Sec. 3.1)      H += X^T X             A = B = X [rows][n]
//   W-update (eq. 7)        Y = Q^T R, W = B + Q S  A = Q resp. Q^T stored row-major
//   gradient (Sec. 3.5)     G = H' (W0 - Wq)        A = H (symmetric)
// Tiles of A and B for KT consecutive k are staged through LDS (double buffered, register
// prefetch of the next tile while the current one is consumed); each 64-lane wave owns a
// (32*FA) x (32*FB) block of the output as FA*FB accumulators of v_mfma_f32_32x32x2_f32.
// Lane l of the wave feeds matrix row  FA*(l%32)+a  and column  FB*(l%32)+b  of its block, so one
// LDS read of FA (FB) consecutive floats serves all FA (FB) accumulators and the epilogue writes
// FB consecutive outputs per lane.
#include <stdlib.h>

#include "common.h"

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx2 __attribute__((ext_vector_type(2)));

namespace {


struct GemmParams {
    const void *A;
    const void *B;
    long lda, ldb;
    long M, N, K;
    float alpha, beta;
    const float *Z;
    long ldz;
    float *out;
    long ldo;
    int tiles_m, tiles_n;
    int lower_only;
    int split_k;
    long k_chunk;
    long slice_stride;
    int vec_ok;     // 1: all rows 16-byte aligned and M, N multiples of 4 (vector global access)
    // projection epilogue (eqs. 8-10), PROJ instantiations only
    float *pV;
    long ldv;
    const float *pd, *pinv_d, *pscales, *pinv_scales, *pzeros;
    long ld_grid;
    int g_shift;
    float levels, rho, inv_rho, inv_rho_next;
    double *res_sq;
};

__device__ inline float bf16_to_f32(unsigned short b) { return __uint_as_float(((unsigned)b) << 16); }

// Loads 4 consecutive elements of row k starting at column c (zero outside [0,cols) x [0,K)).
template <bool BF16>
__device__ inline floatx4 load4(const void *base, long ld, long k, long kend, long c, long cols, bool vec_ok) {
    floatx4 r = {0.f, 0.f, 0.f, 0.f};
    if (k >= kend) return r;
    if (BF16) {
        const unsigned short *row = (const unsigned short *)base + k * ld;
        if (vec_ok && c + 3 < cols) {
            uint2 u = *(const uint2 *)(row + c);
            r.x = __uint_as_float(u.x << 16);
            r.y = __uint_as_float(u.x & 0xFFFF0000u);
            r.z = __uint_as_float(u.y << 16);
            r.w = __uint_as_float(u.y & 0xFFFF0000u);
        } else {
            if (c + 0 < cols) r.x = bf16_to_f32(row[c + 0]);
            if (c + 1 < cols) r.y = bf16_to_f32(row[c + 1]);
            if (c + 2 < cols) r.z = bf16_to_f32(row[c + 2]);
            if (c + 3 < cols) r.w = bf16_to_f32(row[c + 3]);
        }
    } else {
        const float *row = (const float *)base + k * ld;
        if (vec_ok && c + 3 < cols) {
            r = *(const floatx4 *)(row + c);
        } else {
            if (c + 0 < cols) r.x = row[c + 0];
            if (c + 1 < cols) r.y = row[c + 1];
            if (c + 2 < cols) r.z = row[c + 2];
            if (c + 3 < cols) r.w = row[c + 3];
        }
    }
    return r;
}

// Maps a linear block id to a tile so that (i) the blocks one XCD receives (ids congruent mod 8)
// form a compact patch of the tile grid and share operand panels in that XCD's L2, and (ii) inside
// the patch consecutive blocks walk down short columns of GROUP tiles.
__device__ inline void tile_of_block(int bid, int nblocks, int tiles_m, int tiles_n, int &tm, int &tn) {
    int pid = bid;
    if ((nblocks & 7) == 0) pid = (bid & 7) * (nblocks >> 3) + (bid >> 3);
    const int GROUP = 4;
    int per_group = GROUP * tiles_n;
    int grp = pid / per_group;
    int first_m = grp * GROUP;
    int gsz = min(tiles_m - first_m, GROUP);
    int in_grp = pid - grp * per_group;
    tm = first_m + in_grp % gsz;
    tn = in_grp / gsz;
}

// DIR: every tile is interior, rows are 16-byte aligned and every k-stage is whole (the launcher checks), fp32
// operands: stages are filled by direct global -> LDS loads.  One path per instantiation on purpose: with both
// in one loop the compiler joins them with register copies that wait for every outstanding load.
template <int FA, int FB, int WGM, int WGN, int KT, bool ABF16, bool BBF16, bool DIR, bool PROJ = false>
__global__ __launch_bounds__(64 * WGM * WGN, (WGM * WGN == 4 && FA * FB == 8) ? 2 : 1) void gemm_tn_kernel(GemmParams P) {
    static_assert(!DIR || (ABF16 == BBF16), "direct loads: both operands fp32, or both bf16 (kept as bf16 in LDS)");
    static_assert(!PROJ || (DIR && !ABF16), "the projection epilogue belongs to the direct fp32 path");
    // bf16 operands of the direct path stay bf16 in LDS (half the bytes through the load path and the LDS) and
    // are widened when a fragment is read: two shifts / masks per pair, issued in the shadow of the MFMAs
    constexpr bool LB = DIR && ABF16 && BBF16;
    constexpr int BM = 32 * FA * WGM;
    constexpr int BN = 32 * FB * WGN;
    constexpr int NT = 64 * WGM * WGN;
    constexpr int A4 = KT * BM / 4;            // float4 slots in an A stage
    constexpr int B4 = KT * BN / 4;
    constexpr int A_PER = (A4 + NT - 1) / NT;  // float4 loads per thread
    constexpr int B_PER = (B4 + NT - 1) / NT;
    extern __shared__ float lds[];
    float *sA = lds;                      // [2][KT][BM]
    float *sB = lds + 2 * KT * BM;        // [2][KT][BN]
    unsigned short *hA = (unsigned short *)lds;       // the same two arrays as bf16 bit patterns (LB)
    unsigned short *hB = hA + 2 * KT * BM;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave % WGM;
    const int wn = wave / WGM;

    int tile_id = blockIdx.x;
    int slice = 0;
    const int tiles_total = (int)(gridDim.x / P.split_k);
    if (P.split_k > 1) {
        slice = tile_id / tiles_total;
        tile_id -= slice * tiles_total;
    }
    int tm, tn;
    if (P.lower_only) {
        // tile_id enumerates pairs tm >= tn row by row of the triangle: id = tm(tm+1)/2 + tn
        tm = (int)((sqrtf(8.f * (float)tile_id + 1.f) - 1.f) * 0.5f);
        while ((long)(tm + 1) * (tm + 2) / 2 <= tile_id) ++tm;
        while ((long)tm * (tm + 1) / 2 > tile_id) --tm;
        tn = tile_id - tm * (tm + 1) / 2;
    } else {
        tile_of_block(tile_id, tiles_total, P.tiles_m, P.tiles_n, tm, tn);
    }
    const long m0 = (long)tm * BM;
    const long n0 = (long)tn * BN;
    const long kbeg = (long)slice * P.k_chunk;
    const long kend = min(P.K, kbeg + P.k_chunk);
    const bool vec_ok = P.vec_ok != 0;

    floatx16 acc[FA][FB];
#pragma unroll
    for (int a = 0; a < FA; ++a)
#pragma unroll
        for (int b = 0; b < FB; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

    floatx4 ra[A_PER], rb[B_PER];

    // Interior tiles whose rows are 16-byte aligned take a branch-free load path; edge tiles and the last,
    // partial k-stage go through the guarded loads.
    const bool interior = vec_ok && m0 + BM <= P.M && n0 + BN <= P.N;
    auto fetch = [&](long k0) {
        if (interior && k0 + KT <= kend) {
#pragma unroll
            for (int i = 0; i < A_PER; ++i) {
                const int s = tid + i * NT;
                if (A4 % NT == 0 || s < A4) {
                    const long kr = k0 + s / (BM / 4), col = m0 + 4 * (s % (BM / 4));
                    if constexpr (ABF16) {
                        const uint2 u = *(const uint2 *)((const unsigned short *)P.A + kr * P.lda + col);
                        ra[i].x = __uint_as_float(u.x << 16);
                        ra[i].y = __uint_as_float(u.x & 0xFFFF0000u);
                        ra[i].z = __uint_as_float(u.y << 16);
                        ra[i].w = __uint_as_float(u.y & 0xFFFF0000u);
                    } else {
                        ra[i] = *(const floatx4 *)((const float *)P.A + kr * P.lda + col);
                    }
                }
            }
#pragma unroll
            for (int i = 0; i < B_PER; ++i) {
                const int s = tid + i * NT;
                if (B4 % NT == 0 || s < B4) {
                    const long kr = k0 + s / (BN / 4), col = n0 + 4 * (s % (BN / 4));
                    if constexpr (BBF16) {
                        const uint2 u = *(const uint2 *)((const unsigned short *)P.B + kr * P.ldb + col);
                        rb[i].x = __uint_as_float(u.x << 16);
                        rb[i].y = __uint_as_float(u.x & 0xFFFF0000u);
                        rb[i].z = __uint_as_float(u.y << 16);
                        rb[i].w = __uint_as_float(u.y & 0xFFFF0000u);
                    } else {
                        rb[i] = *(const floatx4 *)((const float *)P.B + kr * P.ldb + col);
                    }
                }
            }
            return;
        }
#pragma unroll
        for (int i = 0; i < A_PER; ++i) {
            int s = tid + i * NT;
            if (A4 % NT == 0 || s < A4) {
                int kr = s / (BM / 4);
                int c4 = s % (BM / 4);
                ra[i] = load4<ABF16>(P.A, P.lda, k0 + kr, kend, m0 + 4 * c4, P.M, vec_ok);
            }
        }
#pragma unroll
        for (int i = 0; i < B_PER; ++i) {
            int s = tid + i * NT;
            if (B4 % NT == 0 || s < B4) {
                int kr = s / (BN / 4);
                int c4 = s % (BN / 4);
                rb[i] = load4<BBF16>(P.B, P.ldb, k0 + kr, kend, n0 + 4 * c4, P.N, vec_ok);
            }
        }
    };
    auto stash = [&](int buf) {
        floatx4 *dA = (floatx4 *)(sA + buf * KT * BM);
        floatx4 *dB = (floatx4 *)(sB + buf * KT * BN);
#pragma unroll
        for (int i = 0; i < A_PER; ++i) {
            int s = tid + i * NT;
            if (A4 % NT == 0 || s < A4) dA[s] = ra[i];
        }
#pragma unroll
        for (int i = 0; i < B_PER; ++i) {
            int s = tid + i * NT;
            if (B4 % NT == 0 || s < B4) dB[s] = rb[i];
        }
    };

    // write number i of a stage: the A registers first, then the B registers
    auto stash_one = [&](int buf, int i) {
        if (i < A_PER) {
            const int sidx = tid + i * NT;
            if (A4 % NT == 0 || sidx < A4) ((floatx4 *)(sA + buf * KT * BM))[sidx] = ra[i];
        } else {
            const int sidx = tid + (i - A_PER) * NT;
            if (B4 % NT == 0 || sidx < B4) ((floatx4 *)(sB + buf * KT * BN))[sidx] = rb[i - A_PER];
        }
    };

    // fp32 operands of an interior tile go from global memory straight into the LDS stage (16 bytes per lane,
    // lane l of a wave lands at dst + 16 l, so one wave instruction fills 256 consecutive floats of the stage):
    // no staging registers, and above all no LDS write instructions in front of the barrier, during which the
    // matrix pipe would stand still (a register-only model of this loop on MI355X: 87 % of the fp32 peak with the
    // eight 16-byte LDS writes per thread and stage, 94 % with the direct loads).
    constexpr int NWAVES = NT / 64;
    constexpr int CE = LB ? 512 : 256;                              // elements of a 1 KB chunk
    constexpr int CH_A = KT * BM / CE, CH_B = KT * BN / CE;         // chunks of a stage
    static_assert((KT * BM) % CE == 0 && (KT * BN) % CE == 0, "stage must be whole 1 KB chunks");
    auto fetch_direct = [&](long k0, int buf) {
#pragma unroll
        for (int i = 0; i < (CH_A + NWAVES - 1) / NWAVES; ++i) {
            const int c = wave + i * NWAVES;
            if (CH_A % NWAVES == 0 || c < CH_A) {
                const int e = c * CE + (CE / 64) * lane;
                if constexpr (LB) {
                    const unsigned short *gp = (const unsigned short *)P.A + (k0 + e / BM) * P.lda + m0 + e % BM;
                    __builtin_amdgcn_global_load_lds(
                        gp, (__attribute__((address_space(3))) void *)(hA + buf * KT * BM + c * CE), 16, 0, 0);
                } else {
                    const float *gp = (const float *)P.A + (k0 + e / BM) * P.lda + m0 + e % BM;
                    __builtin_amdgcn_global_load_lds(
                        gp, (__attribute__((address_space(3))) void *)(sA + buf * KT * BM + c * CE), 16, 0, 0);
                }
            }
        }
#pragma unroll
        for (int i = 0; i < (CH_B + NWAVES - 1) / NWAVES; ++i) {
            const int c = wave + i * NWAVES;
            if (CH_B % NWAVES == 0 || c < CH_B) {
                const int e = c * CE + (CE / 64) * lane;
                if constexpr (LB) {
                    const unsigned short *gp = (const unsigned short *)P.B + (k0 + e / BN) * P.ldb + n0 + e % BN;
                    __builtin_amdgcn_global_load_lds(
                        gp, (__attribute__((address_space(3))) void *)(hB + buf * KT * BN + c * CE), 16, 0, 0);
                } else {
                    const float *gp = (const float *)P.B + (k0 + e / BN) * P.ldb + n0 + e % BN;
                    __builtin_amdgcn_global_load_lds(
                        gp, (__attribute__((address_space(3))) void *)(sB + buf * KT * BN + c * CE), 16, 0, 0);
                }
            }
        }
    };

    const int l32 = lane & 31;
    const int khalf = lane >> 5;
    const int offA = wm * (32 * FA) + FA * l32 + khalf * BM;
    const int offB = wn * (32 * FB) + FB * l32 + khalf * BN;
    // fragments of k-step kk (rows 2kk, 2kk+1 of the stage) of buffer `buf`
    auto widen2 = [](unsigned u, float &lo, float &hi) {
        lo = __uint_as_float(u << 16);
        hi = __uint_as_float(u & 0xFFFF0000u);
    };
    auto read_frags = [&](int buf, int kk, float *fa, float *fb) {
        if constexpr (LB) {
            const unsigned short *cA = hA + buf * KT * BM + offA + 2 * kk * BM;
            const unsigned short *cB = hB + buf * KT * BN + offB + 2 * kk * BN;
            if constexpr (FA == 4) {
                const uint2 t = *(const uint2 *)cA;
                widen2(t.x, fa[0], fa[1]);
                widen2(t.y, fa[2], fa[3]);
            } else if constexpr (FA == 2) {
                widen2(*(const unsigned *)cA, fa[0], fa[1]);
            } else {
                fa[0] = __uint_as_float((unsigned)cA[0] << 16);
            }
            if constexpr (FB == 4) {
                const uint2 t = *(const uint2 *)cB;
                widen2(t.x, fb[0], fb[1]);
                widen2(t.y, fb[2], fb[3]);
            } else if constexpr (FB == 2) {
                widen2(*(const unsigned *)cB, fb[0], fb[1]);
            } else {
                fb[0] = __uint_as_float((unsigned)cB[0] << 16);
            }
            return;
        }
        const float *cA = sA + buf * KT * BM + offA + 2 * kk * BM;
        const float *cB = sB + buf * KT * BN + offB + 2 * kk * BN;
        if constexpr (FA == 4) {
            floatx4 t = *(const floatx4 *)cA;
            fa[0] = t.x; fa[1] = t.y; fa[2] = t.z; fa[3] = t.w;
        } else if constexpr (FA == 2) {
            floatx2 t = *(const floatx2 *)cA;
            fa[0] = t.x; fa[1] = t.y;
        } else {
            fa[0] = cA[0];
        }
        if constexpr (FB == 4) {
            floatx4 t = *(const floatx4 *)cB;
            fb[0] = t.x; fb[1] = t.y; fb[2] = t.z; fb[3] = t.w;
        } else if constexpr (FB == 2) {
            floatx2 t = *(const floatx2 *)cB;
            fb[0] = t.x; fb[1] = t.y;
        } else {
            fb[0] = cB[0];
        }
    };
    auto mfma_step = [&](const float *fa, const float *fb) {
#pragma unroll
        for (int a = 0; a < FA; ++a)
#pragma unroll
            for (int b = 0; b < FB; ++b)
                acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[a], fb[b], acc[a][b], 0, 0, 0);
    };

    const long nkt = (kend - kbeg + KT - 1) / KT;
    constexpr int KS = KT / 2;            // k-steps per stage
    float fa[2][FA], fb[2][FB];
    if (nkt > 0) {
        if constexpr (DIR) {
            fetch_direct(kbeg, 0);
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        } else {
            fetch(kbeg);
            stash(0);
        }
    }
    __syncthreads();
    if (nkt > 0) read_frags(0, 0, fa[0], fb[0]);
    // Per stage: the fragments of step kk+1 are read while the matrix cores work on step kk; the next
    // stage is written to the other buffer, the barrier passed and its first fragments requested BEFORE the
    // last step's MFMAs are issued, so that neither the barrier nor the LDS latency leaves the pipe empty.
    // Staged path: the next stage's registers go to the other LDS buffer one 16-byte write per k-step, spread over
    // the last steps before the barrier (nobody reads that buffer during this stage).
    // (Measured on MI355X: worth 4 % for bf16 operands, whose loads carry a conversion; fp32 operands are 1 %
    // faster with all writes after the last-but-one step, so for them nothing is spread.)
    constexpr int NW = A_PER + B_PER;
    constexpr bool SPREAD = ABF16 || BBF16;
    constexpr int W0 = !SPREAD ? KS - 1 : ((KS - 1 - NW) > 0 ? (KS - 1 - NW) : 0);   // first k-step with a write
    for (long kt = 0; kt < nkt; ++kt) {
        const int buf = (int)(kt & 1);
        const bool more = kt + 1 < nkt;
        // the other buffer is free from here on: its last readers finished before the barrier that ended the
        // previous stage
        if (more) {
            if constexpr (DIR) fetch_direct(kbeg + (kt + 1) * KT, buf ^ 1);
            else fetch(kbeg + (kt + 1) * KT);
        }
#pragma unroll
        for (int kk = 0; kk < KS - 1; ++kk) {
            read_frags(buf, kk + 1, fa[(kk + 1) & 1], fb[(kk + 1) & 1]);
            if constexpr (!DIR) {
                if (kk >= W0 && kk - W0 < NW) {
                    if (more) stash_one(buf ^ 1, kk - W0);
                }
            }
            __builtin_amdgcn_sched_barrier(0);      // keep the LDS traffic ahead of this step's MFMAs
            mfma_step(fa[kk & 1], fb[kk & 1]);
            __builtin_amdgcn_sched_barrier(0);
        }
        if constexpr (DIR) {
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");            // this wave's rows have landed
        } else {
            if (more) {
#pragma unroll
                for (int i = (KS - 1 - W0); i < NW; ++i) stash_one(buf ^ 1, i);      // what did not fit above
            }
        }
        __syncthreads();
        if (more) read_frags(buf ^ 1, 0, fa[KS & 1], fb[KS & 1]);
        __builtin_amdgcn_sched_barrier(0);
        mfma_step(fa[(KS - 1) & 1], fb[(KS - 1) & 1]);
        __builtin_amdgcn_sched_barrier(0);
    }

    // Epilogue.  Accumulator register v of lane l holds matrix-core row 8*(v/4) + 4*(l/32) + v%4 and
    // column l%32 of the 32x32 result.
    float *outp = P.out + (long)slice * P.slice_stride;
    const long wm0 = m0 + wm * (32 * FA);
    const long wn0 = n0 + wn * (32 * FB);
    if constexpr (PROJ) {
        // Eqs. 8-10 on the result while it sits in the accumulators: W = acc + Z (alpha = beta = 1, so this is the
        // value the plain epilogue would have stored), then the stand-alone pass's arithmetic, operation for
        // operation.  Rows go RB at a time: their Z, V, d requests are all in flight before the first is used.
        constexpr int RB = 4;
        const long n = wn0 + FB * l32;
        long grp = -1;
        float dl[FB], idl[FB], z0[FB];
        float racc = 0.f;
#pragma unroll
        for (int a = 0; a < FA; ++a) {
#pragma unroll
            for (int v0 = 0; v0 < 16; v0 += RB) {
                float z[RB][FB], vv[RB][FB], di[RB], idi[RB];
#pragma unroll
                for (int u = 0; u < RB; ++u) {
                    const int v = v0 + u;
                    const long m = wm0 + FA * (8 * (v / 4) + 4 * khalf + (v % 4)) + a;
                    const float *zp = P.Z + m * P.ldz + n;
                    const float *vp = P.pV + m * P.ldv + n;
                    if constexpr (FB == 4) {
                        const floatx4 t = *(const floatx4 *)zp, s = *(const floatx4 *)vp;
                        z[u][0] = t.x; z[u][1] = t.y; z[u][2] = t.z; z[u][3] = t.w;
                        vv[u][0] = s.x; vv[u][1] = s.y; vv[u][2] = s.z; vv[u][3] = s.w;
                    } else if constexpr (FB == 2) {
                        const floatx2 t = *(const floatx2 *)zp, s = *(const floatx2 *)vp;
                        z[u][0] = t.x; z[u][1] = t.y;
                        vv[u][0] = s.x; vv[u][1] = s.y;
                    } else {
                        z[u][0] = zp[0];
                        vv[u][0] = vp[0];
                    }
                    di[u] = P.pd[m];
                    idi[u] = P.pinv_d[m];
                }
#pragma unroll
                for (int u = 0; u < RB; ++u) {
                    const int v = v0 + u;
                    const long m = wm0 + FA * (8 * (v / 4) + 4 * khalf + (v % 4)) + a;
                    const long gi = m >> P.g_shift;
                    if (gi != grp) {
                        grp = gi;
#pragma unroll
                        for (int b = 0; b < FB; ++b) {
                            dl[b] = P.pscales[gi * P.ld_grid + n + b];
                            idl[b] = P.pinv_scales[gi * P.ld_grid + n + b];
                            z0[b] = P.pzeros[gi * P.ld_grid + n + b];
                        }
                    }
                    float vn[FB], bn[FB];
#pragma unroll
                    for (int b = 0; b < FB; ++b) {
                        const float w = __fadd_rn(acc[a][b][v], z[u][b]);
                        const float q = __fmul_rn(vv[u][b], P.inv_rho);
                        const float wt = __fadd_rn(w, q);
                        const float x = __fmul_rn(wt, idi[u]);
                        const float y = __fsub_rn(x, z0[b]);
                        const float t = __fmul_rn(y, idl[b]);
                        const float k = fminf(fmaxf(rintf(t), 0.f), P.levels);
                        const float xq = __fadd_rn(__fmul_rn(k, dl[b]), z0[b]);
                        const float Dn = __fmul_rn(di[u], xq);
                        const float r = __fsub_rn(w, Dn);
                        vn[b] = __fadd_rn(vv[u][b], __fmul_rn(P.rho, r));
                        bn[b] = __fsub_rn(Dn, __fmul_rn(vn[b], P.inv_rho_next));
                        racc += r * r;
                    }
                    float *vp = P.pV + m * P.ldv + n;
                    float *op = outp + m * P.ldo + n;
                    if constexpr (FB == 4) {
                        *(floatx4 *)vp = floatx4{vn[0], vn[1], vn[2], vn[3]};
                        *(floatx4 *)op = floatx4{bn[0], bn[1], bn[2], bn[3]};
                    } else if constexpr (FB == 2) {
                        *(floatx2 *)vp = floatx2{vn[0], vn[1]};
                        *(floatx2 *)op = floatx2{bn[0], bn[1]};
                    } else {
                        vp[0] = vn[0];
                        op[0] = bn[0];
                    }
                }
            }
        }
        // squared residual: lanes of a wave, the block's waves through LDS (nobody reads a stage any more: the last
        // k-step's fragments were in registers before the loop's final barrier), one atomic per block
        double tot = (double)racc;
#pragma unroll
        for (int h = 32; h >= 1; h >>= 1) tot += __shfl_xor(tot, h, 64);
        double *red = (double *)lds;
        if (lane == 0) red[wave] = tot;
        __syncthreads();
        if (tid == 0) {
            double s = 0.0;
            for (int w = 0; w < NWAVES; ++w) s += red[w];
            atomicAdd(P.res_sq, s);
        }
        return;
    }
    if constexpr (DIR) {
        // every tile is whole and aligned: no guards, and the rows of Z are requested ZB at a time (one load, one
        // wait, one store per row would pay the memory latency 16 FA times); ZB keeps the kernel free of spills
        constexpr int ZB = FA * FB >= 8 ? 8 : 16;
        const long n = wn0 + FB * l32;
#pragma unroll
        for (int a = 0; a < FA; ++a) {
#pragma unroll
            for (int v0 = 0; v0 < 16; v0 += ZB) {
                float z[ZB][FB];
                if (P.Z) {
#pragma unroll
                    for (int u = 0; u < ZB; ++u) {
                        const int v = v0 + u;
                        const long m = wm0 + FA * (8 * (v / 4) + 4 * khalf + (v % 4)) + a;
                        const float *zp = P.Z + m * P.ldz + n;
                        if constexpr (FB == 4) {
                            const floatx4 t = *(const floatx4 *)zp;
                            z[u][0] = t.x; z[u][1] = t.y; z[u][2] = t.z; z[u][3] = t.w;
                        } else if constexpr (FB == 2) {
                            const floatx2 t = *(const floatx2 *)zp;
                            z[u][0] = t.x; z[u][1] = t.y;
                        } else {
                            z[u][0] = zp[0];
                        }
                    }
                }
#pragma unroll
                for (int u = 0; u < ZB; ++u) {
                    const int v = v0 + u;
                    const long m = wm0 + FA * (8 * (v / 4) + 4 * khalf + (v % 4)) + a;
                    float r[FB];
#pragma unroll
                    for (int b = 0; b < FB; ++b) {
                        r[b] = P.alpha * acc[a][b][v];
                        if (P.Z) r[b] += P.beta * z[u][b];
                    }
                    float *op = outp + m * P.ldo + n;
                    if constexpr (FB == 4) {
                        *(floatx4 *)op = floatx4{r[0], r[1], r[2], r[3]};
                    } else if constexpr (FB == 2) {
                        *(floatx2 *)op = floatx2{r[0], r[1]};
                    } else {
                        op[0] = r[0];
                    }
                }
            }
        }
        return;
    }
#pragma unroll
    for (int a = 0; a < FA; ++a) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int ic = 8 * (v / 4) + 4 * khalf + (v % 4);
            const long m = wm0 + FA * ic + a;
            if (m >= P.M) continue;
            const long n = wn0 + FB * l32;
            float r[FB];
#pragma unroll
            for (int b = 0; b < FB; ++b) r[b] = P.alpha * acc[a][b][v];
            bool done = false;
            if constexpr (FB == 4) {
              if (vec_ok && n + 3 < P.N) {
                floatx4 o = {r[0], r[1], r[2], r[3]};
                if (P.Z) {
                    floatx4 z = *(const floatx4 *)(P.Z + m * P.ldz + n);
                    o.x += P.beta * z.x; o.y += P.beta * z.y; o.z += P.beta * z.z; o.w += P.beta * z.w;
                }
                *(floatx4 *)(outp + m * P.ldo + n) = o;
                done = true;
              }
            }
            if (!done) {
#pragma unroll
                for (int b = 0; b < FB; ++b) {
                    if (n + b < P.N) {
                        float o = r[b];
                        if (P.Z) o += P.beta * P.Z[m * P.ldz + n + b];
                        outp[m * P.ldo + n + b] = o;
                    }
                }
            }
        }
    }
}

template <int FA, int FB, int WGM, int WGN, int KT, bool PROJ_OK = false>
admmq_status launch_cfg(admmq_ctx *ctx, const gemm_tn_args &a) {
    constexpr int BM = 32 * FA * WGM;
    constexpr int BN = 32 * FB * WGN;
    GemmParams P;
    P.A = a.A; P.B = a.B; P.lda = a.lda; P.ldb = a.ldb;
    P.M = a.M; P.N = a.N; P.K = a.K;
    P.alpha = a.alpha; P.beta = a.beta; P.Z = a.Z; P.ldz = a.ldz;
    P.out = a.out; P.ldo = a.ldo;
    P.tiles_m = (int)((a.M + BM - 1) / BM);
    P.tiles_n = (int)((a.N + BN - 1) / BN);
    P.lower_only = a.lower_only;
    P.split_k = a.split_k > 1 ? a.split_k : 1;
    long kc = (a.K + P.split_k - 1) / P.split_k;
    kc = (kc + KT - 1) / KT * KT;
    P.k_chunk = kc;
    P.slice_stride = a.slice_stride;
    auto al16 = [](const void *p) { return ((uintptr_t)p & 15) == 0; };
    const long esz_a = a.a_bf16 ? 2 : 4, esz_b = a.b_bf16 ? 2 : 4;
    bool ok = (a.M % 4 == 0) && (a.N % 4 == 0) && al16(a.out) && (a.ldo % 4 == 0) &&
              ((uintptr_t)a.A % (4 * esz_a) == 0) && (a.lda % 4 == 0) &&
              ((uintptr_t)a.B % (4 * esz_b) == 0) && (a.ldb % 4 == 0) && (a.slice_stride % 4 == 0);
    if (a.Z) ok = ok && al16(a.Z) && (a.ldz % 4 == 0);
    P.vec_ok = ok ? 1 : 0;
    if (a.proj) {
        const gemm_proj_args &q = *a.proj;
        P.pV = q.V; P.ldv = q.ldv; P.pd = q.d; P.pinv_d = q.inv_d; P.pscales = q.scales;
        P.pinv_scales = q.inv_scales; P.pzeros = q.zeros; P.ld_grid = q.ld_grid; P.g_shift = q.g_shift;
        P.levels = q.levels; P.rho = q.rho; P.inv_rho = q.inv_rho; P.inv_rho_next = q.inv_rho_next;
        P.res_sq = q.res_sq;
    } else {
        P.pV = nullptr; P.ldv = 0; P.pd = P.pinv_d = P.pscales = P.pinv_scales = P.pzeros = nullptr;
        P.ld_grid = 0; P.g_shift = 0; P.levels = P.rho = P.inv_rho = P.inv_rho_next = 0.f; P.res_sq = nullptr;
    }
    long tiles;
    if (a.lower_only) {
        if (BM != BN) return ADMMQ_ERR_PARAM;
        tiles = (long)P.tiles_m * (P.tiles_m + 1) / 2;
    } else {
        tiles = (long)P.tiles_m * P.tiles_n;
    }
    const size_t lds_bytes = (size_t)2 * KT * (BM + BN) * sizeof(float);
    dim3 grid((unsigned)(tiles * P.split_k)), block(64 * WGM * WGN);
#define ADMMQ_GEMM_LAUNCH(AB, BB, DR)                                                                  \
    do {                                                                                               \
        auto kern = gemm_tn_kernel<FA, FB, WGM, WGN, KT, AB, BB, DR>;                                      \
        static unsigned long long lds_allowed = 0;                                                     \
        ADMMQ_HIP(admmq_allow_lds((const void *)kern, (int)lds_bytes, ctx->device, &lds_allowed));     \
        hipLaunchKernelGGL(kern, grid, block, lds_bytes, ctx->stream, P);                              \
    } while (0)
    // whole tiles, whole k-stages in every slice, aligned rows: the direct-load kernel
    bool direct = ok && a.M % BM == 0 && a.N % BN == 0 && a.K % KT == 0 && a.K > 0;
    if (a.a_bf16)        // 16-byte loads of bf16 rows
        direct = direct && a.lda % 8 == 0 && a.ldb % 8 == 0 && al16(a.A) && al16(a.B);
    if (a.proj) {
        // the caller has asked admmq_gemm_tn_can_project; anything else here is a mistake of the library's own
        if constexpr (PROJ_OK) {
            if (!direct || a.a_bf16 || a.b_bf16 || !a.Z || a.alpha != 1.f || a.beta != 1.f || a.lower_only ||
                P.split_k != 1 || !al16(a.proj->V) || a.proj->ldv % 4 != 0 || !a.proj->res_sq)
                return ADMMQ_ERR_PARAM;
            auto kern = gemm_tn_kernel<FA, FB, WGM, WGN, KT, false, false, true, true>;
            static unsigned long long lds_allowed = 0;
            ADMMQ_HIP(admmq_allow_lds((const void *)kern, (int)lds_bytes, ctx->device, &lds_allowed));
            hipLaunchKernelGGL(kern, grid, block, lds_bytes, ctx->stream, P);
            ADMMQ_HIP(hipGetLastError());
            return ADMMQ_OK;
        } else {
            return ADMMQ_ERR_PARAM;
        }
    }
    if (a.a_bf16 && a.b_bf16) {
        if (direct) ADMMQ_GEMM_LAUNCH(true, true, true);
        else ADMMQ_GEMM_LAUNCH(true, true, false);
    } else if (!a.a_bf16 && !a.b_bf16) {
        if (direct) ADMMQ_GEMM_LAUNCH(false, false, true);
        else ADMMQ_GEMM_LAUNCH(false, false, false);
    } else return ADMMQ_ERR_PARAM;
#undef ADMMQ_GEMM_LAUNCH
    ADMMQ_HIP(hipGetLastError());
    return ADMMQ_OK;
}

__global__ void sym_reduce_kernel(float *H, long n, const float *P, int slices, long stride, int accumulate) {
    // one thread per lower-triangle element (i >= j) of a 32x32 patch; patch grid covers the square
    __shared__ float tile[32][33];
    const int bi = blockIdx.y, bj = blockIdx.x;
    if (bj > bi) return;
    const int tx = threadIdx.x, ty = threadIdx.y;   // 32 x 8
    for (int r = ty; r < 32; r += 8) {
        long i = (long)bi * 32 + r, j = (long)bj * 32 + tx;
        float s = 0.f;
        if (i < n && j < n && i >= j) {
            for (int q = 0; q < slices; ++q) s += P[(long)q * stride + i * n + j];
            if (accumulate) s += H[i * n + j];
            H[i * n + j] = s;
        }
        tile[r][tx] = s;
    }
    __syncthreads();
    for (int r = ty; r < 32; r += 8) {
        // element (j', i') of the upper triangle = tile[i' - bi*32][j' - bj*32]
        long jj = (long)bj * 32 + r, ii = (long)bi * 32 + tx;
        if (ii < n && jj < n && ii > jj) H[jj * n + ii] = tile[tx][r];
    }
}

}  // namespace

namespace {
// Launch rounds of a full-rectangle product in units of one 256 x 256 tile per compute unit, for the tile the
// choice below makes (128 x 128 tiles run at 130 against 141 TFLOP/s, 64 x 64 tiles at about half of that).
double rounds_cost(long M, long N) {
    const long t256 = ((M + 255) / 256) * ((N + 255) / 256);
    const long t128 = ((M + 127) / 128) * ((N + 127) / 128);
    const long t64 = ((M + 63) / 64) * ((N + 63) / 64);
    if (t256 >= 200) return (double)((t256 + 255) / 256);
    if (t128 >= 128) return (double)((t128 + 255) / 256) * 0.27;
    return (double)((t64 + 255) / 256) * 0.125;
}
}  // namespace

namespace {
int gemm_variant() {
    static int variant = -1;
    if (variant < 0) {
        const char *e = getenv("ADMMQ_GEMM_VARIANT");
        variant = e ? atoi(e) : 0;
    }
    return variant;
}
int gemm_mid_variant() {
    static int mid_variant = -1;
    if (mid_variant < 0) {
        const char *e = getenv("ADMMQ_GEMM_MID");
        mid_variant = e ? atoi(e) : 0;
    }
    return mid_variant;
}
// A tile count just above a multiple of the 256 compute units leaves the last round nearly empty (4096 x 5120:
// 320 tiles, two rounds for 1.25 rounds of work).  Then the leading columns that fill whole rounds go out as
// one launch and the remaining columns as a product of their own, with the smaller tile that suits their
// count.  Every output element is still one k-ordered sum of its tile: the split changes no value, and columns
// handled by the same tile shape as in a narrower call come out bit-identical to that call.
// Returns the number of leading columns of such a split, or 0.
long head_columns(const gemm_tn_args &a) {
    if (a.lower_only || a.split_k > 1) return 0;
    const long tm = (a.M + 255) / 256, tn = (a.N + 255) / 256, t = tm * tn;
    if (t <= 256 || t % 256 == 0) return 0;
    const long c_full = (t / 256) * 256 / tm;          // column tiles that fit whole rounds
    if (c_full < 1 || c_full >= tn) return 0;
    const long n_head = c_full * 256;
    const double whole = (double)((t + 255) / 256);
    const double parts = (double)((c_full * tm + 255) / 256) + rounds_cost(a.M, a.N - n_head);
    return parts < 0.93 * whole ? n_head : 0;
}
// tile choice: the largest tile that still gives every CU work.  0: 256 x 256, 1: 128 x 128, 2: 64 x 64
int tile_class(const gemm_tn_args &a) {
    const long t256 = ((a.M + 255) / 256) * ((a.N + 255) / 256);
    const long t128 = ((a.M + 127) / 128) * ((a.N + 127) / 128);
    const long work = a.split_k > 1 ? a.split_k : 1;
    bool big, mid;
    if (a.lower_only) {
        const long tm256 = (a.M + 255) / 256, tm128 = (a.M + 127) / 128;
        big = tm256 * (tm256 + 1) / 2 * work >= 200;
        mid = tm128 * (tm128 + 1) / 2 * work >= 128;
    } else {
        big = t256 * work >= 200;
        mid = t128 * work >= 128;
    }
    return big ? 0 : mid ? 1 : 2;
}
void shift_columns(gemm_proj_args &q, long c) {
    q.V += c;
    q.scales += c;
    q.inv_scales += c;
    q.zeros += c;
}
}  // namespace

// Whether a product with a.proj set can run with the projection epilogue: the tile shapes that carry it, whole
// tiles and stages, aligned rows (what the launcher then insists on).
bool admmq_gemm_tn_can_project(const gemm_tn_args &a) {
    if (!a.proj || a.M <= 0 || a.N <= 0 || a.K <= 0 || a.lower_only || a.split_k > 1 || a.a_bf16 || a.b_bf16 || !a.Z ||
        a.alpha != 1.f || a.beta != 1.f)
        return false;
    const gemm_proj_args &q = *a.proj;
    auto al16 = [](const void *p) { return ((uintptr_t)p & 15) == 0; };
    if (!q.V || !q.d || !q.inv_d || !q.scales || !q.inv_scales || !q.zeros || !q.res_sq || q.ldv % 4 != 0 ||
        !al16(q.V) || !al16(a.A) || !al16(a.B) || !al16(a.Z) || !al16(a.out) || a.lda % 4 != 0 || a.ldb % 4 != 0 ||
        a.ldz % 4 != 0 || a.ldo % 4 != 0 || q.g_shift < 0 || q.g_shift > 62)
        return false;
    const long n_head = head_columns(a);
    if (n_head > 0) {
        gemm_tn_args head = a, tail = a;
        gemm_proj_args tq = q;
        head.N = n_head;
        tail.N = a.N - n_head;
        tail.B = (const char *)a.B + n_head * 4;
        tail.Z = a.Z + n_head;
        tail.out = a.out + n_head;
        shift_columns(tq, n_head);
        tail.proj = &tq;
        return admmq_gemm_tn_can_project(head) && admmq_gemm_tn_can_project(tail);
    }
    switch (tile_class(a)) {
        case 0: return gemm_variant() == 0 && a.M % 256 == 0 && a.N % 256 == 0 && a.K % 32 == 0;
        case 1: return gemm_mid_variant() == 0 && a.M % 128 == 0 && a.N % 128 == 0 && a.K % 64 == 0;
        default: return false;
    }
}

admmq_status admmq_gemm_tn(admmq_ctx *ctx, const gemm_tn_args &a) {
    if (a.M <= 0 || a.N <= 0 || a.K < 0) return ADMMQ_ERR_SHAPE;
    const int variant = gemm_variant();
    const long n_head = head_columns(a);
    if (n_head > 0) {
        gemm_tn_args head = a, tail = a;
        gemm_proj_args tq;
        head.N = n_head;
        tail.N = a.N - n_head;
        const long eb = a.b_bf16 ? 2 : 4;
        tail.B = (const char *)a.B + n_head * eb;
        if (a.Z) tail.Z = a.Z + n_head;
        tail.out = a.out + n_head;
        if (a.proj) {
            tq = *a.proj;
            shift_columns(tq, n_head);
            tail.proj = &tq;
        }
        ADMMQ_TRY(admmq_gemm_tn(ctx, head));
        return admmq_gemm_tn(ctx, tail);
    }
    const int cls = tile_class(a);
    if (cls == 0) {
        // measured on MI355X (W-update products, n = p = 4096): eight waves of 64 x 128 with 32-row stages
        // reach 135 TFLOP/s, four waves of 128 x 128 with 16-row stages 128 TFLOP/s; variant 6 (128 x 256 tiles,
        // four waves, two blocks per compute unit whose barriers fall at different times) reaches the same
        // 135: the barrier is not what keeps the matrix pipe at 86 % busy
        switch (a.lower_only ? 0 : variant) {      // the triangle enumeration needs square tiles
            case 1: return launch_cfg<4, 4, 2, 2, 16>(ctx, a);
            case 2: return launch_cfg<4, 4, 2, 2, 32>(ctx, a);
            case 3: return launch_cfg<2, 4, 4, 2, 16>(ctx, a);
            case 4: return launch_cfg<4, 2, 2, 4, 32>(ctx, a);
            case 5: return launch_cfg<2, 2, 4, 4, 32>(ctx, a);
            case 6: return launch_cfg<2, 4, 2, 2, 16>(ctx, a);
            default: return launch_cfg<2, 4, 4, 2, 32, true>(ctx, a);
        }
    }
    if (cls == 1) {
        // 128 x 128 tiles, measured on MI355X at 4096 x 1024 x 4096 (256 tiles, one per compute unit) with staged
        // loads: eight waves of 64 x 32 with 64-row stages 118 TFLOP/s, sixteen waves of 32 x 32 116, four waves of
        // 64 x 64 with 16-row stages 106 (one wave per SIMD hides no latency); the first with direct loads: 130
        switch (gemm_mid_variant()) {
            case 1: return launch_cfg<2, 2, 2, 2, 16>(ctx, a);
            case 2: return launch_cfg<1, 1, 4, 4, 32>(ctx, a);
            default: return launch_cfg<2, 1, 2, 4, 64, true>(ctx, a);
        }
    }
    if (a.proj) return ADMMQ_ERR_PARAM;
    return launch_cfg<1, 1, 2, 2, 16>(ctx, a);
}

admmq_status admmq_sym_reduce(admmq_ctx *ctx, float *H, int64_t n, const float *P, int slices,
                              int64_t slice_stride, int accumulate) {
    dim3 block(32, 8), grid((unsigned)((n + 31) / 32), (unsigned)((n + 31) / 32));
    hipLaunchKernelGGL(sym_reduce_kernel, grid, block, 0, ctx->stream, H, (long)n, P, slices, (long)slice_stride,
                       accumulate);
    ADMMQ_HIP(hipGetLastError());
    return ADMMQ_OK;
}
