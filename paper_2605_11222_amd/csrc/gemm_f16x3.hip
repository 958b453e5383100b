// Opt-in fast form of the W-update products (eq. 7):  out = alpha * A^T B + beta * Z  on the fp16 matrix cores.
//
// Each fp32 operand x is split, after a power-of-two scaling s that brings the matrix's largest entry into
// [2^14, 2^15), into two fp16 values  hi = fp16(s x),  lo = fp16(s x - hi):  hi + lo carries 22 bits of s x.  The
// product is accumulated in fp32 as  hiA hiB + hiA loB + loA hiB  (every one of these products is exact in fp32;
// the dropped loA loB is 2^-22 of the term), by v_mfma_f32_32x32x16_f16 at 16 times the fp32 matrix rate, so three
// products still leave a factor of five in issue slots.  What is lost against the fp32 product is operand bits 23
// and 24 and the lo-lo term, about 3e-7 of each term with random signs: an order of magnitude below the fp32
// accumulation error both forms share.
//
// Both operands are k-major, [K][M] and [K][N], as everywhere on this path.  The tile machinery is the one of the
// bf16 Hessian kernel: stages of 16 k-rows of the four fp16 matrices go from global memory straight into an LDS
// ring of four stages, the transposing LDS read hands each lane four k-values of its row or column, reads and
// loads are issued one piece after each product.
#include "common.h"

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef _Float16 halfx8 __attribute__((ext_vector_type(8)));
typedef unsigned uintx2 __attribute__((ext_vector_type(2)));
typedef unsigned uintx4 __attribute__((ext_vector_type(4)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int FX_TILE = 256;
constexpr int FX_KT = 16;                                  // k-rows per stage (one matrix-core step)
constexpr int FX_STAGES = 4;
constexpr int FX_CHUNK = 1024 + 64;                        // two k-rows x 256 columns of fp16, padded (bank windows)
constexpr int FX_MAT = (FX_KT / 2) * FX_CHUNK;             // one of the four matrices in a stage: 8704 B
constexpr int FX_STAGE = 4 * FX_MAT;                       // 34816 B
constexpr int FX_LDS = FX_STAGES * FX_STAGE;               // 139264 B

struct F16x3Params {
    const unsigned short *A1, *A2, *B1, *B2;               // fp16 bit patterns, [K][M] and [K][N], dense rows
    const float *scaleA, *scaleB;                          // device: the power-of-two scalings of A and B
    long M, N, K;
    long ldb;                                              // row length of B1, B2 (>= N: a column window of the pair)
    float alpha, beta;
    const float *Z;
    long ldz;
    float *out;
    long ldo;
    int tiles_m, tiles_n;
    int split;                                             // slices of the k axis (1: the block writes out itself)
    long k_chunk;                                          // k-rows per slice, a multiple of 32
    float *partial;                                        // split > 1: [split][M][N] unscaled partial sums
};

// Same block -> tile map as the fp32 products: the blocks of one XCD (ids equal mod 8) form a compact patch of
// the tile grid, walked in short columns of four tiles.
__device__ inline void fx_tile_of_block(int bid, int nblocks, int tiles_m, int tiles_n, int &tm, int &tn) {
    int pid = bid;
    if ((nblocks & 7) == 0) pid = (bid & 7) * (nblocks >> 3) + (bid >> 3);
    const int GROUP = 4;
    const int per_group = GROUP * tiles_n;
    const int grp = pid / per_group;
    const int first_m = grp * GROUP;
    const int gsz = min(tiles_m - first_m, GROUP);
    const int in_grp = pid - grp * per_group;
    tm = first_m + in_grp % gsz;
    tn = in_grp / gsz;
}

struct FxFrags {
    uintx2 a1[4][2], a2[4][2], b1[4][2], b2[4][2];
};

__global__ __launch_bounds__(256, 1) void gemm_f16x3_kernel(F16x3Params P) {
    extern __shared__ __attribute__((aligned(16))) unsigned char fx_lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave & 1, wn = wave >> 1;               // the wave's 128 x 128 quadrant of the tile
    // with too few tiles to fill the chip the k axis is cut into slices: block = (slice, tile)
    const int tiles_total = P.tiles_m * P.tiles_n;
    const int slice = (int)(blockIdx.x / tiles_total);
    int tm, tn;
    fx_tile_of_block((int)(blockIdx.x - slice * tiles_total), tiles_total, P.tiles_m, P.tiles_n, tm, tn);
    const long m0 = (long)tm * FX_TILE, n0 = (long)tn * FX_TILE;
    const long kbeg = (long)slice * P.k_chunk;
    const int nst = (int)(P.k_chunk / FX_KT);

    floatx16 acc[4][4];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

    // Load number i (0..7) of stage s: matrix i / 2 (A1, A2, B1, B2), chunk wave + 4 (i % 2) of its eight; lane l
    // brings 16 bytes of k-row 2 chunk + l / 32.  Stages past the end are loaded from the last real rows into a
    // buffer nobody reads: every stage costs every wave eight loads and the loop has no branches.
    const long lrow = lane >> 5, lcol = (lane & 31) * 8;
    auto load_one = [&](int s, int i) {
        const long k0 = kbeg + (long)min(s, nst - 1) * FX_KT;
        const int mat = i >> 1, c = wave + 4 * (i & 1);
        const unsigned short *src = mat == 0 ? P.A1 : mat == 1 ? P.A2 : mat == 2 ? P.B1 : P.B2;
        const long ld = mat < 2 ? P.M : P.ldb, c0 = mat < 2 ? m0 : n0;
        unsigned char *dst = fx_lds + (s % FX_STAGES) * FX_STAGE + mat * FX_MAT + c * FX_CHUNK;
        __builtin_amdgcn_global_load_lds(src + (k0 + 2 * c + lrow) * ld + c0 + lcol,
                                         (__attribute__((address_space(3))) void *)dst, 16, 0, 0);
    };

    // Transposing read (see the bf16 Hessian kernel): in every group of 16 lanes, source lane 4 j + q points at four
    // columns of k-row j, lane i receives column i of rows j = 0..3; read h takes k-rows 8 (l / 32) + 2 j + h, the
    // same assignment on both sides of the product.  Written as assembly so that the compiler does not make the
    // reads wait for every outstanding global -> LDS load; the waits are placed by hand.
    const int grp = lane >> 4, jrow = (lane & 15) >> 2, q = lane & 3;
    const int lane_off = (4 * (grp >> 1) + jrow) * FX_CHUNK + (16 * (grp & 1) + 4 * q) * 2;
    const unsigned lds0 = (unsigned)(unsigned long)(__attribute__((address_space(3))) unsigned char *)fx_lds;
    const unsigned offA = lds0 + lane_off + wm * 256;      // 128 columns = 256 bytes per quadrant
    const unsigned offB = lds0 + 2 * FX_MAT + lane_off + wn * 256;
#define FX_RD(dst, addr, off) \
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:" #off : "=v"(dst) : "v"(addr) : "memory")
#define FX_RD2(X, I, addr, K0)                    \
    do {                                          \
        FX_RD(X[I][0], addr, K0 + 64 * I);        \
        FX_RD(X[I][1], addr, K0 + 64 * I + 512);  \
    } while (0)
#define FX_FRAG(X) __builtin_bit_cast(halfx8, __builtin_shufflevector(X[0], X[1], 0, 1, 2, 3))
#define FX_MFMA(FA_, FB_, A_, B_) \
    acc[A_][B_] = __builtin_amdgcn_mfma_f32_32x32x16_f16(FX_FRAG(FA_[A_]), FX_FRAG(FB_[B_]), acc[A_][B_], 0, 0, 0)
#define FX_SB __builtin_amdgcn_sched_barrier(0)
    auto frags_ready = [](FxFrags &f) {
        asm volatile("s_waitcnt lgkmcnt(0)"
                     : "+v"(f.a1[0][0]), "+v"(f.a1[0][1]), "+v"(f.a1[1][0]), "+v"(f.a1[1][1]), "+v"(f.a1[2][0]),
                       "+v"(f.a1[2][1]), "+v"(f.a1[3][0]), "+v"(f.a1[3][1]), "+v"(f.b1[0][0]), "+v"(f.b1[0][1]),
                       "+v"(f.b1[1][0]), "+v"(f.b1[1][1]), "+v"(f.b1[2][0]), "+v"(f.b1[2][1]), "+v"(f.b1[3][0]),
                       "+v"(f.b1[3][1])
                     :
                     : "memory");
        asm volatile(""
                     : "+v"(f.a2[0][0]), "+v"(f.a2[0][1]), "+v"(f.a2[1][0]), "+v"(f.a2[1][1]), "+v"(f.a2[2][0]),
                       "+v"(f.a2[2][1]), "+v"(f.a2[3][0]), "+v"(f.a2[3][1]), "+v"(f.b2[0][0]), "+v"(f.b2[0][1]),
                       "+v"(f.b2[1][0]), "+v"(f.b2[1][1]), "+v"(f.b2[2][0]), "+v"(f.b2[2][1]), "+v"(f.b2[3][0]),
                       "+v"(f.b2[3][1])
                     :
                     : "memory");
    };
    // (The barrier is the bare instruction: with the fences of __syncthreads() the compiler, which sees the direct
    // loads of the stage before in the same straight-line code, puts a wait for ALL of them in front of it.  Every
    // memory operation around it is either assembly or pinned by the scheduling barriers, and waited for by hand.)
    // One stage: wait for the next stage's loads and this stage's fragments, pass the barrier (this stage's buffer
    // is then free for the loads of the stage four ahead, the next stage's rows have landed for every wave), then
    // three sweeps over the 16 accumulators: hi hi, hi lo, lo hi.  The 32 reads of the next stage's fragments follow
    // the first 16 products one pair each, the eight loads the next eight products.
#define FX_STAGE_BODY(CUR, NXT, T)                                                                       \
    do {                                                                                                 \
        const unsigned nb_ = (unsigned)((((T) + 1) % FX_STAGES) * FX_STAGE);                             \
        const unsigned na_ = offA + nb_, nbb_ = offB + nb_;                                              \
        asm volatile("s_waitcnt vmcnt(16)" ::: "memory");                                                \
        frags_ready(CUR);                                                                                \
        __builtin_amdgcn_s_barrier();                                                                    \
        FX_SB;                                                                                           \
        FX_MFMA(CUR.a1, CUR.b1, 0, 0); FX_RD2(NXT.a1, 0, na_, 0);     FX_SB;                              \
        FX_MFMA(CUR.a1, CUR.b1, 0, 1); FX_RD2(NXT.b1, 0, nbb_, 0);    FX_SB;                              \
        FX_MFMA(CUR.a1, CUR.b1, 0, 2); FX_RD2(NXT.b1, 1, nbb_, 0);    FX_SB;                              \
        FX_MFMA(CUR.a1, CUR.b1, 0, 3); FX_RD2(NXT.b1, 2, nbb_, 0);    FX_SB;                              \
        FX_MFMA(CUR.a1, CUR.b1, 1, 0); FX_RD2(NXT.b1, 3, nbb_, 0);    FX_SB;                              \
        FX_MFMA(CUR.a1, CUR.b1, 1, 1); FX_RD2(NXT.a1, 1, na_, 0);     FX_SB;                              \
        FX_MFMA(CUR.a1, CUR.b1, 1, 2); FX_RD2(NXT.a1, 2, na_, 0);     FX_SB;                              \
        FX_MFMA(CUR.a1, CUR.b1, 1, 3); FX_RD2(NXT.a1, 3, na_, 0);     FX_SB;                              \
        FX_MFMA(CUR.a1, CUR.b1, 2, 0); FX_RD2(NXT.b2, 0, nbb_, 8704); FX_SB;                              \
        FX_MFMA(CUR.a1, CUR.b1, 2, 1); FX_RD2(NXT.b2, 1, nbb_, 8704); FX_SB;                              \
        FX_MFMA(CUR.a1, CUR.b1, 2, 2); FX_RD2(NXT.b2, 2, nbb_, 8704); FX_SB;                              \
        FX_MFMA(CUR.a1, CUR.b1, 2, 3); FX_RD2(NXT.b2, 3, nbb_, 8704); FX_SB;                              \
        FX_MFMA(CUR.a1, CUR.b1, 3, 0); FX_RD2(NXT.a2, 0, na_, 8704);  FX_SB;                              \
        FX_MFMA(CUR.a1, CUR.b1, 3, 1); FX_RD2(NXT.a2, 1, na_, 8704);  FX_SB;                              \
        FX_MFMA(CUR.a1, CUR.b1, 3, 2); FX_RD2(NXT.a2, 2, na_, 8704);  FX_SB;                              \
        FX_MFMA(CUR.a1, CUR.b1, 3, 3); FX_RD2(NXT.a2, 3, na_, 8704);  FX_SB;                              \
        FX_MFMA(CUR.a1, CUR.b2, 0, 0); load_one((T) + FX_STAGES, 0);  FX_SB;                              \
        FX_MFMA(CUR.a1, CUR.b2, 0, 1); load_one((T) + FX_STAGES, 1);  FX_SB;                              \
        FX_MFMA(CUR.a1, CUR.b2, 0, 2); load_one((T) + FX_STAGES, 2);  FX_SB;                              \
        FX_MFMA(CUR.a1, CUR.b2, 0, 3); load_one((T) + FX_STAGES, 3);  FX_SB;                              \
        FX_MFMA(CUR.a1, CUR.b2, 1, 0); load_one((T) + FX_STAGES, 4);  FX_SB;                              \
        FX_MFMA(CUR.a1, CUR.b2, 1, 1); load_one((T) + FX_STAGES, 5);  FX_SB;                              \
        FX_MFMA(CUR.a1, CUR.b2, 1, 2); load_one((T) + FX_STAGES, 6);  FX_SB;                              \
        FX_MFMA(CUR.a1, CUR.b2, 1, 3); load_one((T) + FX_STAGES, 7);  FX_SB;                              \
        FX_MFMA(CUR.a1, CUR.b2, 2, 0); FX_MFMA(CUR.a1, CUR.b2, 2, 1); FX_MFMA(CUR.a1, CUR.b2, 2, 2);      \
        FX_MFMA(CUR.a1, CUR.b2, 2, 3); FX_MFMA(CUR.a1, CUR.b2, 3, 0); FX_MFMA(CUR.a1, CUR.b2, 3, 1);      \
        FX_MFMA(CUR.a1, CUR.b2, 3, 2); FX_MFMA(CUR.a1, CUR.b2, 3, 3);                                     \
        FX_MFMA(CUR.a2, CUR.b1, 0, 0); FX_MFMA(CUR.a2, CUR.b1, 0, 1); FX_MFMA(CUR.a2, CUR.b1, 0, 2);      \
        FX_MFMA(CUR.a2, CUR.b1, 0, 3); FX_MFMA(CUR.a2, CUR.b1, 1, 0); FX_MFMA(CUR.a2, CUR.b1, 1, 1);      \
        FX_MFMA(CUR.a2, CUR.b1, 1, 2); FX_MFMA(CUR.a2, CUR.b1, 1, 3); FX_MFMA(CUR.a2, CUR.b1, 2, 0);      \
        FX_MFMA(CUR.a2, CUR.b1, 2, 1); FX_MFMA(CUR.a2, CUR.b1, 2, 2); FX_MFMA(CUR.a2, CUR.b1, 2, 3);      \
        FX_MFMA(CUR.a2, CUR.b1, 3, 0); FX_MFMA(CUR.a2, CUR.b1, 3, 1); FX_MFMA(CUR.a2, CUR.b1, 3, 2);      \
        FX_MFMA(CUR.a2, CUR.b1, 3, 3);                                                                    \
        FX_SB;                                                                                           \
    } while (0)

    FxFrags f0, f1;
    for (int s = 0; s < FX_STAGES; ++s)
#pragma unroll
        for (int i = 0; i < 8; ++i) load_one(s, i);
    asm volatile("s_waitcnt vmcnt(24)" ::: "memory");       // stage 0 has landed: three younger stages may be out
    __syncthreads();
    FX_RD2(f0.a1, 0, offA, 0);    FX_RD2(f0.a1, 1, offA, 0);    FX_RD2(f0.a1, 2, offA, 0);    FX_RD2(f0.a1, 3, offA, 0);
    FX_RD2(f0.a2, 0, offA, 8704); FX_RD2(f0.a2, 1, offA, 8704); FX_RD2(f0.a2, 2, offA, 8704); FX_RD2(f0.a2, 3, offA, 8704);
    FX_RD2(f0.b1, 0, offB, 0);    FX_RD2(f0.b1, 1, offB, 0);    FX_RD2(f0.b1, 2, offB, 0);    FX_RD2(f0.b1, 3, offB, 0);
    FX_RD2(f0.b2, 0, offB, 8704); FX_RD2(f0.b2, 1, offB, 8704); FX_RD2(f0.b2, 2, offB, 8704); FX_RD2(f0.b2, 3, offB, 8704);
    // the launcher makes K a multiple of 32: stages come in pairs, the two fragment sets change roles
    for (int t = 0; t < nst; t += 2) {
        FX_STAGE_BODY(f0, f1, t);
        FX_STAGE_BODY(f1, f0, t + 1);
    }
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
#undef FX_STAGE_BODY
#undef FX_SB
#undef FX_MFMA
#undef FX_FRAG
#undef FX_RD2
#undef FX_RD

    // out = alpha / (sA sB) * acc + beta * Z.  Accumulator register v of lane l holds row 8 (v / 4) + 4 (l / 32) +
    // v % 4 and column l % 32 of its 32 x 32 sub-tile; the rows of Z are requested eight at a time.
    const long wm0 = m0 + wm * 128, wn0 = n0 + wn * 128;
    const int l32 = lane & 31, khalf = lane >> 5;
    if (P.split > 1) {
        // the slice's unscaled partial sums; scaling, Z and the sum over slices are the reduction kernel's
        float *pp = P.partial + (long)slice * P.M * P.N;
#pragma unroll
        for (int a = 0; a < 4; ++a)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const long m = wm0 + 32 * a + 8 * (v / 4) + 4 * khalf + (v % 4);
                float *op = pp + m * P.N + wn0 + l32;
#pragma unroll
                for (int b = 0; b < 4; ++b) op[32 * b] = acc[a][b][v];
            }
        return;
    }
    const float sc = P.alpha * (1.0f / P.scaleA[0]) * (1.0f / P.scaleB[0]);
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int v0 = 0; v0 < 16; v0 += 8) {
            float z[8][4];
            if (P.Z) {
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int v = v0 + u;
                    const long m = wm0 + 32 * a + 8 * (v / 4) + 4 * khalf + (v % 4);
                    const float *zp = P.Z + m * P.ldz + wn0 + l32;
#pragma unroll
                    for (int b = 0; b < 4; ++b) z[u][b] = zp[32 * b];
                }
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int v = v0 + u;
                const long m = wm0 + 32 * a + 8 * (v / 4) + 4 * khalf + (v % 4);
                float *op = P.out + m * P.ldo + wn0 + l32;
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    float r = sc * acc[a][b][v];
                    if (P.Z) r += P.beta * z[u][b];
                    op[32 * b] = r;
                }
            }
        }
}

// out = alpha / (sA sB) * sum over slices of partial + beta * Z  (four columns per thread)
__global__ __launch_bounds__(256) void f16x3_reduce_kernel(const float *__restrict__ partial, int split, long M, long N,
                                                          const float *__restrict__ scaleA,
                                                          const float *__restrict__ scaleB, float alpha, float beta,
                                                          const float *__restrict__ Z, long ldz, float *__restrict__ out,
                                                          long ldo) {
    const float sc = alpha * (1.0f / scaleA[0]) * (1.0f / scaleB[0]);
    const long n4 = N / 4, total = M * n4;
    for (long e = (long)blockIdx.x * 256 + threadIdx.x; e < total; e += (long)gridDim.x * 256) {
        const long m = e / n4, c = (e - m * n4) * 4;
        floatx4 sum = *(const floatx4 *)(partial + m * N + c);
        for (int q = 1; q < split; ++q) {
            const floatx4 t = *(const floatx4 *)(partial + (long)q * M * N + m * N + c);
            sum.x += t.x; sum.y += t.y; sum.z += t.z; sum.w += t.w;
        }
        floatx4 r = {sc * sum.x, sc * sum.y, sc * sum.z, sc * sum.w};
        if (Z) {
            const floatx4 z = *(const floatx4 *)(Z + m * ldz + c);
            r.x += beta * z.x; r.y += beta * z.y; r.z += beta * z.z; r.w += beta * z.w;
        }
        *(floatx4 *)(out + m * ldo + c) = r;
    }
}

// largest |x| of a [rows][cols] fp32 matrix (leading dimension ld) as the bit pattern of the float, by atomic max
// (the patterns of non-negative floats order like the floats); the slot starts at zero
__global__ __launch_bounds__(256) void amax_kernel(const float *__restrict__ src, long rows, long cols, long ld,
                                                  unsigned *__restrict__ slot) {
    const long c4 = cols / 4, total = rows * c4;
    const bool dense = ld == cols;                         // then the matrix is one run of floats: no row arithmetic
    unsigned best = 0;
    for (long e = (long)blockIdx.x * 256 + threadIdx.x; e < total; e += (long)gridDim.x * 256) {
        long off = 4 * e;
        if (!dense) {
            const long r = e / c4;
            off = r * ld + (e - r * c4) * 4;
        }
        const floatx4 x = *(const floatx4 *)(src + off);
        best = max(best, __float_as_uint(fabsf(x.x)));
        best = max(best, __float_as_uint(fabsf(x.y)));
        best = max(best, __float_as_uint(fabsf(x.z)));
        best = max(best, __float_as_uint(fabsf(x.w)));
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) best = max(best, (unsigned)__shfl_xor((int)best, o));
    __shared__ unsigned part[4];
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = best;
    __syncthreads();
    if (threadIdx.x == 0) {
        best = max(max(part[0], part[1]), max(part[2], part[3]));
        if (best > __atomic_load_n(slot, __ATOMIC_RELAXED)) atomicMax(slot, best);   // few blocks raise the maximum
    }
}

// hi = fp16(s x), lo = fp16(s x - hi) with s the power of two that brings the matrix's largest entry into
// [2^14, 2^15) (1 for a zero or non-finite matrix); s is left in scale_out[0] for the product's epilogue
__global__ __launch_bounds__(256) void split_f16_kernel(const float *__restrict__ src, long rows, long cols, long ld,
                                                       const unsigned *__restrict__ amax_slot,
                                                       unsigned short *__restrict__ hi, unsigned short *__restrict__ lo,
                                                       float *__restrict__ scale_out, unsigned *__restrict__ zero_slot) {
    const unsigned bits = amax_slot[0];
    const int ex = (int)((bits >> 23) & 0xffu);
    float s = 1.0f;
    if (ex > 0 && ex < 255) {
        int se = 14 - (ex - 127);                          // exponent of s
        se = se > 120 ? 120 : (se < -120 ? -120 : se);
        s = __uint_as_float((unsigned)(se + 127) << 23);
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        scale_out[0] = s;
        if (zero_slot) zero_slot[0] = 0;                   // the slot of the NEXT matrix's maximum (nobody reads it now)
    }
    const long c8 = cols / 8, total = rows * c8;
    const bool dense = ld == cols;
    for (long e = (long)blockIdx.x * 256 + threadIdx.x; e < total; e += (long)gridDim.x * 256) {
        long r = 0, c = 8 * e, off = 8 * e;
        if (!dense) {
            r = e / c8;
            c = (e - r * c8) * 8;
            off = r * ld + c;
        }
        const floatx4 x0 = *(const floatx4 *)(src + off);
        const floatx4 x1 = *(const floatx4 *)(src + off + 4);
        const float x[8] = {x0.x, x0.y, x0.z, x0.w, x1.x, x1.y, x1.z, x1.w};
        halfx8 h, l;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const float y = x[i] * s;
            const _Float16 top = (_Float16)y;
            h[i] = top;
            l[i] = (_Float16)(y - (float)top);
        }
        *(uintx4 *)(hi + r * cols + c) = __builtin_bit_cast(uintx4, h);
        *(uintx4 *)(lo + r * cols + c) = __builtin_bit_cast(uintx4, l);
    }
}

}  // namespace

// Slices of the k axis for an M x N x K product: 1 when the 256 x 256 tiles alone fill the chip (200 or more), else
// the smallest of 2, 4, 8 that gets (tiles x slices) there with 512 or more k-rows per slice; 0: not for this kernel.
int admmq_gemm_f16x3_split(int64_t M, int64_t N, int64_t K) {
    if (M < FX_TILE || N < FX_TILE || M % FX_TILE || N % FX_TILE || K < 2 * FX_KT || K % (2 * FX_KT)) return 0;
    const int64_t tiles = (M / FX_TILE) * (N / FX_TILE);
    for (int sp = 1; sp <= 8; sp *= 2) {
        if (K % (2 * FX_KT * sp) != 0 || (sp > 1 && K / sp < 512)) return 0;
        if (tiles * sp >= 200) return sp;
    }
    return 0;
}

namespace {
// How a product goes out.  A tile count just above a multiple of the 256 compute units would leave the last launch
// round nearly empty (4096 x 5120: 320 tiles, two rounds for 1.25 rounds of work): then the leading columns that
// fill whole rounds are one launch and the remaining columns a product of their own with the contraction in
// slices.  Costs in launch rounds of whole-k tiles; a sliced part pays 0.15 for its partial sums.
struct FxPlan {
    int64_t n_head = 0;        // columns of the first (or only) launch
    int sp_head = 0;           // its slices; 0: the kernel does not take this product
    int64_t n_tail = 0;        // columns of the second launch (0: none)
    int sp_tail = 0;
};
double fx_rounds(int64_t tiles, int sp) { return (double)((tiles * sp + 255) / 256) / sp + (sp > 1 ? 0.15 : 0.0); }
FxPlan fx_plan(int64_t M, int64_t N, int64_t K) {
    FxPlan pl;
    pl.sp_head = admmq_gemm_f16x3_split(M, N, K);
    if (pl.sp_head == 0) return pl;
    pl.n_head = N;
    const int64_t tm = M / FX_TILE, tn = N / FX_TILE, t = tm * tn;
    if (pl.sp_head == 1 && t > 256 && t % 256 != 0) {
        const int64_t c_full = (t / 256) * 256 / tm;              // column tiles that fill whole rounds
        if (c_full >= 1 && c_full < tn) {
            const int64_t n_head = c_full * FX_TILE;
            const int sp_tail = admmq_gemm_f16x3_split(M, N - n_head, K);
            if (sp_tail > 0 && admmq_gemm_f16x3_split(M, n_head, K) == 1) {
                const double whole = fx_rounds(t, 1);
                const double parts = fx_rounds(c_full * tm, 1) + fx_rounds((tn - c_full) * tm, sp_tail);
                if (parts < 0.93 * whole) {
                    pl.n_head = n_head;
                    pl.n_tail = N - n_head;
                    pl.sp_tail = sp_tail;
                }
            }
        }
    }
    return pl;
}
}  // namespace

bool admmq_gemm_f16x3_ok(int64_t M, int64_t N, int64_t K) { return fx_plan(M, N, K).sp_head > 0; }
size_t admmq_gemm_f16x3_partial_bytes(int64_t M, int64_t N, int64_t K) {
    const FxPlan pl = fx_plan(M, N, K);
    size_t need = 0;
    if (pl.sp_head > 1) need = (size_t)pl.sp_head * (size_t)M * (size_t)pl.n_head * 4;
    if (pl.sp_tail > 1) {
        const size_t t = (size_t)pl.sp_tail * (size_t)M * (size_t)pl.n_tail * 4;
        if (t > need) need = t;
    }
    return need;
}

// hi, lo: [rows][cols] fp16 (dense rows); slots: 2 words of device scratch (word 0: largest |x| as bits, zero on
// entry; word 1: receives s).  next_slots (may be NULL): the slots of the split that follows on this stream; its
// word 0 is zeroed here, which saves that split a launch.  have_max: the producer of src has already accumulated
// the largest |x| into word 0 (projection and tridiagonal solve do so on request), no reduction pass is needed.
admmq_status admmq_k_split_f16(admmq_ctx *ctx, const float *src, int64_t rows, int64_t cols, int64_t ld, void *hi,
                               void *lo, void *slots, void *next_slots, bool have_max) {
    if (cols % 8 != 0 || ld % 4 != 0 || ((uintptr_t)src & 15) || ((uintptr_t)hi & 15) || ((uintptr_t)lo & 15) ||
        next_slots == slots)
        return ADMMQ_ERR_PARAM;
    const long work = rows * (cols / 8);
    const unsigned blocks = (unsigned)(work / 256 + 1 < 2048 ? work / 256 + 1 : 2048);
    if (!have_max)
        hipLaunchKernelGGL(amax_kernel, dim3(blocks), dim3(256), 0, ctx->stream, src, (long)rows, (long)cols, (long)ld,
                           (unsigned *)slots);
    hipLaunchKernelGGL(split_f16_kernel, dim3(blocks), dim3(256), 0, ctx->stream, src, (long)rows, (long)cols, (long)ld,
                       (const unsigned *)slots, (unsigned short *)hi, (unsigned short *)lo, (float *)slots + 1,
                       (unsigned *)next_slots);
    ADMMQ_HIP(hipGetLastError());
    return ADMMQ_OK;
}

namespace {
// one launch (plus the reduction of its slices): columns [0, N) of B1 / B2 rows of length ldb
admmq_status fx_launch(admmq_ctx *ctx, const void *A1, const void *A2, const void *slotsA, const unsigned short *B1,
                       const unsigned short *B2, const void *slotsB, int64_t ldb, int64_t M, int64_t N, int64_t K,
                       int split, float alpha, float beta, const float *Z, int64_t ldz, float *out, int64_t ldo,
                       float *partial) {
    if (split < 1 || (split > 1 && !partial)) return ADMMQ_ERR_PARAM;
    if (split > 1 && (N % 4 || ldz % 4 || ldo % 4 || ((uintptr_t)out & 15) || (Z && ((uintptr_t)Z & 15))))
        return ADMMQ_ERR_PARAM;
    F16x3Params P;
    P.split = split; P.k_chunk = K / split; P.partial = partial;
    P.A1 = (const unsigned short *)A1; P.A2 = (const unsigned short *)A2;
    P.B1 = B1; P.B2 = B2; P.ldb = ldb;
    P.scaleA = (const float *)slotsA + 1; P.scaleB = (const float *)slotsB + 1;
    P.M = M; P.N = N; P.K = K; P.alpha = alpha; P.beta = beta; P.Z = Z; P.ldz = ldz; P.out = out; P.ldo = ldo;
    P.tiles_m = (int)(M / FX_TILE); P.tiles_n = (int)(N / FX_TILE);
    static unsigned long long lds_allowed = 0;
    ADMMQ_HIP(admmq_allow_lds((const void *)gemm_f16x3_kernel, FX_LDS, ctx->device, &lds_allowed));
    hipLaunchKernelGGL(gemm_f16x3_kernel, dim3((unsigned)(P.tiles_m * P.tiles_n * split)), dim3(256), FX_LDS,
                       ctx->stream, P);
    if (split > 1) {
        const long work = M * (N / 4);
        const unsigned blocks = (unsigned)(work / 256 + 1 < 4096 ? work / 256 + 1 : 4096);
        hipLaunchKernelGGL(f16x3_reduce_kernel, dim3(blocks), dim3(256), 0, ctx->stream, partial, split, (long)M,
                           (long)N, P.scaleA, P.scaleB, alpha, beta, Z, (long)ldz, out, (long)ldo);
    }
    ADMMQ_HIP(hipGetLastError());
    return ADMMQ_OK;
}
}  // namespace

admmq_status admmq_gemm_f16x3(admmq_ctx *ctx, const void *A1, const void *A2, const void *slotsA, const void *B1,
                              const void *B2, const void *slotsB, int64_t M, int64_t N, int64_t K, float alpha,
                              float beta, const float *Z, int64_t ldz, float *out, int64_t ldo, float *partial) {
    const FxPlan pl = fx_plan(M, N, K);
    if (pl.sp_head < 1) return ADMMQ_ERR_PARAM;
    const unsigned short *b1 = (const unsigned short *)B1, *b2 = (const unsigned short *)B2;
    ADMMQ_TRY(fx_launch(ctx, A1, A2, slotsA, b1, b2, slotsB, N, M, pl.n_head, K, pl.sp_head, alpha, beta, Z, ldz, out,
                        ldo, partial));
    if (pl.n_tail > 0)
        ADMMQ_TRY(fx_launch(ctx, A1, A2, slotsA, b1 + pl.n_head, b2 + pl.n_head, slotsB, N, M, pl.n_tail, K, pl.sp_tail,
                            alpha, beta, Z ? Z + pl.n_head : nullptr, ldz, out + pl.n_head, ldo, partial));
    return ADMMQ_OK;
}
