// Hessian accumulation (Sec. 3.1, H = X^T X) from bf16 activations on the bf16 matrix cores of gfx950.
//
// The products of two bf16 values are exact in fp32 and v_mfma_f32_32x32x16_bf16 accumulates in fp32, so the
// result differs from the fp32 product of the widened values only by the order of the additions.  X is
// [rows][n] with the channel index contiguous, while the matrix-core operands want, per lane, eight consecutive
// k (token) values of one channel: stages of 32 tokens x 256 channels go from global memory straight into LDS as
// they are stored, and the transposing LDS read (ds_read_b64_tr_b16) hands every lane four tokens of its channel.
//
// Work item = (token slice, 256 x 256 tile of the lower triangle); a block writes its tile of the slice's
// partial sum, the caller adds the slices and mirrors the triangle.
#include "common.h"

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned uintx2 __attribute__((ext_vector_type(2)));

namespace {

constexpr int HB_TILE = 256;           // channels per tile side
constexpr int HB_KT = 32;              // tokens per stage
constexpr int HB_STAGES = 4;           // stages in the LDS ring
// A 1 KB chunk holds two consecutive tokens x 256 channels (what one wave-wide direct load delivers: lane l lands
// at chunk + 16 l); chunks are 1088 bytes apart so that the four tokens a transposing read gathers sit in four
// different 64-byte bank windows.
constexpr int HB_CHUNK = 1024 + 64;
constexpr int HB_CHUNKS = HB_KT / 2;                       // per operand and stage
constexpr int HB_OPERAND = HB_CHUNKS * HB_CHUNK;           // 17408 B
constexpr int HB_STAGE = 2 * HB_OPERAND;                   // 34816 B
constexpr int HB_LDS = HB_STAGES * HB_STAGE;               // 139264 B
constexpr int HB_LOADS = 2 * HB_CHUNKS / 4;                // direct loads per wave and stage (8)

struct HessParams {
    const unsigned short *X;
    long ldx;
    long n;
    long k_main;           // tokens handled here (a multiple of HB_KT)
    long k_chunk;          // tokens per slice (a multiple of HB_KT)
    int tiles_m;           // n / 256
    int tiles;             // tiles_m (tiles_m + 1) / 2
    int split;
    long total;            // tiles * split
    long per_xcd;          // ceil(total / 8)
    float *P;
    long slice_stride;
};

__device__ inline void wait_loads(int later_stages) {
    // outstanding direct loads allowed: those of `later_stages` younger stages (8 per stage and wave)
    if (later_stages >= 2) asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
    else if (later_stages == 1) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
    else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}

__global__ __launch_bounds__(256, 1) void hessian_bf16_kernel(HessParams P) {
    extern __shared__ __attribute__((aligned(16))) unsigned char hb_lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave & 1, wn = wave >> 1;               // the wave's 128 x 128 quadrant of the tile

    // Blocks whose ids agree mod 8 share an XCD (and its L2): each XCD walks a contiguous range of the
    // slice-major work list, so the blocks it runs at one time are neighbouring tiles of one token slice.
    const long w = (long)(blockIdx.x & 7) * P.per_xcd + (blockIdx.x >> 3);
    if (w >= P.total) return;
    const int slice = (int)(w / P.tiles);
    const int tile_id = (int)(w - (long)slice * P.tiles);
    // tile_id enumerates pairs tm >= tn row by row of the triangle: id = tm (tm + 1) / 2 + tn
    int tm = (int)((sqrtf(8.f * (float)tile_id + 1.f) - 1.f) * 0.5f);
    while ((long)(tm + 1) * (tm + 2) / 2 <= tile_id) ++tm;
    while ((long)tm * (tm + 1) / 2 > tile_id) --tm;
    const int tn = tile_id - tm * (tm + 1) / 2;
    const long m0 = (long)tm * HB_TILE, n0 = (long)tn * HB_TILE;
    const long kbeg = min(P.k_main, (long)slice * P.k_chunk);
    const long kend = min(P.k_main, kbeg + P.k_chunk);
    const int nst = (int)((kend - kbeg) / HB_KT);

    floatx16 acc[4][4];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

    // stage s of this block: tokens kbeg + 32 s .. +31; wave w brings chunks w, w+4, w+8, w+12 of both operands
    const unsigned short *gA = P.X + (kbeg + (lane >> 5)) * P.ldx + m0 + (lane & 31) * 8;
    const unsigned short *gB = P.X + (kbeg + (lane >> 5)) * P.ldx + n0 + (lane & 31) * 8;
    auto issue = [&](int s) {
        unsigned char *dst = hb_lds + (s % HB_STAGES) * HB_STAGE;
        const long row = (long)s * HB_KT;
#pragma unroll
        for (int i = 0; i < HB_CHUNKS / 4; ++i) {
            const int c = wave + 4 * i;
            __builtin_amdgcn_global_load_lds(gA + (row + 2 * c) * P.ldx,
                                             (__attribute__((address_space(3))) void *)(dst + c * HB_CHUNK), 16, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < HB_CHUNKS / 4; ++i) {
            const int c = wave + 4 * i;
            __builtin_amdgcn_global_load_lds(
                gB + (row + 2 * c) * P.ldx,
                (__attribute__((address_space(3))) void *)(dst + HB_OPERAND + c * HB_CHUNK), 16, 0, 0);
        }
    };

    // Transposing read: in every group of 16 lanes, source lane 4 j + q points at 8 bytes (4 channels) of token j;
    // lane i of the group receives channel i of tokens j = 0..3.  Lane l feeds channel l % 32 of a 32-wide
    // sub-tile and the k-block l / 32; read h of step kk takes tokens 16 kk + 8 (l / 32) + 2 j + h: the same
    // assignment of tokens to operand slots on both sides of the product, which is all the sum over k needs.
    //
    // The reads are written as assembly: a read the compiler can see is made to wait for EVERY outstanding
    // global -> LDS load (it cannot tell the ring's buffers apart), which would undo the ring.  The waits for the
    // loads and for the reads are therefore placed by hand (wait_loads, frags_ready).
    const int grp = lane >> 4, jrow = (lane & 15) >> 2, q = lane & 3;
    const int lane_off = (4 * (grp >> 1) + jrow) * HB_CHUNK + (16 * (grp & 1) + 4 * q) * 2;
    const unsigned lds0 = (unsigned)(unsigned long)(__attribute__((address_space(3))) unsigned char *)hb_lds;
    const unsigned offA = lds0 + lane_off + wm * 256;      // 128 channels = 256 bytes per quadrant
    const unsigned offB = lds0 + HB_OPERAND + lane_off + wn * 256;
#define HB_RD(dst, addr, off) \
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:" #off : "=v"(dst) : "v"(addr) : "memory")
    // fragments of step KK (0 or 1) of the stage whose LDS byte offsets are pa (A side) and pb (B side)
#define HB_READ_STEP(F, pa, pb, K0)                                                                    \
    do {                                                                                               \
        HB_RD(F.a[0][0], pa, K0 + 0);   HB_RD(F.a[0][1], pa, K0 + 512);                                \
        HB_RD(F.a[1][0], pa, K0 + 64);  HB_RD(F.a[1][1], pa, K0 + 576);                                \
        HB_RD(F.a[2][0], pa, K0 + 128); HB_RD(F.a[2][1], pa, K0 + 640);                                \
        HB_RD(F.a[3][0], pa, K0 + 192); HB_RD(F.a[3][1], pa, K0 + 704);                                \
        HB_RD(F.b[0][0], pb, K0 + 0);   HB_RD(F.b[0][1], pb, K0 + 512);                                \
        HB_RD(F.b[1][0], pb, K0 + 64);  HB_RD(F.b[1][1], pb, K0 + 576);                                \
        HB_RD(F.b[2][0], pb, K0 + 128); HB_RD(F.b[2][1], pb, K0 + 640);                                \
        HB_RD(F.b[3][0], pb, K0 + 192); HB_RD(F.b[3][1], pb, K0 + 704);                                \
    } while (0)
    struct Frags {
        uintx2 a[4][2], b[4][2];
    };
    // every read issued so far has delivered; naming the registers ties the products that use them to this wait
    auto frags_ready = [](Frags &f) {
        asm volatile("s_waitcnt lgkmcnt(0)"
                     : "+v"(f.a[0][0]), "+v"(f.a[0][1]), "+v"(f.a[1][0]), "+v"(f.a[1][1]), "+v"(f.a[2][0]),
                       "+v"(f.a[2][1]), "+v"(f.a[3][0]), "+v"(f.a[3][1]), "+v"(f.b[0][0]), "+v"(f.b[0][1]),
                       "+v"(f.b[1][0]), "+v"(f.b[1][1]), "+v"(f.b[2][0]), "+v"(f.b[2][1]), "+v"(f.b[3][0]),
                       "+v"(f.b[3][1])
                     :
                     : "memory");
    };
    auto mfma_step = [&](const Frags &f) {
        bf16x8 fa[4], fb[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            fa[i] = __builtin_bit_cast(bf16x8, __builtin_shufflevector(f.a[i][0], f.a[i][1], 0, 1, 2, 3));
            fb[i] = __builtin_bit_cast(bf16x8, __builtin_shufflevector(f.b[i][0], f.b[i][1], 0, 1, 2, 3));
        }
#pragma unroll
        for (int a = 0; a < 4; ++a)
#pragma unroll
            for (int b = 0; b < 4; ++b)
                acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[a], fb[b], acc[a][b], 0, 0, 0);
    };

    Frags f0, f1;
    if (nst > 0) {
        for (int s = 0; s < HB_STAGES && s < nst; ++s) issue(s);
        // stage 0 has landed once at most the loads of the (up to three) younger stages are outstanding
        const int younger = min(HB_STAGES - 1, nst - 1);
        if (younger >= 3) asm volatile("s_waitcnt vmcnt(24)" ::: "memory");
        else wait_loads(younger);
        __syncthreads();
        HB_READ_STEP(f0, offA, offB, 0);
    }
    // Per stage: the second step's fragments are read while the matrix cores work on the first; then the wave
    // waits for the next stage's loads, passes the barrier (after which this stage's buffer is free and is handed
    // to the loads of the stage four ahead), requests the next stage's first fragments and only then issues the
    // second step's products, so that neither the barrier nor the LDS latency leaves the pipe empty.
    for (int t = 0; t < nst; ++t) {
        const unsigned cur = (unsigned)((t % HB_STAGES) * HB_STAGE);
        const unsigned nxt = (unsigned)(((t + 1) % HB_STAGES) * HB_STAGE);
        const unsigned pa = offA + cur, pb = offB + cur;
        frags_ready(f0);
        HB_READ_STEP(f1, pa, pb, 8704);                   // 8 chunks on: tokens 16..31 of the stage
        mfma_step(f0);
        __builtin_amdgcn_sched_barrier(0);
        const bool more = t + 1 < nst;
        if (more) wait_loads(min(2, nst - 2 - t));
        frags_ready(f1);                                   // (also: this wave no longer reads the stage's buffer)
        __syncthreads();
        if (t + HB_STAGES < nst) issue(t + HB_STAGES);
        if (more) {
            const unsigned na = offA + nxt, nb = offB + nxt;
            HB_READ_STEP(f0, na, nb, 0);
        }
        mfma_step(f1);
        __builtin_amdgcn_sched_barrier(0);
    }
#undef HB_READ_STEP
#undef HB_RD

    // Accumulator register v of lane l holds row 8 (v / 4) + 4 (l / 32) + v % 4 and column l % 32 of its 32 x 32
    // sub-tile.
    float *outp = P.P + (long)slice * P.slice_stride;
    const long wm0 = m0 + wm * 128, wn0 = n0 + wn * 128;
    const int l32 = lane & 31, khalf = lane >> 5;
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const long m = wm0 + 32 * a + 8 * (v / 4) + 4 * khalf + (v % 4);
            float *op = outp + m * P.n + wn0 + l32;
#pragma unroll
            for (int b = 0; b < 4; ++b) op[32 * b] = acc[a][b][v];
        }
}

}  // namespace

bool admmq_hessian_bf16_ok(const void *X, int64_t n, int64_t ldx, int64_t rows) {
    return n >= HB_TILE && n % HB_TILE == 0 && ldx % 8 == 0 && ((uintptr_t)X & 15) == 0 && rows >= HB_KT;
}

int64_t admmq_hessian_bf16_main_rows(int64_t rows) { return rows / HB_KT * HB_KT; }

// P[s][i][j] (i >= j tiles) = sum over the tokens of slice s of X[k][i] X[k][j], for the first k_main tokens.
admmq_status admmq_hessian_bf16(admmq_ctx *ctx, const void *X, int64_t ldx, int64_t k_main, int64_t n, float *P,
                                int split, int64_t slice_stride) {
    if (!admmq_hessian_bf16_ok(X, n, ldx, k_main) || k_main % HB_KT != 0 || split < 1) return ADMMQ_ERR_PARAM;
    HessParams hp;
    hp.X = (const unsigned short *)X;
    hp.ldx = ldx;
    hp.n = n;
    hp.k_main = k_main;
    long kc = (k_main + split - 1) / split;
    hp.k_chunk = (kc + HB_KT - 1) / HB_KT * HB_KT;
    hp.tiles_m = (int)(n / HB_TILE);
    hp.tiles = hp.tiles_m * (hp.tiles_m + 1) / 2;
    hp.split = split;
    hp.total = (long)hp.tiles * split;
    hp.per_xcd = (hp.total + 7) / 8;
    hp.P = P;
    hp.slice_stride = slice_stride;
    static bool attr_set = false;
    if (!attr_set) {
        ADMMQ_HIP(hipFuncSetAttribute((const void *)hessian_bf16_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                      HB_LDS));
        attr_set = true;
    }
    hipLaunchKernelGGL(hessian_bf16_kernel, dim3((unsigned)(hp.per_xcd * 8)), dim3(256), HB_LDS, ctx->stream, hp);
    ADMMQ_HIP(hipGetLastError());
    return ADMMQ_OK;
}
