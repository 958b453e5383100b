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

    // Stage s of this block: tokens kbeg + 32 s .. +31; wave w brings chunks w, w+4, w+8, w+12 of both operands.
    // Stages past the slice's end are loaded all the same, from the last real stage's rows, into a ring buffer
    // nobody reads any more: every stage then costs every wave eight loads, the loop has no branches and one
    // constant in its wait for the loads.
    const unsigned short *gA = P.X + (kbeg + (lane >> 5)) * P.ldx + m0 + (lane & 31) * 8;
    const unsigned short *gB = P.X + (kbeg + (lane >> 5)) * P.ldx + n0 + (lane & 31) * 8;
    // load number i (0..3: operand A, 4..7: operand B) of stage s
    auto load_one = [&](int s, int i) {
        const long row = (long)min(s, nst - 1) * HB_KT;
        unsigned char *dst = hb_lds + (s % HB_STAGES) * HB_STAGE + (i >> 2) * HB_OPERAND;
        const int c = wave + 4 * (i & 3);
        __builtin_amdgcn_global_load_lds(((i >> 2) ? gB : gA) + (row + 2 * c) * P.ldx,
                                         (__attribute__((address_space(3))) void *)(dst + c * HB_CHUNK), 16, 0, 0);
    };

    // Transposing read: in every group of 16 lanes, source lane 4 j + q points at 8 bytes (4 channels) of token j;
    // lane i of the group receives channel i of tokens j = 0..3.  Lane l feeds channel l % 32 of a 32-wide
    // sub-tile and the k-block l / 32; read h of step kk takes tokens 16 kk + 8 (l / 32) + 2 j + h: the same
    // assignment of tokens to operand slots on both sides of the product, which is all the sum over k needs.
    //
    // The reads are written as assembly: a read the compiler can see is made to wait for EVERY outstanding
    // global -> LDS load (it cannot tell the ring's buffers apart), which would undo the ring.  The waits for the
    // loads and for the reads are therefore placed by hand (vmcnt below, frags_ready).
    const int grp = lane >> 4, jrow = (lane & 15) >> 2, q = lane & 3;
    const int lane_off = (4 * (grp >> 1) + jrow) * HB_CHUNK + (16 * (grp & 1) + 4 * q) * 2;
    const unsigned lds0 = (unsigned)(unsigned long)(__attribute__((address_space(3))) unsigned char *)hb_lds;
    const unsigned offA = lds0 + lane_off + wm * 256;      // 128 channels = 256 bytes per quadrant
    const unsigned offB = lds0 + HB_OPERAND + lane_off + wn * 256;
    struct Frags {
        uintx2 a[4][2], b[4][2];
    };
#define HB_RD(dst, addr, off) \
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:" #off : "=v"(dst) : "v"(addr) : "memory")
    // the two reads (tokens of even and of odd parity) that make sub-tile I's operand of the step at offset K0
#define HB_RD2(X, I, addr, K0)                    \
    do {                                          \
        HB_RD(X[I][0], addr, K0 + 64 * I);        \
        HB_RD(X[I][1], addr, K0 + 64 * I + 512);  \
    } while (0)
#define HB_FRAG(X) __builtin_bit_cast(bf16x8, __builtin_shufflevector(X[0], X[1], 0, 1, 2, 3))
#define HB_MFMA(F, A_, B_) \
    acc[A_][B_] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(HB_FRAG(F.a[A_]), HB_FRAG(F.b[B_]), acc[A_][B_], 0, 0, 0)
#define HB_SB __builtin_amdgcn_sched_barrier(0)
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

    Frags f0, f1;
    if (nst > 0) {
        for (int s = 0; s < HB_STAGES; ++s)
#pragma unroll
            for (int i = 0; i < HB_LOADS; ++i) load_one(s, i);
        asm volatile("s_waitcnt vmcnt(24)" ::: "memory");   // stage 0 has landed: three younger stages may be out
        __syncthreads();
        HB_RD2(f0.a, 0, offA, 0); HB_RD2(f0.a, 1, offA, 0); HB_RD2(f0.a, 2, offA, 0); HB_RD2(f0.a, 3, offA, 0);
        HB_RD2(f0.b, 0, offB, 0); HB_RD2(f0.b, 1, offB, 0); HB_RD2(f0.b, 2, offB, 0); HB_RD2(f0.b, 3, offB, 0);
    }
    // Per stage, two steps of 16 products.  Everything else is issued in the shadow of the products, one piece
    // after each: during the first step the reads of the second step's fragments; then the wave waits for the next
    // stage's loads and passes the barrier (after which this stage's buffer is free); during the second step the
    // reads of the next stage's first fragments and the eight loads of the stage four ahead into the freed buffer.
    for (int t = 0; t < nst; ++t) {
        const unsigned cur = (unsigned)((t % HB_STAGES) * HB_STAGE);
        const unsigned nxt = (unsigned)(((t + 1) % HB_STAGES) * HB_STAGE);
        const unsigned pa = offA + cur, pb = offB + cur, na = offA + nxt, nb = offB + nxt;
        frags_ready(f0);
        HB_SB;
        HB_MFMA(f0, 0, 0); HB_RD2(f1.a, 0, pa, 8704); HB_SB;      // 8 chunks on: tokens 16..31 of the stage
        HB_MFMA(f0, 0, 1); HB_RD2(f1.b, 0, pb, 8704); HB_SB;
        HB_MFMA(f0, 0, 2); HB_RD2(f1.b, 1, pb, 8704); HB_SB;
        HB_MFMA(f0, 0, 3); HB_RD2(f1.b, 2, pb, 8704); HB_SB;
        HB_MFMA(f0, 1, 0); HB_RD2(f1.b, 3, pb, 8704); HB_SB;
        HB_MFMA(f0, 1, 1); HB_RD2(f1.a, 1, pa, 8704); HB_SB;
        HB_MFMA(f0, 1, 2); HB_RD2(f1.a, 2, pa, 8704); HB_SB;
        HB_MFMA(f0, 1, 3); HB_RD2(f1.a, 3, pa, 8704); HB_SB;
        HB_MFMA(f0, 2, 0); HB_MFMA(f0, 2, 1); HB_MFMA(f0, 2, 2); HB_MFMA(f0, 2, 3);
        HB_MFMA(f0, 3, 0); HB_MFMA(f0, 3, 1); HB_MFMA(f0, 3, 2); HB_MFMA(f0, 3, 3);
        HB_SB;
        asm volatile("s_waitcnt vmcnt(16)" ::: "memory");   // stage t+1 has landed: stages t+2, t+3 may be out
        frags_ready(f1);                                    // (also: this wave no longer reads stage t's buffer)
        __syncthreads();
        HB_SB;
        HB_MFMA(f1, 0, 0); HB_RD2(f0.a, 0, na, 0); HB_SB;
        HB_MFMA(f1, 0, 1); HB_RD2(f0.b, 0, nb, 0); HB_SB;
        HB_MFMA(f1, 0, 2); HB_RD2(f0.b, 1, nb, 0); HB_SB;
        HB_MFMA(f1, 0, 3); HB_RD2(f0.b, 2, nb, 0); HB_SB;
        HB_MFMA(f1, 1, 0); HB_RD2(f0.b, 3, nb, 0); HB_SB;
        HB_MFMA(f1, 1, 1); HB_RD2(f0.a, 1, na, 0); HB_SB;
        HB_MFMA(f1, 1, 2); HB_RD2(f0.a, 2, na, 0); HB_SB;
        HB_MFMA(f1, 1, 3); HB_RD2(f0.a, 3, na, 0); HB_SB;
        HB_MFMA(f1, 2, 0); load_one(t + HB_STAGES, 0); HB_SB;
        HB_MFMA(f1, 2, 1); load_one(t + HB_STAGES, 1); HB_SB;
        HB_MFMA(f1, 2, 2); load_one(t + HB_STAGES, 2); HB_SB;
        HB_MFMA(f1, 2, 3); load_one(t + HB_STAGES, 3); HB_SB;
        HB_MFMA(f1, 3, 0); load_one(t + HB_STAGES, 4); HB_SB;
        HB_MFMA(f1, 3, 1); load_one(t + HB_STAGES, 5); HB_SB;
        HB_MFMA(f1, 3, 2); load_one(t + HB_STAGES, 6); HB_SB;
        HB_MFMA(f1, 3, 3); load_one(t + HB_STAGES, 7); HB_SB;
    }
    // nothing of the ring is in flight when the wave retires (the last stages' loads were never read)
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
#undef HB_SB
#undef HB_MFMA
#undef HB_FRAG
#undef HB_RD2
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
    static unsigned long long lds_allowed = 0;
    ADMMQ_HIP(admmq_allow_lds((const void *)hessian_bf16_kernel, HB_LDS, ctx->device, &lds_allowed));
    hipLaunchKernelGGL(hessian_bf16_kernel, dim3((unsigned)(hp.per_xcd * 8)), dim3(256), HB_LDS, ctx->stream, hp);
    ADMMQ_HIP(hipGetLastError());
    return ADMMQ_OK;
}
