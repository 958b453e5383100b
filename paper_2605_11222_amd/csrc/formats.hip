// Projections of other quantization formats (Sec. 4.3): the D-update changes, the W- and V-updates do not.
//
//   dual grid : every entry carries a flag (1 = outlier); inliers and outliers of a group of an output channel sit
//               on separate uniform grids of the same bit width, each fitted by min/max over its own subset;
//   codebook  : every output channel has L = 2^bits strictly ascending levels; an entry goes to the nearest one
//               (the lower one when two are equally near); entries flagged as kept are unconstrained: their
//               projection is the target itself and their dual is zero.
//
// Arithmetic contract (bit-exact codes depend on it), single correctly rounded fp32 operations, no fused
// multiply-add; up to the unscaled target x it is the uniform projection's:
//   q = V*inv_rho; wt = W+q; x = wt*inv_d[i];
//   dual grid : (delta, inv_delta, z0) of the entry's subset; k = clamp(rint((x-z0)*inv_delta), 0, L-1);
//               xq = k*delta + z0
//   codebook  : k = #{ l : x > m_l },  m_l = (c_l + c_{l+1}) * 0.5f;  xq = c_k
//   Dn = d[i]*xq  (kept entry: Dn = wt);  r = W-Dn;  Vn = V + rho*r  (kept entry: 0);  Bn = Dn - Vn*inv_rho_next
#include "common.h"

typedef float floatx4 __attribute__((ext_vector_type(4)));

namespace {

__device__ inline double wave_sum(double v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o, 64);
    return v;
}

constexpr int FMT_ROWS = 16;      // rows per thread (4 columns each), as in the uniform projection pass

// ---- per-thread projector state: the parameters of 4 adjacent columns -------------------------------------------
struct DualGridCols {
    const float *scales, *inv_scales, *zeros;     // [2][n/g][p]
    long g, p, gstride;                           // gstride = (n/g) * p: distance between the two grids
    float levels;
    long grp = -1;
    float dl[2][4], idl[2][4], z0[2][4];

    __device__ void row(long i, long c0, int nc) {
        const long gi = i / g;
        if (gi == grp) return;
        grp = gi;
#pragma unroll
        for (int s = 0; s < 2; ++s)
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const long at = s * gstride + gi * p + c0 + c;
                dl[s][c] = c < nc ? scales[at] : 0.f;
                idl[s][c] = c < nc ? inv_scales[at] : 0.f;
                z0[s][c] = c < nc ? zeros[at] : 0.f;
            }
    }
    __device__ void project(float x, int c, int flag, float &k, float &xq) const {
        // selects, not an index: the parameters stay in registers
        const float z = flag ? z0[1][c] : z0[0][c];
        const float id = flag ? idl[1][c] : idl[0][c];
        const float dd = flag ? dl[1][c] : dl[0][c];
        const float t = __fmul_rn(__fsub_rn(x, z), id);
        k = fminf(fmaxf(rintf(t), 0.f), levels);
        xq = __fadd_rn(__fmul_rn(k, dd), z);
    }
};

template <int L>
struct CodebookCols {
    float lev[L][4], mid[L - 1][4];

    __device__ void load(const float *__restrict__ cb, long p, long c0, int nc, bool vec) {
#pragma unroll
        for (int l = 0; l < L; ++l) {
            if (vec) {
                const floatx4 t = *(const floatx4 *)(cb + (long)l * p + c0);
                lev[l][0] = t.x; lev[l][1] = t.y; lev[l][2] = t.z; lev[l][3] = t.w;
            } else {
#pragma unroll
                for (int c = 0; c < 4; ++c) lev[l][c] = c < nc ? cb[(long)l * p + c0 + c] : 0.f;
            }
        }
#pragma unroll
        for (int l = 0; l + 1 < L; ++l)
#pragma unroll
            for (int c = 0; c < 4; ++c) mid[l][c] = __fmul_rn(__fadd_rn(lev[l][c], lev[l + 1][c]), 0.5f);
    }
    // the midpoints ascend with l, so the last one below x names the level
    __device__ void project(float x, int c, float &k, float &xq) const {
        k = 0.f;
        xq = lev[0][c];
#pragma unroll
        for (int l = 0; l + 1 < L; ++l) {
            const bool up = x > mid[l][c];
            k = up ? (float)(l + 1) : k;
            xq = up ? lev[l + 1][c] : xq;
            // keeps the chain a chain of register selects: folded into one indexed load it would push the
            // levels out of registers into scratch memory
            asm volatile("" : "+v"(xq));
        }
    }
};

// ---- fused projection + dual + residual, other formats ------------------------------------------------------
// KIND 1 = dual grid, 2 = codebook with L levels.  Thread: 4 columns x FMT_ROWS rows; grid (ceil(p4/256),
// ceil(n/FMT_ROWS)), block 256.  B may be W (each element is read before it is written, by the same thread).
// LAST also stores the codes and the projected unscaled values.
template <int KIND, int L, bool LAST>
__global__ __launch_bounds__(256) void project_format_kernel(
    const float *W, float *__restrict__ V, long n, long p, const float *__restrict__ d,
    const float *__restrict__ inv_d, const uint8_t *__restrict__ flags, DualGridCols dg,
    const float *__restrict__ codebook, float rho, float inv_rho, float inv_rho_next, uint8_t *__restrict__ codes,
    float *B, float *__restrict__ Xq, double *__restrict__ res_sq, int vec_ok, unsigned *__restrict__ amax_out) {
    __shared__ double sh[4];
    const long c0 = ((long)blockIdx.x * 256 + threadIdx.x) * 4;
    const long row0 = (long)blockIdx.y * FMT_ROWS;
    float acc = 0.f;
    unsigned bmax = 0;                   // largest |B| written, as the float's bit pattern
    if (c0 < p) {
        const int nc = (int)min(4L, p - c0);
        const bool vec = vec_ok != 0;            // p % 4 == 0 and every array 16-byte aligned (codes, flags: 4)
        CodebookCols<KIND == 2 ? L : 2> cbk;
        if (KIND == 2) cbk.load(codebook, p, c0, nc, vec);
        for (int r4 = 0; r4 < FMT_ROWS; r4 += 4) {
            float w[4][4], v[4][4];
            uint32_t fl[4];
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) {
                const long i = row0 + r4 + rr;
                const long off = i * p + c0;
                fl[rr] = 0;
                if (i < n) {
                    if (vec) {
                        const floatx4 tw = *(const floatx4 *)(W + off);
                        const floatx4 tv = *(const floatx4 *)(V + off);
                        w[rr][0] = tw.x; w[rr][1] = tw.y; w[rr][2] = tw.z; w[rr][3] = tw.w;
                        v[rr][0] = tv.x; v[rr][1] = tv.y; v[rr][2] = tv.z; v[rr][3] = tv.w;
                        if (flags) fl[rr] = *(const uint32_t *)(flags + off);
                    } else {
#pragma unroll
                        for (int c = 0; c < 4; ++c) {
                            w[rr][c] = c < nc ? W[off + c] : 0.f;
                            v[rr][c] = c < nc ? V[off + c] : 0.f;
                            if (flags && c < nc) fl[rr] |= (uint32_t)flags[off + c] << (8 * c);
                        }
                    }
                }
            }
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) {
                const long i = row0 + r4 + rr;
                if (i >= n) break;
                const long off = i * p + c0;
                if (KIND == 1) dg.row(i, c0, nc);
                const float di = d[i], idi = inv_d[i];
                float vn[4], bn[4], xo[4];
                uint8_t kq[4];
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const int flag = (fl[rr] >> (8 * c)) & 0xFF;
                    const float q = __fmul_rn(v[rr][c], inv_rho);
                    const float wt = __fadd_rn(w[rr][c], q);
                    const float x = __fmul_rn(wt, idi);
                    float k, xq;
                    if (KIND == 1) dg.project(x, c, flag, k, xq);
                    else cbk.project(x, c, k, xq);
                    float Dn = __fmul_rn(di, xq);
                    const bool kept = KIND == 2 && flag != 0;
                    if (kept) {
                        Dn = wt;
                        xq = x;
                        k = 0.f;
                    }
                    const float r = __fsub_rn(w[rr][c], Dn);
                    vn[c] = kept ? 0.f : __fadd_rn(v[rr][c], __fmul_rn(rho, r));
                    bn[c] = __fsub_rn(Dn, __fmul_rn(vn[c], inv_rho_next));
                    kq[c] = (uint8_t)k;
                    xo[c] = xq;
                    if (c < nc) {
                        acc += r * r;
                        bmax = max(bmax, __float_as_uint(fabsf(bn[c])));
                    }
                }
                if (vec) {
                    const floatx4 ov = {vn[0], vn[1], vn[2], vn[3]};
                    const floatx4 ob = {bn[0], bn[1], bn[2], bn[3]};
                    *(floatx4 *)(V + off) = ov;
                    *(floatx4 *)(B + off) = ob;
                    if (LAST) {
                        if (codes)
                            *(uint32_t *)(codes + off) = (uint32_t)kq[0] | ((uint32_t)kq[1] << 8) |
                                                         ((uint32_t)kq[2] << 16) | ((uint32_t)kq[3] << 24);
                        if (Xq) {
                            const floatx4 ox = {xo[0], xo[1], xo[2], xo[3]};
                            *(floatx4 *)(Xq + off) = ox;
                        }
                    }
                } else {
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        if (c < nc) {
                            V[off + c] = vn[c];
                            B[off + c] = bn[c];
                            if (LAST && codes) codes[off + c] = kq[c];
                            if (LAST && Xq) Xq[off + c] = xo[c];
                        }
                    }
                }
            }
        }
    }
    if (res_sq) {
        double tot = wave_sum((double)acc);
        const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
        if (lane == 0) sh[w] = tot;
        __syncthreads();
        if (threadIdx.x == 0) atomicAdd(res_sq, (sh[0] + sh[1]) + (sh[2] + sh[3]));
    }
    if (amax_out) {
        // for the split-fp16 products: the largest |B| of the whole pass; a wave whose maximum is already covered
        // skips the atomic
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) bmax = max(bmax, (unsigned)__shfl_xor((int)bmax, o));
        if ((threadIdx.x & 63) == 0 && bmax > __atomic_load_n(amax_out, __ATOMIC_RELAXED)) atomicMax(amax_out, bmax);
    }
}

// ---- plain projection of the dense weights: E = proj(W0) - W0 (and the codes, if asked) -------------------
// one element per thread; unscaled space (x = W0)
template <int KIND>
__global__ void nearest_error_kernel(const float *__restrict__ W0, long ldw, long n, long p,
                                     const uint8_t *__restrict__ flags, const float *__restrict__ scales,
                                     const float *__restrict__ zeros, long g, float levels,
                                     const float *__restrict__ codebook, int L, uint8_t *__restrict__ codes,
                                     float *__restrict__ E) {
    const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= n * p) return;
    const long i = idx / p, j = idx - i * p;
    const float x = W0[i * ldw + j];
    const int flag = flags ? flags[idx] : 0;
    float k, xq;
    if (KIND == 1) {
        const long at = (flag ? (n / g) * p : 0) + (i / g) * p + j;
        const float dl = scales[at], z0 = zeros[at];
        const float idl = dl == 0.f ? 0.f : __fdiv_rn(1.0f, dl);
        k = fminf(fmaxf(rintf(__fmul_rn(__fsub_rn(x, z0), idl)), 0.f), levels);
        xq = __fadd_rn(__fmul_rn(k, dl), z0);
    } else {
        k = 0.f;
        xq = codebook[j];
        for (int l = 0; l + 1 < L; ++l) {
            const float lo = codebook[(long)l * p + j], hi = codebook[(long)(l + 1) * p + j];
            if (x > __fmul_rn(__fadd_rn(lo, hi), 0.5f)) {
                k = (float)(l + 1);
                xq = hi;
            }
        }
        if (flag) {
            k = 0.f;
            xq = x;
        }
    }
    if (codes) codes[idx] = (uint8_t)k;
    E[idx] = __fsub_rn(xq, x);
}

// E = A - W0 (A dense [n][p], W0 with leading dimension ldw)
__global__ void diff_kernel(const float *__restrict__ A, const float *__restrict__ W0, long ldw, long n, long p,
                            float *__restrict__ E) {
    const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= n * p) return;
    const long i = idx / p, j = idx - i * p;
    E[idx] = __fsub_rn(A[idx], W0[i * ldw + j]);
}

// ---- dual-grid fit: min / max per (group, column) over each subset -----------------------------------------
// block (64, 16): 64 columns x 16 row lanes; grid (ceil(p/64), n/g); scales / zeros [2][n/g][p]
__global__ __launch_bounds__(1024) void dual_grid_init_kernel(const float *__restrict__ W0, long n, long p, long ldw,
                                                              long g, float levels,
                                                              const uint8_t *__restrict__ flags,
                                                              float *__restrict__ scales,
                                                              float *__restrict__ zeros) {
    __shared__ float smn[2][16][64], smx[2][16][64];
    const int tx = threadIdx.x, ty = threadIdx.y;
    const long j = (long)blockIdx.x * 64 + tx;
    const long r0 = (long)blockIdx.y * g;
    float mn[2] = {INFINITY, INFINITY}, mx[2] = {-INFINITY, -INFINITY};
    if (j < p) {
        for (long i = ty; i < g; i += 16) {
            const float w = W0[(r0 + i) * ldw + j];
            const int s = flags[(r0 + i) * p + j] ? 1 : 0;
            mn[s] = fminf(mn[s], w);
            mx[s] = fmaxf(mx[s], w);
        }
    }
    for (int s = 0; s < 2; ++s) {
        smn[s][ty][tx] = mn[s];
        smx[s][ty][tx] = mx[s];
    }
    __syncthreads();
    if (ty == 0 && j < p) {
        for (int s = 0; s < 2; ++s) {
            float a = mn[s], b = mx[s];
            for (int q = 1; q < 16; ++q) {
                a = fminf(a, smn[s][q][tx]);
                b = fmaxf(b, smx[s][q][tx]);
            }
            if (b < a) {         // empty subset: a degenerate grid
                a = 0.f;
                b = 0.f;
            }
            const long at = (long)s * (n / g) * p + (long)blockIdx.y * p + j;
            scales[at] = __fdiv_rn(__fsub_rn(b, a), levels);
            zeros[at] = a;
        }
    }
}

// counts the places where a codebook is not finite or not strictly ascending
__global__ void codebook_check_kernel(const float *__restrict__ cb, int L, long p, double *__restrict__ bad) {
    const long j = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= p) return;
    int wrong = 0;
    for (int l = 0; l < L; ++l) {
        const float c = cb[(long)l * p + j];
        if (!isfinite(c)) ++wrong;
        if (l > 0 && !(c > cb[(long)(l - 1) * p + j])) ++wrong;
    }
    if (wrong) atomicAdd(bad, (double)wrong);
}

unsigned blocks_of(long count, int per) { return (unsigned)((count + per - 1) / per); }

}  // namespace

admmq_status admmq_k_dual_grid_init(admmq_ctx *ctx, const float *W0, int64_t n, int64_t p, int64_t ldw, int bits,
                                    int64_t g, const uint8_t *flags, float *scales, float *zeros) {
    dim3 block(64, 16), grid((unsigned)((p + 63) / 64), (unsigned)(n / g));
    hipLaunchKernelGGL(dual_grid_init_kernel, grid, block, 0, ctx->stream, W0, (long)n, (long)p, (long)ldw, (long)g,
                       (float)((1 << bits) - 1), flags, scales, zeros);
    ADMMQ_HIP(hipGetLastError());
    return ADMMQ_OK;
}

admmq_status admmq_k_codebook_check(admmq_ctx *ctx, const float *codebook, int L, int64_t p, double *dev_bad) {
    hipLaunchKernelGGL(codebook_check_kernel, dim3(blocks_of(p, 256)), dim3(256), 0, ctx->stream, codebook, L,
                       (long)p, dev_bad);
    ADMMQ_HIP(hipGetLastError());
    return ADMMQ_OK;
}

// kind 1: scales / inv_scales / zeros are [2][n/g][p]; kind 2: codebook [2^bits][p], flags may be null.
// `last` != 0 stores codes and Xq (either may be null).
admmq_status admmq_k_project_format(admmq_ctx *ctx, int kind, const float *W, float *V, int64_t n, int64_t p,
                                    const float *d, const float *inv_d, int bits, int64_t g,
                                    const uint8_t *flags, const float *scales, const float *inv_scales,
                                    const float *zeros, const float *codebook, float rho, float inv_rho,
                                    float inv_rho_next, int last, uint8_t *codes, float *B_out, float *Xq,
                                    double *dev_res_sq, unsigned *amax_out) {
    const long p4 = (p + 3) / 4;
    dim3 block(256), grid((unsigned)((p4 + 255) / 256), (unsigned)((n + FMT_ROWS - 1) / FMT_ROWS));
    DualGridCols dg;
    dg.scales = scales; dg.inv_scales = inv_scales; dg.zeros = zeros;
    dg.g = g > 0 ? g : n; dg.p = p; dg.gstride = (n / dg.g) * p;
    dg.levels = (float)((1 << bits) - 1);
    const int vec_ok = (p % 4 == 0) && (((uintptr_t)W | (uintptr_t)V | (uintptr_t)B_out | (uintptr_t)Xq | (uintptr_t)codebook) % 16 == 0) &&
                       (((uintptr_t)codes | (uintptr_t)flags) % 4 == 0);
#define ADMMQ_PF(K, LL, LA)                                                                                      \
    hipLaunchKernelGGL((project_format_kernel<K, LL, LA>), grid, block, 0, ctx->stream, W, V, (long)n, (long)p, d, \
                       inv_d, flags, dg, codebook, rho, inv_rho, inv_rho_next, codes, B_out, Xq, dev_res_sq, vec_ok, amax_out)
#define ADMMQ_PF2(K, LL) do { if (last) ADMMQ_PF(K, LL, true); else ADMMQ_PF(K, LL, false); } while (0)
    if (kind == 1) ADMMQ_PF2(1, 2);
    else if (kind == 2 && bits == 1) ADMMQ_PF2(2, 2);
    else if (kind == 2 && bits == 2) ADMMQ_PF2(2, 4);
    else if (kind == 2 && bits == 3) ADMMQ_PF2(2, 8);
    else if (kind == 2 && bits == 4) ADMMQ_PF2(2, 16);
    else return ADMMQ_ERR_PARAM;
#undef ADMMQ_PF2
#undef ADMMQ_PF
    ADMMQ_HIP(hipGetLastError());
    return ADMMQ_OK;
}

// E = proj(W0) - W0 in the unscaled space; codes optional
admmq_status admmq_k_nearest_error(admmq_ctx *ctx, int kind, const float *W0, int64_t ldw, int64_t n, int64_t p,
                                   int bits, int64_t g, const uint8_t *flags, const float *scales,
                                   const float *zeros, const float *codebook, uint8_t *codes, float *E) {
    const unsigned nb = blocks_of(n * p, 256);
    const float levels = (float)((1 << bits) - 1);
    if (kind == 1)
        hipLaunchKernelGGL(nearest_error_kernel<1>, dim3(nb), dim3(256), 0, ctx->stream, W0, (long)ldw, (long)n,
                           (long)p, flags, scales, zeros, (long)(g > 0 ? g : n), levels, codebook, 1 << bits, codes, E);
    else
        hipLaunchKernelGGL(nearest_error_kernel<2>, dim3(nb), dim3(256), 0, ctx->stream, W0, (long)ldw, (long)n,
                           (long)p, flags, scales, zeros, (long)(g > 0 ? g : n), levels, codebook, 1 << bits, codes, E);
    ADMMQ_HIP(hipGetLastError());
    return ADMMQ_OK;
}

admmq_status admmq_k_diff(admmq_ctx *ctx, const float *A, const float *W0, int64_t ldw, int64_t n, int64_t p,
                          float *E) {
    hipLaunchKernelGGL(diff_kernel, dim3(blocks_of(n * p, 256)), dim3(256), 0, ctx->stream, A, W0, (long)ldw,
                       (long)n, (long)p, E);
    ADMMQ_HIP(hipGetLastError());
    return ADMMQ_OK;
}
