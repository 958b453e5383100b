// Memory-bound streaming kernels of the ADMM-Q path: grid fit (Sec. 3.4), the fused projection +
// dual update + residual pass (eqs. 8-10 and 9), and the small elementwise helpers around them.
//
// Arithmetic contract of the projection (bit-exact integer codes depend on it): every operation is a
// single correctly rounded fp32 operation, in this order, with no fused multiply-add:
//   q = V*inv_rho; wt = W+q; x = wt*inv_d[i]; y = x-z0; t = y*inv_delta; k = clamp(rint(t),0,L)
//   xq = k*delta; xq = xq+z0; Dn = d[i]*xq; r = W-Dn; Vn = V + rho*r; Bn = Dn - Vn*inv_rho_next
// inv_rho, inv_d, inv_delta are fp32 reciprocals formed once with IEEE division (inv_delta = 0 for a
// group whose scale is 0, which pins its codes to 0).
#include <stdlib.h>

#include "common.h"

typedef float floatx4 __attribute__((ext_vector_type(4)));

namespace {

__device__ inline double wave_sum(double v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o, 64);
    return v;
}

__device__ inline double block_sum(double v, double *sh) {
    v = wave_sum(v);
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    if (lane == 0) sh[w] = v;
    __syncthreads();
    const int nw = (blockDim.x + 63) >> 6;
    double r = 0.0;
    if (w == 0) {
        r = lane < nw ? sh[lane] : 0.0;
        r = wave_sum(r);
    }
    __syncthreads();
    return r;   // valid in thread 0
}

// ---- grid fit ---------------------------------------------------------------------------------
// block (64, 16): 64 columns x 16 row lanes; grid (ceil(p/64), n/g)
__global__ __launch_bounds__(1024) void grid_init_kernel(const float *__restrict__ W0, long n, long p, long ldw,
                                                         long g, float levels, float *__restrict__ scales,
                                                         float *__restrict__ zeros) {
    __shared__ float smn[16][64], smx[16][64];
    const int tx = threadIdx.x, ty = threadIdx.y;
    const long j = (long)blockIdx.x * 64 + tx;
    const long r0 = (long)blockIdx.y * g;
    float mn = INFINITY, mx = -INFINITY;
    if (j < p) {
        for (long i = ty; i < g; i += 16) {
            float w = W0[(r0 + i) * ldw + j];
            mn = fminf(mn, w);
            mx = fmaxf(mx, w);
        }
    }
    smn[ty][tx] = mn;
    smx[ty][tx] = mx;
    __syncthreads();
    if (ty == 0 && j < p) {
        for (int q = 1; q < 16; ++q) {
            mn = fminf(mn, smn[q][tx]);
            mx = fmaxf(mx, smx[q][tx]);
        }
        scales[(long)blockIdx.y * p + j] = __fdiv_rn(__fsub_rn(mx, mn), levels);
        zeros[(long)blockIdx.y * p + j] = mn;
    }
}

// Grid fit with options (Sec. 3.4 "Clipping heuristics", App. D): symmetric range [-a, a] and / or an MSE
// search over ranges shrunk towards 0 by r_i = 1 - i/points, i < ncand; the candidate with the smallest
// squared quantization error of the group's dense weights wins (the widest one on ties).
// Same block shape as grid_init_kernel: 64 columns x 16 row lanes per (column block, group).
__global__ __launch_bounds__(1024) void grid_fit_search_kernel(const float *__restrict__ W0, long n, long p, long ldw,
                                                               long g, float levels, int symmetric, int points,
                                                               int ncand, float *__restrict__ scales,
                                                               float *__restrict__ zeros) {
    __shared__ float smn[16][64], smx[16][64];
    const int tx = threadIdx.x, ty = threadIdx.y;
    const long j = (long)blockIdx.x * 64 + tx;
    const long r0 = (long)blockIdx.y * g;
    float mn = INFINITY, mx = -INFINITY;
    if (j < p) {
        for (long i = ty; i < g; i += 16) {
            float w = W0[(r0 + i) * ldw + j];
            mn = fminf(mn, w);
            mx = fmaxf(mx, w);
        }
    }
    smn[ty][tx] = mn;
    smx[ty][tx] = mx;
    __syncthreads();
    for (int q = 0; q < 16; ++q) {
        mn = fminf(mn, smn[q][tx]);
        mx = fmaxf(mx, smx[q][tx]);
    }
    __syncthreads();
    if (symmetric) {
        const float a = fmaxf(fabsf(mn), fabsf(mx));
        mn = -a;
        mx = a;
    }
    const float range = __fsub_rn(mx, mn);
    float best_err = INFINITY, best_dl = __fdiv_rn(range, levels), best_z0 = mn;
    for (int c = 0; c < ncand; ++c) {
        const float r = __fsub_rn(1.0f, __fdiv_rn((float)c, (float)points));
        const float z0 = __fmul_rn(r, mn);
        const float dl = __fdiv_rn(__fmul_rn(r, range), levels);
        const float idl = dl == 0.f ? 0.f : __fdiv_rn(1.0f, dl);
        float e = 0.f;
        if (j < p) {
            for (long i = ty; i < g; i += 16) {
                const float w = W0[(r0 + i) * ldw + j];
                const float k = fminf(fmaxf(rintf(__fmul_rn(__fsub_rn(w, z0), idl)), 0.f), levels);
                const float q = __fsub_rn(__fadd_rn(__fmul_rn(k, dl), z0), w);
                e += q * q;
            }
        }
        smn[ty][tx] = e;
        __syncthreads();
        if (ty == 0) {
            float tot = 0.f;
            for (int q = 0; q < 16; ++q) tot += smn[q][tx];
            if (tot < best_err) {
                best_err = tot;
                best_dl = dl;
                best_z0 = z0;
            }
        }
        __syncthreads();
    }
    if (ty == 0 && j < p) {
        scales[(long)blockIdx.y * p + j] = best_dl;
        zeros[(long)blockIdx.y * p + j] = best_z0;
    }
}

__global__ void recip_kernel(const float *__restrict__ x, float *__restrict__ inv, long count) {
    long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) {
        float v = x[i];
        inv[i] = v == 0.f ? 0.f : __fdiv_rn(1.0f, v);
    }
}

// ---- fused projection + dual + residual -------------------------------------------------------
// Each thread owns 4 consecutive columns and walks ROWS rows of one group, so the grid parameters of
// its columns are read once.  B may be the same array as W (every element is read before it is written,
// by the same thread): the ADMM loop uses that to keep the pass on two arrays instead of three.  grid: (ceil(p4 / 256), ceil(n / ROWS)), block 256.
constexpr int PD_ROWS = 16;     // measured inside the ADMM loop on MI355X: 16 rows per thread is the fastest

template <bool CODES, bool FLIPS, bool VEC>
__global__ __launch_bounds__(256) void project_dual_kernel(
    const float *W, float *__restrict__ V, long n, long p, const float *__restrict__ d,
    const float *__restrict__ inv_d, float levels, long g, const float *__restrict__ scales,
    const float *__restrict__ inv_scales, const float *__restrict__ zeros, float rho, float inv_rho,
    float inv_rho_next, uint8_t *__restrict__ codes, float *B, double *__restrict__ res_sq,
    unsigned long long *__restrict__ flips, int rows_per_block, int nontemporal, long ldw,
    unsigned *__restrict__ amax_out) {
    __shared__ double sh[4];
    const long c0 = ((long)blockIdx.x * 256 + threadIdx.x) * 4;
    const long row0 = (long)blockIdx.y * rows_per_block;
    float acc = 0.f;
    unsigned nflip = 0;
    unsigned bmax = 0;                   // largest |B| written, as the float's bit pattern (orders like the float)
    if (c0 < p) {
        const int nc = (int)min(4L, p - c0);
        long grp = -1;
        float dl[4], idl[4], z0[4];
        for (int r4 = 0; r4 < rows_per_block; r4 += 4) {
            // stage 1: issue the loads of up to 4 rows before any arithmetic depends on them
            float w[4][4], v[4][4];
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) {
                const long i = row0 + r4 + rr;
                const long off = i * p + c0, offw = i * ldw + c0;
                if (i < n) {
                    if (VEC) {
                        floatx4 tw, tv;
                        if (nontemporal & 1) tw = __builtin_nontemporal_load((const floatx4 *)(W + offw));
                        else tw = *(const floatx4 *)(W + offw);
                        if (nontemporal & 2) tv = __builtin_nontemporal_load((const floatx4 *)(V + off));
                        else tv = *(const floatx4 *)(V + off);
                        w[rr][0] = tw.x; w[rr][1] = tw.y; w[rr][2] = tw.z; w[rr][3] = tw.w;
                        v[rr][0] = tv.x; v[rr][1] = tv.y; v[rr][2] = tv.z; v[rr][3] = tv.w;
                    } else {
#pragma unroll
                        for (int c = 0; c < 4; ++c) {
                            w[rr][c] = c < nc ? W[offw + c] : 0.f;
                            v[rr][c] = c < nc ? V[off + c] : 0.f;
                        }
                    }
                }
            }
            // stage 2: arithmetic and stores, row by row
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) {
                const long i = row0 + r4 + rr;
                if (i >= n) break;
                const long off = i * p + c0, offw = i * ldw + c0;
                const long gi = i / g;
                if (gi != grp) {
                    grp = gi;
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        if (c < nc) {
                            dl[c] = scales[gi * p + c0 + c];
                            idl[c] = inv_scales[gi * p + c0 + c];
                            z0[c] = zeros[gi * p + c0 + c];
                        } else {
                            dl[c] = 0.f; idl[c] = 0.f; z0[c] = 0.f;
                        }
                    }
                }
                const float di = d[i], idi = inv_d[i];
                float vn[4], bn[4];
                uint8_t kq[4];
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    float q = __fmul_rn(v[rr][c], inv_rho);
                    float wt = __fadd_rn(w[rr][c], q);
                    float x = __fmul_rn(wt, idi);
                    float y = __fsub_rn(x, z0[c]);
                    float t = __fmul_rn(y, idl[c]);
                    float k = fminf(fmaxf(rintf(t), 0.f), levels);
                    float xq = __fadd_rn(__fmul_rn(k, dl[c]), z0[c]);
                    float Dn = __fmul_rn(di, xq);
                    float r = __fsub_rn(w[rr][c], Dn);
                    vn[c] = __fadd_rn(v[rr][c], __fmul_rn(rho, r));
                    bn[c] = __fsub_rn(Dn, __fmul_rn(vn[c], inv_rho_next));
                    kq[c] = (uint8_t)k;
                    if (c < nc) {
                        acc += r * r;
                        bmax = max(bmax, __float_as_uint(fabsf(bn[c])));
                    }
                }
                if (VEC) {
                    floatx4 ov = {vn[0], vn[1], vn[2], vn[3]};
                    floatx4 ob = {bn[0], bn[1], bn[2], bn[3]};
                    if (nontemporal & 2) __builtin_nontemporal_store(ov, (floatx4 *)(V + off));
                    else *(floatx4 *)(V + off) = ov;
                    if (nontemporal & 4) __builtin_nontemporal_store(ob, (floatx4 *)(B + offw));
                    else *(floatx4 *)(B + offw) = ob;
                    if (CODES) {
                        uint32_t packed = (uint32_t)kq[0] | ((uint32_t)kq[1] << 8) | ((uint32_t)kq[2] << 16) |
                                          ((uint32_t)kq[3] << 24);
                        if (FLIPS) {
                            uint32_t old = *(const uint32_t *)(codes + off);
                            uint32_t x = old ^ packed;
                            nflip += ((x & 0xFFu) != 0) + ((x & 0xFF00u) != 0) + ((x & 0xFF0000u) != 0) +
                                     ((x & 0xFF000000u) != 0);
                        }
                        *(uint32_t *)(codes + off) = packed;
                    }
                } else {
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        if (c < nc) {
                            V[off + c] = vn[c];
                            B[offw + c] = bn[c];
                            if (CODES) {
                                if (FLIPS) nflip += codes[off + c] != kq[c];
                                codes[off + c] = kq[c];
                            }
                        }
                    }
                }
            }
        }
    }
    if (res_sq) {
        double tot = block_sum((double)acc, sh);
        if (threadIdx.x == 0) atomicAdd(res_sq, tot);
    }
    if (FLIPS && flips) {
        double tot = block_sum((double)nflip, sh);
        if (threadIdx.x == 0 && tot > 0.0) atomicAdd(flips, (unsigned long long)tot);
    }
    if (amax_out) {
        // for the split-fp16 products: the largest |B| of the whole pass, one atomic per wave
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) bmax = max(bmax, (unsigned)__shfl_xor((int)bmax, o));
        // (most waves find a value at least as large already there and skip the atomic: thousands of atomics on
        // one address would take longer than the pass itself)
        if ((threadIdx.x & 63) == 0 && bmax > __atomic_load_n(amax_out, __ATOMIC_RELAXED)) atomicMax(amax_out, bmax);
    }
}

// ---- grid refresh (App. B) ----------------------------------------------------------------------
// min / max per group of the projection target x = (W + V*inv_rho)*inv_d -> refitted (scale, zero).
// Same block shape as grid_init_kernel.
__global__ __launch_bounds__(1024) void refit_grid_kernel(const float *__restrict__ W, const float *__restrict__ V,
                                                          long n, long p, const float *__restrict__ inv_d,
                                                          float inv_rho, long g, float levels,
                                                          float *__restrict__ scales, float *__restrict__ zeros) {
    __shared__ float smn[16][64], smx[16][64];
    const int tx = threadIdx.x, ty = threadIdx.y;
    const long j = (long)blockIdx.x * 64 + tx;
    const long r0 = (long)blockIdx.y * g;
    float mn = INFINITY, mx = -INFINITY;
    if (j < p) {
        for (long i = ty; i < g; i += 16) {
            const long off = (r0 + i) * p + j;
            const float x = __fmul_rn(__fadd_rn(W[off], __fmul_rn(V[off], inv_rho)), inv_d[r0 + i]);
            mn = fminf(mn, x);
            mx = fmaxf(mx, x);
        }
    }
    smn[ty][tx] = mn;
    smx[ty][tx] = mx;
    __syncthreads();
    if (ty == 0 && j < p) {
        for (int q = 1; q < 16; ++q) {
            mn = fminf(mn, smn[q][tx]);
            mx = fmaxf(mx, smx[q][tx]);
        }
        scales[(long)blockIdx.y * p + j] = __fdiv_rn(__fsub_rn(mx, mn), levels);
        zeros[(long)blockIdx.y * p + j] = mn;
    }
}

// Both sides of eq. 12: part[2*b] = sum (D_old - Wt)^2, part[2*b+1] = sum (D_new - Wt)^2 over block b's
// elements (scaled variables).  One element per thread, grid-stride; fixed order inside a block.
__global__ __launch_bounds__(256) void refresh_error_kernel(const float *__restrict__ W, const float *__restrict__ V,
                                                            long n, long p, const float *__restrict__ d,
                                                            const float *__restrict__ inv_d, float inv_rho, long g,
                                                            float levels, const float *__restrict__ sc_old,
                                                            const float *__restrict__ zr_old,
                                                            const float *__restrict__ sc_new,
                                                            const float *__restrict__ zr_new,
                                                            double *__restrict__ part) {
    __shared__ double sh[4];
    double eo = 0.0, en = 0.0;
    const long total = n * p;
    for (long idx = (long)blockIdx.x * 256 + threadIdx.x; idx < total; idx += (long)gridDim.x * 256) {
        const long i = idx / p, j = idx - i * p;
        const long gi = (i / g) * p + j;
        const float wt = __fadd_rn(W[idx], __fmul_rn(V[idx], inv_rho));
        const float x = __fmul_rn(wt, inv_d[i]);
        {
            const float dl = sc_old[gi], z0 = zr_old[gi];
            const float idl = dl == 0.f ? 0.f : __fdiv_rn(1.0f, dl);
            const float k = fminf(fmaxf(rintf(__fmul_rn(__fsub_rn(x, z0), idl)), 0.f), levels);
            const float e = __fsub_rn(__fmul_rn(d[i], __fadd_rn(__fmul_rn(k, dl), z0)), wt);
            eo += (double)e * (double)e;
        }
        {
            const float dl = sc_new[gi], z0 = zr_new[gi];
            const float idl = dl == 0.f ? 0.f : __fdiv_rn(1.0f, dl);
            const float k = fminf(fmaxf(rintf(__fmul_rn(__fsub_rn(x, z0), idl)), 0.f), levels);
            const float e = __fsub_rn(__fmul_rn(d[i], __fadd_rn(__fmul_rn(k, dl), z0)), wt);
            en += (double)e * (double)e;
        }
    }
    const double to = block_sum(eo, sh);
    const double tn = block_sum(en, sh);
    if (threadIdx.x == 0) {
        part[2 * blockIdx.x] = to;
        part[2 * blockIdx.x + 1] = tn;
    }
}

// ---- helpers ----------------------------------------------------------------------------------
__global__ void scale_rows_kernel(const float *__restrict__ W0, long ldw, const float *__restrict__ d, long n,
                                  long p, float *__restrict__ out, long ldo) {
    long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx < n * p) {
        long i = idx / p, j = idx - i * p;
        out[i * ldo + j] = __fmul_rn(d[i], W0[i * ldw + j]);
    }
}

__global__ void form_b_kernel(const float *__restrict__ D, const float *__restrict__ V, float inv_rho,
                              long count, float *__restrict__ B) {
    long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx < count) B[idx] = __fsub_rn(D[idx], __fmul_rn(V[idx], inv_rho));
}

__global__ void fill_f32_kernel(float *x, float v, long count) {
    long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx < count) x[idx] = v;
}

__global__ void fill_u32_kernel(uint32_t *x, uint32_t v, long count) {
    long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx < count) x[idx] = v;
}

__global__ void fill_u8_kernel(uint8_t *x, uint8_t v, long count) {
    long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx < count) x[idx] = v;
}

// Plain copy, 16 bytes per lane, four rows of loads in flight per thread (the shape of the projection pass without
// its arithmetic): the reference for what a streaming kernel of this library reaches on the memory system.
__global__ __launch_bounds__(256) void stream_copy_kernel(const floatx4 *__restrict__ src, floatx4 *__restrict__ dst,
                                                          long count) {
    const long base = ((long)blockIdx.x * 256) * 4 + threadIdx.x;
    floatx4 v[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const long i = base + (long)k * 256;
        if (i < count) v[k] = src[i];
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const long i = base + (long)k * 256;
        if (i < count) dst[i] = v[k];
    }
}

// mode 0: E = dequant(codes) - W0 ; mode 1: E = W0 - dequant(codes);
// mode 2: codes are first set to round-to-nearest of W0 on the grid, then E = dequant - W0
__global__ void quant_error_kernel(const float *__restrict__ W0, long ldw, uint8_t *__restrict__ codes, long n,
                                   long p, long g, const float *__restrict__ scales,
                                   const float *__restrict__ zeros, float levels, int mode,
                                   float *__restrict__ E) {
    long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= n * p) return;
    long i = idx / p, j = idx - i * p;
    long gi = (i / g) * p + j;
    float dl = scales[gi], z0 = zeros[gi], w = W0[i * ldw + j];
    float k;
    if (mode == 2) {
        float idl = dl == 0.f ? 0.f : __fdiv_rn(1.0f, dl);
        k = fminf(fmaxf(rintf(__fmul_rn(__fsub_rn(w, z0), idl)), 0.f), levels);
        codes[idx] = (uint8_t)k;
    } else {
        k = (float)codes[idx];
    }
    float wq = __fadd_rn(__fmul_rn(k, dl), z0);
    E[idx] = mode == 1 ? __fsub_rn(w, wq) : __fsub_rn(wq, w);
}

__global__ __launch_bounds__(256) void dot_kernel(const float *__restrict__ A, const float *__restrict__ B,
                                                  long count, double *__restrict__ out) {
    __shared__ double sh[4];
    double s = 0.0;
    for (long i = (long)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += (long)gridDim.x * blockDim.x)
        s += (double)A[i] * (double)B[i];
    double tot = block_sum(s, sh);
    if (threadIdx.x == 0) atomicAdd(out, tot);
}

// out[0] += trace, out[1] += #non-finite entries, out[2] += #diagonal entries <= 0
__global__ __launch_bounds__(256) void matrix_check_kernel(const float *__restrict__ H, long n,
                                                           double *__restrict__ out) {
    __shared__ double sh[4];
    double tr = 0.0, bad = 0.0, nonpos = 0.0;
    const long total = n * n;
    for (long i = (long)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (long)gridDim.x * blockDim.x) {
        float v = H[i];
        if (!isfinite(v)) bad += 1.0;
        long r = i / n;
        if (i - r * n == r) {
            tr += (double)v;
            if (!(v > 0.f)) nonpos += 1.0;
        }
    }
    double t0 = block_sum(tr, sh);
    double t1 = block_sum(bad, sh);
    double t2 = block_sum(nonpos, sh);
    if (threadIdx.x == 0) {
        atomicAdd(out + 0, t0);
        if (t1 > 0.0) atomicAdd(out + 1, t1);
        if (t2 > 0.0) atomicAdd(out + 2, t2);
    }
}

__global__ __launch_bounds__(256) void count_nonfinite_kernel(const float *__restrict__ A, long rows, long cols,
                                                              long ld, double *__restrict__ out) {
    __shared__ double sh[4];
    double bad = 0.0;
    const long total = rows * cols;
    for (long i = (long)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (long)gridDim.x * blockDim.x) {
        long r = i / cols;
        if (!isfinite(A[r * ld + (i - r * cols)])) bad += 1.0;
    }
    double t = block_sum(bad, sh);
    if (threadIdx.x == 0 && t > 0.0) atomicAdd(out, t);
}

inline unsigned blocks_for(long count, int bs) { return (unsigned)((count + bs - 1) / bs); }

}  // namespace

admmq_status admmq_k_grid_init(admmq_ctx *ctx, const float *W0, int64_t n, int64_t p, int64_t ldw, int bits,
                               int64_t g, float *scales, float *zeros) {
    dim3 block(64, 16), grid((unsigned)((p + 63) / 64), (unsigned)(n / g));
    hipLaunchKernelGGL(grid_init_kernel, grid, block, 0, ctx->stream, W0, (long)n, (long)p, (long)ldw, (long)g,
                       (float)((1 << bits) - 1), scales, zeros);
    ADMMQ_HIP(hipGetLastError());
    return ADMMQ_OK;
}

admmq_status admmq_k_grid_fit(admmq_ctx *ctx, const float *W0, int64_t n, int64_t p, int64_t ldw, int bits,
                              int64_t g, int symmetric, int clip_points, double clip_shrink, float *scales,
                              float *zeros) {
    if (!symmetric && clip_points <= 0) return admmq_k_grid_init(ctx, W0, n, p, ldw, bits, g, scales, zeros);
    const int ncand = clip_points > 0 ? (int)(clip_shrink * (double)clip_points) : 0;
    dim3 block(64, 16), grid((unsigned)((p + 63) / 64), (unsigned)(n / g));
    hipLaunchKernelGGL(grid_fit_search_kernel, grid, block, 0, ctx->stream, W0, (long)n, (long)p, (long)ldw, (long)g,
                       (float)((1 << bits) - 1), symmetric, clip_points > 0 ? clip_points : 1, ncand, scales, zeros);
    ADMMQ_HIP(hipGetLastError());
    return ADMMQ_OK;
}

admmq_status admmq_k_recip(admmq_ctx *ctx, const float *x, float *inv, int64_t count) {
    hipLaunchKernelGGL(recip_kernel, dim3(blocks_for(count, 256)), dim3(256), 0, ctx->stream, x, inv, (long)count);
    ADMMQ_HIP(hipGetLastError());
    return ADMMQ_OK;
}

admmq_status admmq_k_project_dual(admmq_ctx *ctx, const float *W, float *V, int64_t n, int64_t p, const float *d,
                                  const float *inv_d, int bits, int64_t g, const float *scales,
                                  const float *inv_scales, const float *zeros, float rho, float inv_rho,
                                  float inv_rho_next, uint8_t *codes, int count_flips, float *B_out,
                                  double *dev_res_sq, unsigned long long *dev_flips, int64_t ldw, unsigned *amax_out) {
    // ldw: leading dimension of W and B_out (several matrices side by side); V, codes and the grid are [.][p]
    const long p4 = (p + 3) / 4;
    static int rows_cfg = -1, nt_cfg = 0;
    if (rows_cfg < 0) {
        const char *e = getenv("ADMMQ_PD_ROWS");
        rows_cfg = e ? atoi(e) : PD_ROWS;
        if (rows_cfg < 4 || rows_cfg % 4 != 0 || rows_cfg > 256) rows_cfg = PD_ROWS;
        const char *e2 = getenv("ADMMQ_PD_NT");
        nt_cfg = e2 ? atoi(e2) : 0;
    }
    const int rows_per_block = rows_cfg;
    dim3 block(256), grid((unsigned)((p4 + 255) / 256), (unsigned)((n + rows_per_block - 1) / rows_per_block));
    const bool vec = (p % 4 == 0) && (ldw % 4 == 0) && (((uintptr_t)W | (uintptr_t)V | (uintptr_t)B_out) % 16 == 0) &&
                     (codes == nullptr || (uintptr_t)codes % 4 == 0);
    const float levels = (float)((1 << bits) - 1);
#define ADMMQ_PD(C, F, VV)                                                                                   \
    hipLaunchKernelGGL((project_dual_kernel<C, F, VV>), grid, block, 0, ctx->stream, W, V, (long)n, (long)p, d, \
                       inv_d, levels, (long)g, scales, inv_scales, zeros, rho, inv_rho, inv_rho_next, codes,  \
                       B_out, dev_res_sq, dev_flips, rows_per_block, nt_cfg, (long)ldw, amax_out)
    if (codes && count_flips) { if (vec) ADMMQ_PD(true, true, true); else ADMMQ_PD(true, true, false); }
    else if (codes)           { if (vec) ADMMQ_PD(true, false, true); else ADMMQ_PD(true, false, false); }
    else                      { if (vec) ADMMQ_PD(false, false, true); else ADMMQ_PD(false, false, false); }
#undef ADMMQ_PD
    ADMMQ_HIP(hipGetLastError());
    return ADMMQ_OK;
}

admmq_status admmq_k_scale_rows(admmq_ctx *ctx, const float *W0, int64_t ldw, const float *d, int64_t n, int64_t p,
                                float *out, int64_t ldo) {
    hipLaunchKernelGGL(scale_rows_kernel, dim3(blocks_for(n * p, 256)), dim3(256), 0, ctx->stream, W0, (long)ldw, d,
                       (long)n, (long)p, out, (long)ldo);
    ADMMQ_HIP(hipGetLastError());
    return ADMMQ_OK;
}

admmq_status admmq_k_form_b(admmq_ctx *ctx, const float *D, const float *V, float inv_rho, int64_t count,
                            float *B) {
    hipLaunchKernelGGL(form_b_kernel, dim3(blocks_for(count, 256)), dim3(256), 0, ctx->stream, D, V, inv_rho,
                       (long)count, B);
    ADMMQ_HIP(hipGetLastError());
    return ADMMQ_OK;
}

admmq_status admmq_k_fill_f32(admmq_ctx *ctx, float *x, float v, int64_t count) {
    if (count <= 0) return ADMMQ_OK;
    hipLaunchKernelGGL(fill_f32_kernel, dim3(blocks_for(count, 256)), dim3(256), 0, ctx->stream, x, v, (long)count);
    ADMMQ_HIP(hipGetLastError());
    return ADMMQ_OK;
}

admmq_status admmq_k_fill_bytes(admmq_ctx *ctx, void *x, int v, size_t bytes) {
    if (bytes == 0) return ADMMQ_OK;
    const uint32_t b = (uint32_t)(v & 0xFF);
    uint8_t *base = (uint8_t *)x;
    size_t head = 0;
    if (((uintptr_t)base & 3) == 0) {
        const long words = (long)(bytes / 4);
        if (words > 0)
            hipLaunchKernelGGL(fill_u32_kernel, dim3(blocks_for(words, 256)), dim3(256), 0, ctx->stream,
                               (uint32_t *)base, b | (b << 8) | (b << 16) | (b << 24), words);
        head = (size_t)words * 4;
    }
    if (head < bytes)
        hipLaunchKernelGGL(fill_u8_kernel, dim3(blocks_for((long)(bytes - head), 256)), dim3(256), 0, ctx->stream,
                           base + head, (uint8_t)b, (long)(bytes - head));
    ADMMQ_HIP(hipGetLastError());
    return ADMMQ_OK;
}

admmq_status admmq_k_stream_copy(admmq_ctx *ctx, void *dst, const void *src, size_t bytes) {
    const long count = (long)(bytes / 16);
    if (count == 0) return ADMMQ_OK;
    hipLaunchKernelGGL(stream_copy_kernel, dim3(blocks_for(count, 1024)), dim3(256), 0, ctx->stream,
                       (const floatx4 *)src, (floatx4 *)dst, count);
    ADMMQ_HIP(hipGetLastError());
    return ADMMQ_OK;
}

admmq_status admmq_k_quant_error(admmq_ctx *ctx, const float *W0, int64_t ldw, uint8_t *codes, int64_t n,
                                 int64_t p, int64_t g, const float *scales, const float *zeros, int bits, int mode,
                                 float *E) {
    hipLaunchKernelGGL(quant_error_kernel, dim3(blocks_for(n * p, 256)), dim3(256), 0, ctx->stream, W0, (long)ldw,
                       codes, (long)n, (long)p, (long)g, scales, zeros, (float)((1 << bits) - 1), mode, E);
    ADMMQ_HIP(hipGetLastError());
    return ADMMQ_OK;
}

admmq_status admmq_k_dot(admmq_ctx *ctx, const float *A, const float *B, int64_t count, double *dev_out) {
    unsigned nb = (unsigned)min((long)2048, (long)((count + 255) / 256));
    hipLaunchKernelGGL(dot_kernel, dim3(nb), dim3(256), 0, ctx->stream, A, B, (long)count, dev_out);
    ADMMQ_HIP(hipGetLastError());
    return ADMMQ_OK;
}

admmq_status admmq_k_matrix_check(admmq_ctx *ctx, const float *H, int64_t n, double *dev_out) {
    unsigned nb = (unsigned)min((long)2048, (long)((n * n + 255) / 256));
    hipLaunchKernelGGL(matrix_check_kernel, dim3(nb), dim3(256), 0, ctx->stream, H, (long)n, dev_out);
    ADMMQ_HIP(hipGetLastError());
    return ADMMQ_OK;
}

admmq_status admmq_k_count_nonfinite(admmq_ctx *ctx, const float *A, int64_t rows, int64_t cols, int64_t ld,
                                     double *dev_out) {
    unsigned nb = (unsigned)min((long)2048, (long)((rows * cols + 255) / 256));
    hipLaunchKernelGGL(count_nonfinite_kernel, dim3(nb), dim3(256), 0, ctx->stream, A, (long)rows, (long)cols,
                       (long)ld, dev_out);
    ADMMQ_HIP(hipGetLastError());
    return ADMMQ_OK;
}

admmq_status admmq_k_refit_grid(admmq_ctx *ctx, const float *W, const float *V, int64_t n, int64_t p,
                                const float *inv_d, float inv_rho, int bits, int64_t g, float *scales, float *zeros) {
    dim3 block(64, 16), grid((unsigned)((p + 63) / 64), (unsigned)(n / g));
    hipLaunchKernelGGL(refit_grid_kernel, grid, block, 0, ctx->stream, W, V, (long)n, (long)p, inv_d, inv_rho,
                       (long)g, (float)((1 << bits) - 1), scales, zeros);
    ADMMQ_HIP(hipGetLastError());
    return ADMMQ_OK;
}

int admmq_refresh_error_blocks() { return 1024; }

admmq_status admmq_k_refresh_error(admmq_ctx *ctx, const float *W, const float *V, int64_t n, int64_t p,
                                   const float *d, const float *inv_d, float inv_rho, int bits, int64_t g,
                                   const float *sc_old, const float *zr_old, const float *sc_new,
                                   const float *zr_new, double *part) {
    hipLaunchKernelGGL(refresh_error_kernel, dim3(admmq_refresh_error_blocks()), dim3(256), 0, ctx->stream, W, V,
                       (long)n, (long)p, d, inv_d, inv_rho, (long)g, (float)((1 << bits) - 1), sc_old, zr_old, sc_new,
                       zr_new, part);
    ADMMQ_HIP(hipGetLastError());
    return ADMMQ_OK;
}
