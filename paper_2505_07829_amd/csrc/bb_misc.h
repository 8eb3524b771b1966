// Small kernels: the row-wise operators of the UNFUSED block programs
// (Example 3 / Example 2, initial block programs), the column vectors
// gamma^T W and beta^T W of Rule 5, fills, and the calibration kernels used
// for roofline denominators.
#pragma once
#include "bb_common.h"

namespace bb {

__device__ __forceinline__ float block_sum_256(float v, float* scratch /* >= 4 floats */) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) scratch[threadIdx.x >> 6] = v;
    __syncthreads();
    return scratch[0] + scratch[1] + scratch[2] + scratch[3];
}

// Xh[i,:] = bf16( g * x * rsqrt(mean(x^2) + eps) ), one workgroup per row.
__global__ __launch_bounds__(256) void rmsnorm_rows_kernel(const u16* X, const u16* g, u16* Xh, int D, float eps) {
    __shared__ float red[4];
    const size_t row = blockIdx.x;
    const u16* x = X + row * D;
    float s = 0.f;
    for (int c = threadIdx.x * 8; c < D; c += 256 * 8) {
        const u32x4 v = ldg16(x + c);
#pragma unroll
        for (int q = 0; q < 4; ++q) { const float a = bf_lo(v[q]), b = bf_hi(v[q]); s += a * a + b * b; }
    }
    s = block_sum_256(s, red);
    const float r = rsqrtf(s / (float)D + eps);
    for (int c = threadIdx.x * 8; c < D; c += 256 * 8) {
        const u32x4 v = ldg16(x + c), gv = ldg16(g + c);
        u32x4 o;
#pragma unroll
        for (int q = 0; q < 4; ++q)
            o[q] = pack_bf16(bf_lo(gv[q]) * bf_lo(v[q]) * r, bf_hi(gv[q]) * bf_hi(v[q]) * r);
        *reinterpret_cast<u32x4*>(Xh + row * D + c) = o;
    }
}

// The statistics loop of Example 3's first snapshot as a kernel of its own, with the gain:
// Xg[i,:] = bf16( g * x ) and rstd[i] = rsqrt(mean(x^2) + eps); one workgroup per row, X read once.
__global__ __launch_bounds__(256) void rms_gain_rows_kernel(const u16* X, const u16* g, u16* Xg, float* rstd, int D,
                                                            float eps) {
    __shared__ float red[4];
    const size_t row = blockIdx.x;
    const u16* x = X + row * D;
    float s = 0.f;
    for (int c = threadIdx.x * 8; c < D; c += 256 * 8) {
        const u32x4 v = ldg16(x + c), gv = ldg16(g + c);
        u32x4 o;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const float a = bf_lo(v[q]), b = bf_hi(v[q]);
            s += a * a + b * b;
            o[q] = pack_bf16(bf_lo(gv[q]) * a, bf_hi(gv[q]) * b);
        }
        *reinterpret_cast<u32x4*>(Xg + row * D + c) = o;
    }
    s = block_sum_256(s, red);
    if (threadIdx.x == 0) rstd[row] = rsqrtf(s / (float)D + eps);
}

// Z[i,:] = bf16( gamma * (x - mean) * rsqrt(var + eps) + beta ), biased variance, two passes.
__global__ __launch_bounds__(256) void layernorm_rows_kernel(const u16* X, const u16* gamma, const u16* beta,
                                                             u16* Z, int D, float eps) {
    __shared__ float red[4];
    const size_t row = blockIdx.x;
    const u16* x = X + row * D;
    float s = 0.f;
    for (int c = threadIdx.x * 8; c < D; c += 256 * 8) {
        const u32x4 v = ldg16(x + c);
#pragma unroll
        for (int q = 0; q < 4; ++q) s += bf_lo(v[q]) + bf_hi(v[q]);
    }
    const float mu = block_sum_256(s, red) / (float)D;
    float s2 = 0.f;
    for (int c = threadIdx.x * 8; c < D; c += 256 * 8) {
        const u32x4 v = ldg16(x + c);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const float a = bf_lo(v[q]) - mu, b = bf_hi(v[q]) - mu;
            s2 += a * a + b * b;
        }
    }
    const float r = rsqrtf(block_sum_256(s2, red) / (float)D + eps);
    for (int c = threadIdx.x * 8; c < D; c += 256 * 8) {
        const u32x4 v = ldg16(x + c), gv = ldg16(gamma + c), bv = ldg16(beta + c);
        u32x4 o;
#pragma unroll
        for (int q = 0; q < 4; ++q)
            o[q] = pack_bf16(fmaf(bf_lo(gv[q]) * (bf_lo(v[q]) - mu), r, bf_lo(bv[q])),
                             fmaf(bf_hi(gv[q]) * (bf_hi(v[q]) - mu), r, bf_hi(bv[q])));
        *reinterpret_cast<u32x4*>(Z + row * D + c) = o;
    }
}

// The statistics loop of Example 2's first snapshot as a kernel of its own, with gamma:
// Xg[i,:] = bf16( gamma * x ), stat[i] = (rsqrt(var + eps), mean), biased variance, two passes;
// one workgroup per row.
__global__ __launch_bounds__(256) void ln_gain_rows_kernel(const u16* X, const u16* gamma, u16* Xg, float* stat,
                                                           int D, float eps) {
    __shared__ float red[4];
    const size_t row = blockIdx.x;
    const u16* x = X + row * D;
    float s = 0.f;
    for (int c = threadIdx.x * 8; c < D; c += 256 * 8) {
        const u32x4 v = ldg16(x + c), gv = ldg16(gamma + c);
        u32x4 o;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const float a = bf_lo(v[q]), b = bf_hi(v[q]);
            s += a + b;
            o[q] = pack_bf16(bf_lo(gv[q]) * a, bf_hi(gv[q]) * b);
        }
        *reinterpret_cast<u32x4*>(Xg + row * D + c) = o;
    }
    const float mu = block_sum_256(s, red) / (float)D;
    float s2 = 0.f;
    for (int c = threadIdx.x * 8; c < D; c += 256 * 8) {
        const u32x4 v = ldg16(x + c);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const float a = bf_lo(v[q]) - mu, b = bf_hi(v[q]) - mu;
            s2 += a * a + b * b;
        }
    }
    s2 = block_sum_256(s2, red);
    if (threadIdx.x == 0) {
        stat[2 * row] = rsqrtf(s2 / (float)D + eps);
        stat[2 * row + 1] = mu;
    }
}

// H = bf16( SiLU(P) * Q ), elementwise over n8 groups of 8 bf16.
__global__ __launch_bounds__(256) void silu_mul_kernel(const u16* P, const u16* Q, u16* H, size_t n8) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n8; i += (size_t)gridDim.x * 256) {
        const u32x4 a = ldg16(P + 8 * i), b = ldg16(Q + 8 * i);
        u32x4 o;
#pragma unroll
        for (int q = 0; q < 4; ++q)
            o[q] = pack_bf16(swiglu(bf_lo(a[q]), bf_lo(b[q])), swiglu(bf_hi(a[q]), bf_hi(b[q])));
        *reinterpret_cast<u32x4*>(H + 8 * i) = o;
    }
}

// colc[n] = sum_d gamma[d] W[d,n],  colb[n] = sum_d beta[d] W[d,n]   (Rule 5:
// the column sums of the gain-scaled weight; beta's image is the bias row).
// W is streamed once.  Workgroup (x, y) takes 512 columns and the y-th of
// COLVEC_SPLITS row ranges; each wavefront reads whole 1 KiB row segments (one
// 16-byte load per lane, eight rows in flight), the four wavefronts' sums are
// added through LDS and written as partial sums part[y][0/1][n]; a second
// small kernel adds the COLVEC_SPLITS partial sums (fixed order, no atomics).
constexpr int COLVEC_SPLITS = 8;
__global__ __launch_bounds__(256) void colvec_partial_kernel(const u16* W, const u16* gamma, const u16* beta,
                                                             float* part, int D, int N) {
    __shared__ float red[3][2][512];
    const int t = threadIdx.x, lane = t & 63, w = __builtin_amdgcn_readfirstlane(t >> 6);
    const int col = blockIdx.x * 512 + 8 * lane;
    const int dper = ((D + COLVEC_SPLITS - 1) / COLVEC_SPLITS + 7) / 8 * 8;      // multiple of 8 (so is D)
    const int dbeg = blockIdx.y * dper, dend = min(D, dbeg + dper);
    float c[8], b[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) { c[j] = 0.f; b[j] = 0.f; }
    if (col < N) {
        // a wavefront takes 8 consecutive rows per turn: one 16-byte load of gamma
        // and of beta serves them, and the 8 row segments are in flight together
        for (int d0 = dbeg + 8 * w; d0 < dend; d0 += 8 * 4) {
            u32x4 wv[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) wv[u] = ldg16(W + (size_t)(d0 + u) * N + col);
            const u32x4 gv = ldg16(gamma + d0), bv = ldg16(beta + d0);
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const float ga = (u & 1) ? bf_hi(gv[u >> 1]) : bf_lo(gv[u >> 1]);
                const float be = (u & 1) ? bf_hi(bv[u >> 1]) : bf_lo(bv[u >> 1]);
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const float w0 = bf_lo(wv[u][q]), w1 = bf_hi(wv[u][q]);
                    c[2 * q] = fmaf(ga, w0, c[2 * q]);
                    c[2 * q + 1] = fmaf(ga, w1, c[2 * q + 1]);
                    b[2 * q] = fmaf(be, w0, b[2 * q]);
                    b[2 * q + 1] = fmaf(be, w1, b[2 * q + 1]);
                }
            }
        }
    }
    if (w > 0) {
#pragma unroll
        for (int j = 0; j < 8; ++j) { red[w - 1][0][8 * lane + j] = c[j]; red[w - 1][1][8 * lane + j] = b[j]; }
    }
    __syncthreads();
    if (w == 0 && col < N) {
        float* pc = part + ((size_t)blockIdx.y * 2 + 0) * N + col;
        float* pb = part + ((size_t)blockIdx.y * 2 + 1) * N + col;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            pc[j] = c[j] + red[0][0][8 * lane + j] + red[1][0][8 * lane + j] + red[2][0][8 * lane + j];
            pb[j] = b[j] + red[0][1][8 * lane + j] + red[1][1][8 * lane + j] + red[2][1][8 * lane + j];
        }
    }
}
__global__ __launch_bounds__(256) void colvec_sum_kernel(const float* part, float* colc, float* colb, int N) {
    const int n = blockIdx.x * 256 + threadIdx.x;
    if (n >= N) return;
    float c = 0.f, b = 0.f;
#pragma unroll
    for (int y = 0; y < COLVEC_SPLITS; ++y) {
        c += part[((size_t)y * 2 + 0) * N + n];
        b += part[((size_t)y * 2 + 1) * N + n];
    }
    colc[n] = c;
    colb[n] = b;
}

// The same column vectors for a transposed weight Wt [N, D]: colc[n] = sum_d
// gamma[d] Wt[n,d], colb[n] = sum_d beta[d] Wt[n,d].  One wavefront per row n
// (contiguous reads of 1 KiB), wavefront reduction at the end.
__global__ __launch_bounds__(256) void colvec_t_kernel(const u16* Wt, const u16* gamma, const u16* beta,
                                                       float* colc, float* colb, int D, int N) {
    const int lane = threadIdx.x & 63;
    const int n = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (n >= N) return;
    float c = 0.f, b = 0.f;
    for (int d0 = 8 * lane; d0 < D; d0 += 512 * 4) {          // four chunks in flight
        u32x4 wv[4], gv[4], bv[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int d = d0 + 512 * u;
            const bool ok = d < D;
            wv[u] = ok ? ldg16(Wt + (size_t)n * D + d) : zero4();
            gv[u] = ok ? ldg16(gamma + d) : zero4();
            bv[u] = ok ? ldg16(beta + d) : zero4();
        }
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const float w0 = bf_lo(wv[u][q]), w1 = bf_hi(wv[u][q]);
                c = fmaf(bf_lo(gv[u][q]), w0, c); c = fmaf(bf_hi(gv[u][q]), w1, c);
                b = fmaf(bf_lo(bv[u][q]), w0, b); b = fmaf(bf_hi(bv[u][q]), w1, b);
            }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) { c += __shfl_xor(c, o); b += __shfl_xor(b, o); }
    if (lane == 0) { colc[n] = c; colb[n] = b; }
}

__global__ __launch_bounds__(256) void fill_zero_kernel(u32x4* p, size_t n16) {
    const u32x4 z = {0u, 0u, 0u, 0u};
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256) p[i] = z;
}

// ---- calibration -----------------------------------------------------------
__global__ __launch_bounds__(256) void calib_copy_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst,
                                                         size_t n16) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256) dst[i] = src[i];
}

__global__ __launch_bounds__(256) void calib_read_kernel(const u32x4* __restrict__ src, size_t n16, float* sink) {
    const size_t stride = (size_t)gridDim.x * 256;
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    u32 acc = 0;
    for (; i + 7 * stride < n16; i += 8 * stride) {
        u32x4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = src[i + u * stride];
#pragma unroll
        for (int u = 0; u < 8; ++u) acc ^= v[u][0] ^ v[u][1] ^ v[u][2] ^ v[u][3];
    }
    for (; i < n16; i += stride) { const u32x4 v = src[i]; acc ^= v[0] ^ v[1] ^ v[2] ^ v[3]; }
    if (acc == 0x9e3779b9u) sink[blockIdx.x & 4095] = 1.f;   // practically never: keeps the loads alive
}

__global__ __launch_bounds__(256) void calib_mfma_kernel(float* sink, int iters) {
    Chunk a, b;
#pragma unroll
    for (int q = 0; q < 4; ++q) { a.u[q] = 0x3f803f80u; b.u[q] = 0x3f003f00u; }
    f32x16 acc[16];
#pragma unroll
    for (int s = 0; s < 16; ++s)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[s][v] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int s = 0; s < 16; ++s) acc[s] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.v, b.v, acc[s], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int k = 0; k < 16; ++k)
#pragma unroll
        for (int v = 0; v < 16; ++v) s += acc[k][v];
    if (s == -1.f) sink[threadIdx.x & 63] = s;
}

// Same instruction stream, but the operands come from memory (lane t takes the
// 16-byte chunks t, t + 256, ... of `src`, 8 chunks in all): with real-valued
// random operands the matrix cores draw more power than with constants and the
// chip lowers its clock, so this is the attainable rate for real data.
__global__ __launch_bounds__(256) void calib_mfma_data_kernel(const u32x4* src, float* sink, int iters) {
    Chunk a[4], b[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) { a[i].u = src[threadIdx.x + 256 * i]; b[i].u = src[threadIdx.x + 256 * (i + 4)]; }
    f32x16 acc[16];
#pragma unroll
    for (int s = 0; s < 16; ++s)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[s][v] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int s = 0; s < 16; ++s)
            acc[s] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[s & 3].v, b[s >> 2].v, acc[s], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int k = 0; k < 16; ++k)
#pragma unroll
        for (int v = 0; v < 16; ++v) s += acc[k][v];
    if (s == -1.f) sink[threadIdx.x & 63] = s;
}

}  // namespace bb
