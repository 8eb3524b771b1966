// Weight-streaming RMSNorm -> FFN-SwiGLU kernel for few rows (decode), gfx950.
//
// With at most 16 rows the operator is a pure stream over the three weight
// matrices.  One cooperative persistent kernel (one workgroup per compute
// unit) runs the two maps of Example 3's first fused snapshot back to back:
//
//   phase 1 (K-map): work item = (block of 128 hidden units, block of 32 model
//     channels).  Items are dealt out evenly over the workgroups, so the
//     reduction over the model dimension is a PARALLEL reduction (Rule 3,
//     atomic form): partial pre-activations (X diag(g)) W1, (X diag(g)) W3 are
//     summed with fp32 atomics into a cache-resident scratch of 2 x 16 x F
//     floats, together with sum x^2.
//   grid barrier
//   phase 2 (N-map): work item = (block of 128 output columns, block of 32
//     hidden units).  The consumer applies the inverse norm after the dots
//     (Rule 4), Swish and the gate to the pre-activations it reads back, and
//     contracts with W2; partial outputs are again reduced with fp32 atomics.
//     The last workgroup to finish an output block converts it to bf16.
//
// Every weight element is read from HBM exactly once, by exactly one
// wavefront, with 16-byte loads that cover 256 contiguous bytes per row; the
// 8x8 in-register transposition turns them into matrix-instruction operands
// without touching LDS.  Scratch buffers are all-zero on entry and are
// returned to all-zero: the output accumulator by the finishing workgroup,
// the pre-activation buffer by the NEXT call (two buffers alternate).
#pragma once
#include <hip/hip_cooperative_groups.h>

#include "bb_common.h"

namespace bb {

constexpr int STREAM_THREADS = 256;

struct StreamArgs {
    const u16* X;      // [M, D], M <= 16
    const u16* g;      // [D]
    const u16* W1;     // [D, F]
    const u16* W3;     // [D, F]
    const u16* W2;     // [F, D]
    u16* Y;            // [M, D]
    float* pq;         // [2][16][Fp] pre-activations of this call, zero on entry
    float* ssq;        // [16] row sums of squares of this call, zero on entry
    float* zero_ptr;   // the other call parity's pq+ssq block, zeroed here
    int zero_count4;   // its length in float4
    float* yacc;       // [16][D] output accumulator, zero on entry and exit
    unsigned* cnt;     // [nnb] arrival counters, zero on entry and exit
    int M, D, F, Fp;
    int nkb1, items1, per1;   // phase 1: D/32 blocks, total items, items per workgroup
    int nkb2, items2, per2;   // phase 2: F/32 blocks
    float eps;
};

struct StreamSmem {
    float red[4][2][16][128];   // per-wavefront partial tiles
    unsigned flag;
};

__device__ __forceinline__ void atomic_add_f32(float* p, float v) {
    __hip_atomic_fetch_add(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float coherent_load_f32(const float* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// loads the 8 rows x 8 columns block of a row-major matrix this lane owns
__device__ __forceinline__ void load_block(const u16* base, int ld, int row0, int nrows, int col,
                                           bool col_ok, u32x4 (&r)[8]) {
#pragma unroll
    for (int i = 0; i < 8; ++i)
        r[i] = (col_ok && row0 + i < nrows) ? ldg16(base + (size_t)(row0 + i) * ld + col) : zero4();
}

__global__ __launch_bounds__(STREAM_THREADS) void ffn_stream_kernel(const StreamArgs p) {
    __shared__ StreamSmem sm;
    const int t = threadIdx.x, lane = t & 63, w = t >> 6;
    const int jn = lane & 15, g4 = lane >> 4;
    const int G = gridDim.x, b = blockIdx.x;

    // ---- return the other parity's scratch to zero (nobody uses it now)
    {
        f32x4* z = reinterpret_cast<f32x4*>(p.zero_ptr);
        const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
        for (int i = b * STREAM_THREADS + t; i < p.zero_count4; i += G * STREAM_THREADS) z[i] = zero;
    }

    // =====================  phase 1: pre-activations  =====================
    {
        int i = b * p.per1;
        const int iend = min(i + p.per1, p.items1);
        while (i < iend) {                         // one segment = one hidden block
            const int fb = i / p.nkb1, kb0 = i % p.nkb1;
            const int kb1 = min(p.nkb1, kb0 + (iend - i));
            const int col = 128 * fb + 8 * jn;
            const bool col_ok = col < p.F;
            f32x4 accP[8], accQ[8];
#pragma unroll
            for (int c = 0; c < 8; ++c) { accP[c] = f32x4{0, 0, 0, 0}; accQ[c] = f32x4{0, 0, 0, 0}; }
            float ssq = 0.f;

            u32x4 r1[8], r3[8], rx, rg;
            auto issue = [&](int kb) {
                const int d0 = 32 * kb + 8 * g4;
                load_block(p.W1, p.F, d0, p.D, col, col_ok, r1);
                load_block(p.W3, p.F, d0, p.D, col, col_ok, r3);
                const bool ok = d0 < p.D;
                rx = (ok && jn < p.M) ? ldg16(p.X + (size_t)jn * p.D + d0) : zero4();
                rg = ok ? ldg16(p.g + d0) : zero4();
            };
            int kb = kb0 + w;
            if (kb < kb1) issue(kb);
            while (kb < kb1) {
                // consume the registers of item kb, then refill them for kb + 4
                Chunk xa;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const float x0 = bf_lo(rx[q]), x1 = bf_hi(rx[q]);
                    ssq = fmaf(x0, x0, ssq);
                    ssq = fmaf(x1, x1, ssq);
                    xa.u[q] = pack_bf16(x0 * bf_lo(rg[q]), x1 * bf_hi(rg[q]));
                }
                u32x4 t1[8], t3[8];
                transpose8x8(r1, t1);
                transpose8x8(r3, t3);
                kb += 4;
                if (kb < kb1) issue(kb);
#pragma unroll
                for (int c = 0; c < 8; ++c) {
                    Chunk b1, b3;
                    b1.u = t1[c];
                    b3.u = t3[c];
                    accP[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xa.v, b1.v, accP[c], 0, 0, 0);
                    accQ[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xa.v, b3.v, accQ[c], 0, 0, 0);
                }
            }
            // ---- reduce the 4 wavefronts in LDS, then one atomic per element.
            // accX[c][e] is row (token) 4*g4+e, column 8*jn+c of the block.
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const f32x4 p0 = {accP[0][e], accP[1][e], accP[2][e], accP[3][e]};
                const f32x4 p1 = {accP[4][e], accP[5][e], accP[6][e], accP[7][e]};
                const f32x4 q0 = {accQ[0][e], accQ[1][e], accQ[2][e], accQ[3][e]};
                const f32x4 q1 = {accQ[4][e], accQ[5][e], accQ[6][e], accQ[7][e]};
                float* rp = &sm.red[w][0][4 * g4 + e][8 * jn];
                float* rq = &sm.red[w][1][4 * g4 + e][8 * jn];
                *reinterpret_cast<f32x4*>(rp) = p0;
                *reinterpret_cast<f32x4*>(rp + 4) = p1;
                *reinterpret_cast<f32x4*>(rq) = q0;
                *reinterpret_cast<f32x4*>(rq + 4) = q1;
            }
            if (fb == 0) {   // sum x^2 is counted once: by the items of hidden block 0
                ssq += __shfl_xor(ssq, 16);
                ssq += __shfl_xor(ssq, 32);
                if (lane < 16 && ssq != 0.f) atomic_add_f32(p.ssq + lane, ssq);
            }
            __syncthreads();
#pragma unroll 4
            for (int j = 0; j < 16; ++j) {
                const int idx = t + STREAM_THREADS * j;       // [pq][token][col]
                const int cc = idx & 127, tok = (idx >> 7) & 15, sel = idx >> 11;
                const float v = sm.red[0][sel][tok][cc] + sm.red[1][sel][tok][cc] +
                                sm.red[2][sel][tok][cc] + sm.red[3][sel][tok][cc];
                if (v != 0.f) atomic_add_f32(p.pq + (size_t)(sel * 16 + tok) * p.Fp + 128 * fb + cc, v);
            }
            __syncthreads();
            i += kb1 - kb0;
        }
    }

    // ---- phase 2 work of this workgroup; the first weight blocks are
    // requested BEFORE the grid barrier so that HBM stays busy across it.
    int i2 = b * p.per2;
    const int iend2 = min(i2 + p.per2, p.items2);
    u32x4 rA[8], rB[8];
    auto issue2 = [&](int nb, int kb, int kb1) {
        const int col = 128 * nb + 8 * jn;
        const bool col_ok = col < p.D;
        load_block(p.W2, p.D, 32 * kb + 8 * g4, p.F, col, col_ok && kb < kb1, rA);
        load_block(p.W2, p.D, 32 * (kb + 4) + 8 * g4, p.F, col, col_ok && kb + 4 < kb1, rB);
    };
    bool preloaded = false;
    if (i2 < iend2) {
        const int nb = i2 / p.nkb2, kb0 = i2 % p.nkb2;
        const int kb1 = min(p.nkb2, kb0 + (iend2 - i2));
        issue2(nb, kb0 + w, kb1);
        preloaded = true;
    }

    cooperative_groups::this_grid().sync();

    // =====================  phase 2: down projection  =====================
    {
        const float invD = 1.0f / (float)p.D;
        const float rinv = rsqrtf(coherent_load_f32(p.ssq + jn) * invD + p.eps);  // token jn
        // hidden fragment of token jn, hidden units 32 kb + 8 g4 .. +7 (zero past the end)
        auto hidden = [&](int kb, int kb1) -> Chunk {
            Chunk ha;
            if (kb < kb1) {
                const float* pp = p.pq + (size_t)jn * p.Fp + 32 * kb + 8 * g4;
                const float* qq = pp + (size_t)16 * p.Fp;
                float h[8];
#pragma unroll
                for (int s = 0; s < 8; ++s)
                    h[s] = swiglu(rinv * coherent_load_f32(pp + s), rinv * coherent_load_f32(qq + s));
#pragma unroll
                for (int q = 0; q < 4; ++q) ha.u[q] = pack_bf16(h[2 * q], h[2 * q + 1]);
            } else {
                ha.u = zero4();
            }
            return ha;
        };
        int i = i2;
        const int iend = iend2;
        while (i < iend) {                         // one segment = one output column block
            const int nb = i / p.nkb2, kb0 = i % p.nkb2;
            const int kb1 = min(p.nkb2, kb0 + (iend - i));
            f32x4 acc[8];
#pragma unroll
            for (int c = 0; c < 8; ++c) acc[c] = f32x4{0, 0, 0, 0};
            int kb = kb0 + w;
            if (!preloaded) issue2(nb, kb, kb1);
            preloaded = false;
            while (kb < kb1) {                     // two items (kb, kb + 4) per turn
                const Chunk hA = hidden(kb, kb1), hB = hidden(kb + 4, kb1);
                u32x4 tA[8], tB[8];
                transpose8x8(rA, tA);
                transpose8x8(rB, tB);
                kb += 8;
                if (kb < kb1) issue2(nb, kb, kb1);
#pragma unroll
                for (int c = 0; c < 8; ++c) {
                    Chunk bA, bB;
                    bA.u = tA[c];
                    bB.u = tB[c];
                    acc[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(hA.v, bA.v, acc[c], 0, 0, 0);
                    acc[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(hB.v, bB.v, acc[c], 0, 0, 0);
                }
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const f32x4 y0 = {acc[0][e], acc[1][e], acc[2][e], acc[3][e]};
                const f32x4 y1 = {acc[4][e], acc[5][e], acc[6][e], acc[7][e]};
                float* rp = &sm.red[w][0][4 * g4 + e][8 * jn];
                *reinterpret_cast<f32x4*>(rp) = y0;
                *reinterpret_cast<f32x4*>(rp + 4) = y1;
            }
            __syncthreads();
#pragma unroll 4
            for (int j = 0; j < 8; ++j) {
                const int idx = t + STREAM_THREADS * j;       // [token][col]
                const int cc = idx & 127, tok = idx >> 7;
                const float v = sm.red[0][0][tok][cc] + sm.red[1][0][tok][cc] +
                                sm.red[2][0][tok][cc] + sm.red[3][0][tok][cc];
                if (tok < p.M && 128 * nb + cc < p.D && v != 0.f)
                    atomic_add_f32(p.yacc + (size_t)tok * p.D + 128 * nb + cc, v);
            }
            // ---- arrival count; the last workgroup of this column block
            // converts it to bf16 and returns accumulator and counter to zero
            __threadfence();
            __syncthreads();
            if (t == 0) {
                const unsigned n = (unsigned)(kb1 - kb0);
                const unsigned old = __hip_atomic_fetch_add(p.cnt + nb, n, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
                sm.flag = (old + n == (unsigned)p.nkb2) ? 1u : 0u;
            }
            __syncthreads();
            if (sm.flag) {
                __threadfence();
#pragma unroll 2
                for (int j = 0; j < 4; ++j) {
                    const int idx = t + STREAM_THREADS * j;   // [token][column pair]
                    const int cp = idx & 63, tok = idx >> 6;
                    const int c0 = 128 * nb + 2 * cp;
                    if (tok < p.M && c0 < p.D) {
                        float* a = p.yacc + (size_t)tok * p.D + c0;
                        const float v0 = coherent_load_f32(a), v1 = coherent_load_f32(a + 1);
                        *reinterpret_cast<u32*>(p.Y + (size_t)tok * p.D + c0) = pack_bf16(v0, v1);
                        __hip_atomic_store(a, 0.f, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        __hip_atomic_store(a + 1, 0.f, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    }
                }
                if (t == 0) __hip_atomic_store(p.cnt + nb, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            __syncthreads();
            i += kb1 - kb0;
        }
    }
}

}  // namespace bb
