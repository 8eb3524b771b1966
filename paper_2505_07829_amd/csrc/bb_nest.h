// The fully fused nest of Example 3 (the listing after Step 26) with one block of output columns
// (N = 1, the case of the Epilogue in which the extended maps replicate no work), for model
// dimensions up to 512, gfx950:
//
//   forall m (block of 16 rows):                       one workgroup
//     statistics loop: sum x^2, bf16(x g) -> local memory
//     for k (block of 128 hidden units):               serial; wavefront w of NW takes blocks w, w + NW, ...
//       P = (x g) W1[:, k],  Q = (x g) W3[:, k]        contraction over the whole model dimension
//       h = SiLU(r P) (r Q)                            inverse norm after the dots (Rule 4); bf16
//       y += h W2[k, :]                                the row block of the output stays in registers
//     store y (+ residual)
//
// Nothing but X, the weights and Y touches global memory: the normalised activations, the
// pre-activations and the hidden never leave the compute unit, and the whole operator is one
// launch.  A 16 x D block of fp32 outputs fits the registers of a workgroup only for small D (a
// wavefront keeps 16 x D partial outputs over its own hidden blocks: 32 registers per 128 columns);
// the wavefronts' partial outputs are added through local memory once, after the loop.
//
// Weight blocks go global memory -> registers -> matrix instruction like in the weight-streaming
// kernel: a lane loads 8 rows x 8 columns with eight 16-byte loads, the 8x8 in-register
// transposition makes them operands of 16x16x32 bf16 matrix instructions.
#pragma once
#include "bb_common.h"

namespace bb {

// wavefronts per workgroup (one per SIMD: a wavefront then has 512 registers for its 16 x D partial outputs, the
// pre-activations and the weight blocks in flight; with two per SIMD the weight blocks no longer fit)
constexpr int nest_waves(int nd) { return 4; }
constexpr int NEST_ROWS = 16;         // rows per workgroup
constexpr int NEST_MAXD = 512;

struct NestArgs {
    const u16* X;      // [M, D]
    const u16* g;      // [D]
    const u16* W1;     // [D, F]
    const u16* W3;     // [D, F]
    const u16* W2;     // [F, D]
    u16* Y;            // [M, D]
    const u16* R;      // [M, D] residual added before the output's one rounding, or null
    int M, D, F;
    float eps;
};

#ifndef BB_HOST_ONLY
// ND: blocks of 128 model channels (D <= 128 ND)
template <int ND>
__global__ __launch_bounds__(64 * nest_waves(ND)) void ffn_nest_kernel(const NestArgs p) {
    constexpr int NW = nest_waves(ND);
    constexpr int TPR = 4 * NW;                    // threads per row in the statistics loop and the final sum
    constexpr int DP = 128 * ND;                   // padded model dimension
    constexpr int AS = DP + 8;                     // row strides in local memory (elements): 16 consecutive rows
    constexpr int HS = 128 + 8;                    // at one column offset fall on 16 different groups of banks
    __shared__ __attribute__((aligned(16))) u16 As[NEST_ROWS * AS];          // bf16(x g)
    __shared__ __attribute__((aligned(16))) u16 Hs[NW * NEST_ROWS * HS];     // a block of the hidden per wavefront
    __shared__ __attribute__((aligned(16))) float red[NW][NEST_ROWS][128];
    __shared__ float rinv[NEST_ROWS];
    const int t = threadIdx.x, lane = t & 63;
    const int w = __builtin_amdgcn_readfirstlane(t >> 6);
    const int jn = lane & 15, g4 = lane >> 4;
    const int r0 = NEST_ROWS * blockIdx.x;

    // ---- statistics loop: TPR threads per row
    {
        const int row = t / TPR, sub = t % TPR;
        const bool row_ok = r0 + row < p.M;
        float ss = 0.f;
#pragma unroll
        for (int j0 = 0; j0 < DP / 8; j0 += TPR) {
            const int j = j0 + sub;                // chunk of 8 model channels
            u32x4 a = zero4();
            if (row_ok && 8 * j < p.D) {
                const u32x4 x = ldg16(p.X + (size_t)(r0 + row) * p.D + 8 * j);
                const u32x4 gg = ldg16(p.g + 8 * j);
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const float x0 = bf_lo(x[q]), x1 = bf_hi(x[q]);
                    ss = fmaf(x0, x0, ss);
                    ss = fmaf(x1, x1, ss);
                    a[q] = pack_bf16(x0 * bf_lo(gg[q]), x1 * bf_hi(gg[q]));
                }
            }
            if (j < DP / 8) *reinterpret_cast<u32x4*>(&As[row * AS + 8 * j]) = a;
        }
        ss += __shfl_xor(ss, 1);
        ss += __shfl_xor(ss, 2);
        ss += __shfl_xor(ss, 4);
        ss += __shfl_xor(ss, 8);
        if (TPR == 32) ss += __shfl_xor(ss, 16);
        if (sub == 0) rinv[row] = row_ok ? rsqrtf(ss / (float)p.D + p.eps) : 0.f;   // rows past M stay exactly zero
    }
    __syncthreads();

    f32x4 accY[ND][8];
#pragma unroll
    for (int nb = 0; nb < ND; ++nb)
#pragma unroll
        for (int c = 0; c < 8; ++c) accY[nb][c] = f32x4{0, 0, 0, 0};
    float ri[4];                                   // inverse norms of the rows of this lane's accumulator elements
#pragma unroll
    for (int e = 0; e < 4; ++e) ri[e] = rinv[4 * g4 + e];
    u16* Hw = Hs + w * NEST_ROWS * HS;

    const int nfb = (p.F + 127) / 128;
    for (int fb = w; fb < nfb; fb += NW) {
        // ---- the two products of the block over the whole model dimension
        const int col = 128 * fb + 8 * jn;
        const bool col_ok = col < p.F;
        f32x4 accP[8], accQ[8];
#pragma unroll
        for (int c = 0; c < 8; ++c) { accP[c] = f32x4{0, 0, 0, 0}; accQ[c] = f32x4{0, 0, 0, 0}; }
        // (D <= 256: two blocks of 32 model channels per trip, 32 loads in flight; beyond, the output block
        // takes the registers that would need)
#pragma clang loop unroll_count(ND <= 2 ? 2 : 1)
        for (int kb = 0; kb < 4 * ND; ++kb) {
            const int d0 = 32 * kb + 8 * g4;
            u32x4 r1[8], r3[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const bool ok = col_ok && d0 + i < p.D;
                r1[i] = ok ? ldg16(p.W1 + (size_t)(d0 + i) * p.F + col) : zero4();
                r3[i] = ok ? ldg16(p.W3 + (size_t)(d0 + i) * p.F + col) : zero4();
            }
            Chunk xa;
            xa.u = *reinterpret_cast<const u32x4*>(&As[jn * AS + d0]);
            u32x4 t1[8], t3[8];
            transpose8x8(r1, t1);
            transpose8x8(r3, t3);
#pragma unroll
            for (int c = 0; c < 8; ++c) {
                Chunk b1, b3;
                b1.u = t1[c];
                b3.u = t3[c];
                accP[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xa.v, b1.v, accP[c], 0, 0, 0);
                accQ[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xa.v, b3.v, accQ[c], 0, 0, 0);
            }
        }
        // ---- the hidden block: acc[c][e] is row 4 g4 + e, hidden unit 8 jn + c of the block
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            u32x4 h;
#pragma unroll
            for (int q = 0; q < 4; ++q)
                h[q] = pack_bf16(swiglu(ri[e] * accP[2 * q][e], ri[e] * accQ[2 * q][e]),
                                 swiglu(ri[e] * accP[2 * q + 1][e], ri[e] * accQ[2 * q + 1][e]));
            *reinterpret_cast<u32x4*>(&Hw[(4 * g4 + e) * HS + 8 * jn]) = h;
        }
        // (written and read by this wavefront only: its local-memory operations execute in order, and the
        // compiler keeps the order of accesses to one array that it cannot tell apart)
        // ---- y += h W2[block, :]
#pragma clang loop unroll_count(ND <= 2 ? 2 : 1)
        for (int kb2 = 0; kb2 < 4; ++kb2) {
            const int h0 = 128 * fb + 32 * kb2 + 8 * g4;
            Chunk ha;
            ha.u = *reinterpret_cast<const u32x4*>(&Hw[jn * HS + 32 * kb2 + 8 * g4]);
#pragma unroll
            for (int nb = 0; nb < ND; ++nb) {
                const int cy = 128 * nb + 8 * jn;
                u32x4 r2[8];
#pragma unroll
                for (int i = 0; i < 8; ++i)
                    r2[i] = (cy < p.D && h0 + i < p.F) ? ldg16(p.W2 + (size_t)(h0 + i) * p.D + cy) : zero4();
                u32x4 t2[8];
                transpose8x8(r2, t2);
#pragma unroll
                for (int c = 0; c < 8; ++c) {
                    Chunk b2;
                    b2.u = t2[c];
                    accY[nb][c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ha.v, b2.v, accY[nb][c], 0, 0, 0);
                }
            }
        }
    }

    // ---- the wavefronts' partial outputs are added, the residual joins, one rounding, store
#pragma unroll
    for (int nb = 0; nb < ND; ++nb) {
        __syncthreads();
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const f32x4 lo = {accY[nb][0][e], accY[nb][1][e], accY[nb][2][e], accY[nb][3][e]};
            const f32x4 hi = {accY[nb][4][e], accY[nb][5][e], accY[nb][6][e], accY[nb][7][e]};
            float* s = &red[w][4 * g4 + e][8 * jn];
            *reinterpret_cast<f32x4*>(s) = lo;
            *reinterpret_cast<f32x4*>(s + 4) = hi;
        }
        __syncthreads();
        const int row = t >> 4, cc = 8 * (t & 15);
        const int cy = 128 * nb + cc;
        if (t < 256 && r0 + row < p.M && cy < p.D) {
            f32x4 y0 = {0, 0, 0, 0}, y1 = y0;
#pragma unroll
            for (int ww = 0; ww < NW; ++ww) {
                y0 += *reinterpret_cast<const f32x4*>(&red[ww][row][cc]);
                y1 += *reinterpret_cast<const f32x4*>(&red[ww][row][cc + 4]);
            }
            if (p.R != nullptr) {
                const u32x4 rr = ldg16(p.R + (size_t)(r0 + row) * p.D + cy);
                y0 += f32x4{bf_lo(rr[0]), bf_hi(rr[0]), bf_lo(rr[1]), bf_hi(rr[1])};
                y1 += f32x4{bf_lo(rr[2]), bf_hi(rr[2]), bf_lo(rr[3]), bf_hi(rr[3])};
            }
            const u32x4 o = {pack_bf16(y0[0], y0[1]), pack_bf16(y0[2], y0[3]), pack_bf16(y1[0], y1[1]),
                             pack_bf16(y1[2], y1[3])};
            *reinterpret_cast<u32x4*>(p.Y + (size_t)(r0 + row) * p.D + cy) = o;
        }
    }
}
#endif  // BB_HOST_ONLY

}  // namespace bb
