// The fully fused nest of Example 3 (the listing after Step 26) with one block of output columns
// (N = 1, the case of the Epilogue in which the extended maps replicate no work), for model
// dimensions up to 512, gfx950:
//
//   forall m (block of 16 rows):                       one workgroup
//     statistics loop: sum x^2, bf16(x g) -> local memory
//     for k (block of 128 hidden units):               serial; pair j of NP wavefront pairs takes blocks j, j + NP, ...
//       P = (x g) W1[:, k],  Q = (x g) W3[:, k]        contraction over the whole model dimension
//       h = SiLU(r P) (r Q)                            inverse norm after the dots (Rule 4); bf16
//       y += h W2[k, :]                                the row block of the output stays in registers
//     store y (+ residual)
//
// Nothing but X, the weights and Y touches global memory: the normalised activations, the
// pre-activations and the hidden never leave the compute unit, and the whole operator is one
// launch.  A 16 x D block of fp32 outputs fits the registers of a workgroup only for small D.
//
// A block of rows is served by ONE compute unit, which reads all three weight matrices along a chain
// of dependent load -> matrix instruction steps, so the kernel is bound by the latency of that chain
// and by how many loads the compute unit keeps in flight.  Hence many wavefronts with few registers
// each: the two wavefronts of a pair share a hidden block - one computes P, the other Q; P crosses
// over through local memory, the Q wavefront forms the hidden block in local memory, and each of the
// two then multiplies it with its half of the columns of W2.  With six (four) pairs, as many hidden
// blocks are in flight per compute unit.  The pairs' partial outputs are added through local memory
// once, after the loop.
//
// Weight blocks go global memory -> registers -> matrix instruction like in the weight-streaming
// kernel: a lane loads 8 rows x 8 columns with eight 16-byte loads, the 8x8 in-register
// transposition makes them operands of 16x16x32 bf16 matrix instructions.
#pragma once
#include <type_traits>

#include "bb_common.h"

namespace bb {

// wavefronts per workgroup: 12 (three per SIMD, 168 registers each: the kernel needs 162) while a wavefront's share of
// the output block is 16 x 128 (D <= 256), else 8
constexpr int nest_waves(int nd) { return nd <= 2 ? 12 : 8; }
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
// ND: blocks of 128 model channels (D <= 128 ND), 2 or 4
template <int ND>
__global__ __launch_bounds__(64 * nest_waves(ND)) void ffn_nest_kernel(const NestArgs p) {
    static_assert(ND == 2 || ND == 4, "two or four blocks of 128 model channels");
    constexpr int NW = nest_waves(ND), NP = NW / 2;
    constexpr int NBW = ND / 2;                    // blocks of 128 output columns per wavefront
    constexpr int DP = 128 * ND;                   // padded model dimension
    constexpr int AS = DP + 8;                     // row strides in local memory (elements): 16 consecutive rows
    constexpr int HS = 128 + 8;                    // at one column offset fall on 16 different groups of banks
    __shared__ __attribute__((aligned(16))) u16 As[NEST_ROWS * AS];          // bf16(x g)
    __shared__ __attribute__((aligned(16))) u16 Hs[NP * NEST_ROWS * HS];     // a block of the hidden per pair
    // P on its way from one wavefront of a pair to the other ([pair][register][lane]); after the loop the pairs'
    // partial outputs ([pair][row][128 columns])
    __shared__ __attribute__((aligned(16))) f32x4 Px[NP * 8 * 64];
    __shared__ float rinv[NEST_ROWS];
    const int t = threadIdx.x, lane = t & 63;
    const int w = __builtin_amdgcn_readfirstlane(t >> 6);
    const int pr = w >> 1, half = w & 1;           // half 0: W1 and the even output blocks; 1: W3 and the odd ones
    const int jn = lane & 15, g4 = lane >> 4;
    const int r0 = NEST_ROWS * blockIdx.x;

    u16* const Hp = Hs + pr * NEST_ROWS * HS;
    f32x4* const Pp = Px + pr * 8 * 64;
    const u16* const Wa = half ? p.W3 : p.W1;
    const int nfb = (p.F + 127) / 128;

    // weight blocks: 8 rows x 8 columns per lane (rows d0 .. d0 + 7 of W1 or W3, columns col .. col + 7)
    auto load_pq = [&](int fb, int kb, u32x4 (&r)[8]) {
        const int col = 128 * fb + 8 * jn, d0 = 32 * kb + 8 * g4;
        const bool col_ok = fb < nfb && col < p.F;
#pragma unroll
        for (int i = 0; i < 8; ++i)
            r[i] = (col_ok && d0 + i < p.D) ? ldg16(Wa + (size_t)(d0 + i) * p.F + col) : zero4();
    };
    // (rows h0 .. h0 + 7 of W2, this wavefront's i2-th block of output columns)
    auto load_w2 = [&](int fb, int kb2, int i2, u32x4 (&r2)[8]) {
        const int h0 = 128 * fb + 32 * kb2 + 8 * g4, cy = 128 * (2 * i2 + half) + 8 * jn;
#pragma unroll
        for (int i = 0; i < 8; ++i)
            r2[i] = (fb < nfb && cy < p.D && h0 + i < p.F) ? ldg16(p.W2 + (size_t)(h0 + i) * p.D + cy) : zero4();
    };

    // The weights do not depend on the rows: the first block of this wavefront's first product is requested
    // before the statistics loop and arrives while that loop runs.
    u32x4 rfirst[8];
    load_pq(pr, 0, rfirst);

    // ---- statistics loop: 32 threads per row (the first 512 threads)
    if (t < 32 * NEST_ROWS) {
        const int row = t >> 5, sub = t & 31;
        const bool row_ok = r0 + row < p.M;
        float ss = 0.f;
#pragma unroll
        for (int j0 = 0; j0 < DP / 8; j0 += 32) {
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
            *reinterpret_cast<u32x4*>(&As[row * AS + 8 * j]) = a;
        }
        ss += __shfl_xor(ss, 1);
        ss += __shfl_xor(ss, 2);
        ss += __shfl_xor(ss, 4);
        ss += __shfl_xor(ss, 8);
        ss += __shfl_xor(ss, 16);
        if (sub == 0) rinv[row] = row_ok ? rsqrtf(ss / (float)p.D + p.eps) : 0.f;   // rows past M stay exactly zero
    }
    __syncthreads();

    f32x4 accY[NBW][8];
#pragma unroll
    for (int i = 0; i < NBW; ++i)
#pragma unroll
        for (int c = 0; c < 8; ++c) accY[i][c] = f32x4{0, 0, 0, 0};

    // One trip of the serial loop over hidden blocks: pair `pr` takes block fb0 + pr.  Every pair makes the same
    // number of trips (the barriers inside are the workgroup's); FIRST: the trip whose first weight block is
    // already on its way.
    auto trip = [&](int fb0, auto FIRST) {
        const int fb = fb0 + pr;
        const bool active = fb < nfb;
        // ---- this wavefront's product of the block over the whole model dimension
        f32x4 acc[8];
#pragma unroll
        for (int c = 0; c < 8; ++c) acc[c] = f32x4{0, 0, 0, 0};
        auto pq_step = [&](const u32x4 (&r)[8], int kb) {
            Chunk xa;
            xa.u = *reinterpret_cast<const u32x4*>(&As[jn * AS + 32 * kb + 8 * g4]);
            u32x4 tr[8];
            transpose8x8(r, tr);
#pragma unroll
            for (int c = 0; c < 8; ++c) {
                Chunk b;
                b.u = tr[c];
                acc[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xa.v, b.v, acc[c], 0, 0, 0);
            }
        };
        if (active) {
            if (decltype(FIRST)::value) pq_step(rfirst, 0);
#pragma clang loop unroll_count(ND <= 2 ? 1 : 2)
            for (int kb = decltype(FIRST)::value ? 1 : 0; kb < 4 * ND; ++kb) {
                u32x4 r[8];
                load_pq(fb, kb, r);
                pq_step(r, kb);
            }
        }
        // (W2 does not depend on the hidden block: its first block is requested before the exchange)
        u32x4 r2first[8];
        load_w2(fb, 0, 0, r2first);
        // ---- P crosses over; the Q wavefront forms the hidden block: acc[c][e] is row 4 g4 + e, hidden unit
        // 8 jn + c of the block
        if (half == 0) {
#pragma unroll
            for (int c = 0; c < 8; ++c) Pp[c * 64 + lane] = acc[c];
        }
        __syncthreads();
        if (half == 1 && active) {
            float ri[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) ri[e] = rinv[4 * g4 + e];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const f32x4 p0 = Pp[(2 * q) * 64 + lane], p1 = Pp[(2 * q + 1) * 64 + lane];
                u32 h[4];
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    h[e] = pack_bf16(swiglu(ri[e] * p0[e], ri[e] * acc[2 * q][e]),
                                     swiglu(ri[e] * p1[e], ri[e] * acc[2 * q + 1][e]));
#pragma unroll
                for (int e = 0; e < 4; ++e) *reinterpret_cast<u32*>(&Hp[(4 * g4 + e) * HS + 8 * jn + 2 * q]) = h[e];
            }
        }
        __syncthreads();
        // ---- y += h W2[block, :] for this wavefront's blocks of output columns
        if (active) {
            auto y_step = [&](const u32x4 (&r2)[8], int kb2, int i2) {
                Chunk ha;
                ha.u = *reinterpret_cast<const u32x4*>(&Hp[jn * HS + 32 * kb2 + 8 * g4]);
                u32x4 t2[8];
                transpose8x8(r2, t2);
#pragma unroll
                for (int c = 0; c < 8; ++c) {
                    Chunk b2;
                    b2.u = t2[c];
                    accY[i2][c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ha.v, b2.v, accY[i2][c], 0, 0, 0);
                }
            };
            y_step(r2first, 0, 0);
#pragma clang loop unroll_count(ND <= 2 ? 1 : 2)
            for (int s = 1; s < 4 * NBW; ++s) {            // step s: block s / NBW of 32 hidden units, column block s % NBW
                u32x4 r2[8];
                load_w2(fb, s / NBW, s % NBW, r2);
                y_step(r2, s / NBW, s % NBW);
            }
        }
        // (the next trip writes P after this trip's hidden block has been formed, and the hidden block after the
        // next barrier, which every wavefront reaches only when it is done reading this one)
    };
    trip(0, std::true_type());
    for (int fb0 = NP; fb0 < nfb; fb0 += NP) trip(fb0, std::false_type());

    // ---- the pairs' partial outputs are added, the residual joins, one rounding, store: one block of 128
    // output columns at a time
    float* const red = reinterpret_cast<float*>(Px);          // [pair][row][128]
#pragma unroll
    for (int nb = 0; nb < ND; ++nb) {
        __syncthreads();
        if (half == (nb & 1)) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const f32x4 lo = {accY[nb >> 1][0][e], accY[nb >> 1][1][e], accY[nb >> 1][2][e], accY[nb >> 1][3][e]};
                const f32x4 hi = {accY[nb >> 1][4][e], accY[nb >> 1][5][e], accY[nb >> 1][6][e], accY[nb >> 1][7][e]};
                float* s = &red[(pr * NEST_ROWS + 4 * g4 + e) * 128 + 8 * jn];
                *reinterpret_cast<f32x4*>(s) = lo;
                *reinterpret_cast<f32x4*>(s + 4) = hi;
            }
        }
        __syncthreads();
        const int row = t >> 4, cc = 8 * (t & 15);
        const int cy = 128 * nb + cc;
        if (t < 256 && r0 + row < p.M && cy < p.D) {
            f32x4 y0 = {0, 0, 0, 0}, y1 = y0;
#pragma unroll
            for (int pp = 0; pp < NP; ++pp) {
                y0 += *reinterpret_cast<const f32x4*>(&red[(pp * NEST_ROWS + row) * 128 + cc]);
                y1 += *reinterpret_cast<const f32x4*>(&red[(pp * NEST_ROWS + row) * 128 + cc + 4]);
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
