// Norm-prologue bf16 GEMM for gfx950.
//
// One kernel template covers the compute-bound block programs:
//
//  MODE_GATEUP  first stage of Example 3's first snapshot (the K-map of the
//               fused M-map): per output tile one serial loop over the model
//               dimension that accumulates sum x^2 and both products
//               (X diag(g)) W1, (X diag(g)) W3 from ONE load of the X tile
//               (Rule 2), then applies the inverse norm after the dots
//               (Rule 4), Swish, the Hadamard product, and stores the hidden.
//  MODE_LN      Example 2's final fused nest: one loop accumulating sum x,
//               sum x^2 and (X diag(gamma)) W; epilogue
//               r (P - mu c) + b with c = gamma^T W, b = beta^T W (Rule 5, 4).
//  MODE_PLAIN   C = A B, used for the contraction with W2 and by the unfused
//               block programs.
//
// Layouts: A [M,K] row-major, B [K,N] row-major (contraction index strided),
// C [M,N] row-major, all bf16.  fp32 accumulation in 32x32x16 matrix
// instructions.
//
// Tiling: 256 threads = 4 wavefronts (2x2), workgroup tile BM x 256 columns
// (GATEUP: 128 hidden units = 128 columns of W1 + the same 128 of W3),
// contraction step 64.  Tiles go global -> registers -> LDS.  LDS is double
// buffered with one barrier per step.  While step k is multiplied, tile k+1
// moves from the registers into the idle LDS buffer in four parts, one after
// each group of matrix instructions, and each part's registers are at once
// refilled with tile k+2; so the vector ALU work of the prologue and the
// global-load latency both run in the shadow of the matrix cores.
// The A tile is scaled by the gain and rounded to bf16 on its way
// into LDS and its row sums are accumulated from the same registers.  The B
// tile is transposed 8x8 in registers so that LDS holds contraction-contiguous
// 16-byte chunks for both operands.  B columns are stored in LDS in a permuted
// order chosen so that (a) LDS writes and reads are bank-conflict free and
// (b) every lane ends up owning consecutive output columns for wide stores.
#pragma once
#include <type_traits>

#include "bb_common.h"

namespace bb {

enum { MODE_PLAIN = 0, MODE_GATEUP = 1, MODE_LN = 2 };

struct GemmArgs {
    const u16* A;        // [M, K]
    const u16* B0;       // [K, N]
    const u16* B1;       // [K, N]  (GATEUP only: W3)
    u16* C;              // [M, N]
    const u16* gain;     // [K]     (GATEUP: g, LN: gamma)
    const float* colc;   // [N]     (LN: gamma^T W)
    const float* colb;   // [N]     (LN: beta^T W)
    int M, N, K;
    int lda, ldb, ldc;
    int tiles_m, tiles_n, tiles_per_xcd;
    float eps;
};

constexpr int GEMM_THREADS = 256;
constexpr int GEMM_BK = 64;

template <int MODE, int BM>
struct GemmSmem {
    u32x4 a[2][BM * 8];
    u32x4 b[2][256 * 8];
    float stat0[BM];   // inverse norm / inverse std
    float stat1[BM];   // mean (LN)
};

// FULL: every tile is complete (M % BM == 0, N % columns-per-tile == 0,
// K % 64 == 0), so the main loop has no bounds checks and no branches.
template <int MODE, int BM, bool FULL>
__global__ __launch_bounds__(GEMM_THREADS) void gemm_kernel(const GemmArgs p) {
    constexpr int AI = BM / 32;   // A chunks per thread per step
    constexpr int MT = BM / 64;   // 32-row subtiles per wavefront
    constexpr int NCOL = (MODE == MODE_GATEUP) ? 128 : 256;  // output columns per tile
    __shared__ GemmSmem<MODE, BM> sm;

    // ---- tile coordinates: workgroup id -> XCD (id % 8) -> contiguous range
    // of tiles per XCD, row tiles fastest, so the tiles resident on one XCD
    // share B columns and A rows in that XCD's L2.
    const int xcd = blockIdx.x & 7, local = blockIdx.x >> 3;
    const int lin = xcd * p.tiles_per_xcd + local;
    if (local >= p.tiles_per_xcd || lin >= p.tiles_m * p.tiles_n) return;
    const int tm = lin % p.tiles_m, tn = lin / p.tiles_m;
    const int m0 = tm * BM, n0 = tn * NCOL;

    const int t = threadIdx.x, lane = t & 63, w = t >> 6;
    const int wm = w >> 1, wn = w & 1;
    const int l32 = lane & 31, lhi = lane >> 5;

    // ---- global-load roles
    const int kcA = t & 7, rowA = t >> 3;     // A: chunk kcA of rows rowA + 32 i
    const int kgB = t >> 5, ngB = t & 31;     // B: rows 8 kgB .. +7, column group ngB
    const u16* Bsrc;
    int colB;                                  // first of the 8 columns this thread loads
    if (MODE == MODE_GATEUP) {
        Bsrc = (ngB >> 4) ? p.B1 : p.B0;
        colB = n0 + 8 * (ngB & 15);
    } else {
        Bsrc = p.B0;
        colB = n0 + 8 * ngB;
    }
    const bool colB_ok = FULL || colB < p.N;

    // LDS row (rho) of each of this thread's 8 B columns
    int rhoB[8];
#pragma unroll
    for (int c = 0; c < 8; ++c) {
        if (MODE == MODE_GATEUP) {
            const int which = ngB >> 4, ngp = ngB & 15;
            const int tt = 4 * (ngp >> 3) + 2 * which + (c & 1);
            rhoB[c] = 32 * tt + (ngp & 7) + 8 * (c >> 1);
        } else {
            rhoB[c] = 32 * (4 * (ngB >> 4) + (c & 3)) + 16 * (c >> 2) + (ngB & 15);
        }
    }

    // one register set holds the tile that is in flight (two steps ahead of the
    // one being multiplied); the gain chunk alternates between two registers
    u32x4 ra[AI], rb[2][8], rg_cur = zero4(), rg_nxt = zero4();
    float ssq[AI], ssum[AI];
#pragma unroll
    for (int i = 0; i < AI; ++i) { ssq[i] = 0.f; ssum[i] = 0.f; }
    constexpr int APER = AI / 4;

    // B block (8 contraction rows x 8 columns) of tile kt -> B register set S
    auto gload_b = [&](int kt, auto SETC) {
        constexpr int S = decltype(SETC)::value;
        const int k0 = kt * GEMM_BK;
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            const int k = k0 + 8 * kgB + r;
            rb[S][r] = (FULL || (colB_ok && k < p.K)) ? ldg16(Bsrc + (size_t)k * p.ldb + colB) : zero4();
        }
    };
    // loads part `part` (0..3) of the A tile kt: AI/4 chunks
    auto gload_part = [&](int kt, auto PARTC) {
        constexpr int part = decltype(PARTC)::value;
        const int k0 = kt * GEMM_BK;
        const int ka = k0 + 8 * kcA;
        const bool ka_ok = FULL || ka < p.K;
#pragma unroll
        for (int ii = 0; ii < APER; ++ii) {
            const int i = part * APER + ii;
            const int m = m0 + rowA + 32 * i;
            ra[i] = (FULL || (ka_ok && m < p.M)) ? ldg16(p.A + (size_t)m * p.lda + ka) : zero4();
        }
    };
    auto gload_gain = [&](int kt) {      // gain chunk of tile kt -> rg_nxt
        if (MODE != MODE_PLAIN) {
            const int ka = kt * GEMM_BK + 8 * kcA;
            rg_nxt = (FULL || ka < p.K) ? ldg16(p.gain + ka) : zero4();
        }
    };

    // part `part` of writing the registers into LDS buffer buf: AI/4 A chunks
    // (scaled, rounded, row sums updated) and the transposed B columns 2 part,
    // 2 part + 1 of B register set S
    auto sstore_part = [&](int buf, auto SETC, auto PARTC) {      // uses the gain chunk in rg_cur
        constexpr int S = decltype(SETC)::value;
        constexpr int part = decltype(PARTC)::value;
        const u32x4 gv = rg_cur;
#pragma unroll
        for (int ii = 0; ii < APER; ++ii) {
            const int i = part * APER + ii;
            u32x4 v = ra[i];
            if (MODE != MODE_PLAIN) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const u32 xw = v[q];
                    const bf16x2 xb = *reinterpret_cast<const bf16x2*>(&xw);
                    ssq[i] = __builtin_amdgcn_fdot2_f32_bf16(xb, xb, ssq[i], false);
                    if (MODE == MODE_LN) {
                        const u32 onew = 0x3f803f80u;
                        ssum[i] = __builtin_amdgcn_fdot2_f32_bf16(xb, *reinterpret_cast<const bf16x2*>(&onew), ssum[i], false);
                    }
                    v[q] = pack_bf16(bf_lo(xw) * bf_lo(gv[q]), bf_hi(xw) * bf_hi(gv[q]));
                }
            }
            sm.a[buf][lds_pos(rowA + 32 * i, kcA)] = v;
        }
#pragma unroll
        for (int cc = 0; cc < 2; ++cc) {
            const int c = 2 * part + cc;
            u32x4 o;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const u32 a = rb[S][2 * q][c >> 1], b = rb[S][2 * q + 1][c >> 1];
                o[q] = (c & 1) ? pack_hi(a, b) : pack_lo(a, b);
            }
            sm.b[buf][lds_pos(rhoB[c], kgB)] = o;
        }
    };

    f32x16 acc[MT][4];
#pragma unroll
    for (int s = 0; s < MT; ++s)
#pragma unroll
        for (int tt = 0; tt < 4; ++tt)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[s][tt][v] = 0.f;

    using C0 = std::integral_constant<int, 0>;
    using C1 = std::integral_constant<int, 1>;
    using C2 = std::integral_constant<int, 2>;
    using C3 = std::integral_constant<int, 3>;

    const int nk = (p.K + GEMM_BK - 1) / GEMM_BK;
    using CT = std::true_type;
    using CF = std::false_type;

    // one contraction step: multiply LDS buffer kt&1; meanwhile (STORE) tile
    // kt+1 goes from the registers into the other buffer, one part per group
    // of 16 matrix instructions, and (LOAD) each part's registers are refilled
    // with tile kt+2.  The scheduling directives spread each part's vector
    // ALU, LDS and global-load instructions between the matrix instructions
    // (they issue in order, so only instructions placed between two matrix
    // instructions run in the shadow of the first), and fetch the fragments of
    // the next group while the current one is multiplied.
    Chunk fa[2][MT], fb[2][4];
    auto frag_load = [&](int buf, int ks, auto SETC) {
        constexpr int S = decltype(SETC)::value;
        const int kc = 2 * ks + lhi;
#pragma unroll
        for (int s = 0; s < MT; ++s) fa[S][s].u = sm.a[buf][lds_pos(wm * (BM / 2) + 32 * s + l32, kc)];
#pragma unroll
        for (int tt = 0; tt < 4; ++tt) fb[S][tt].u = sm.b[buf][lds_pos(wn * 128 + 32 * tt + l32, kc)];
    };
    auto mma = [&](auto SETC) {
        constexpr int S = decltype(SETC)::value;
#pragma unroll
        for (int s = 0; s < MT; ++s)
#pragma unroll
            for (int tt = 0; tt < 4; ++tt)
                acc[s][tt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[S][s].v, fb[S][tt].v, acc[s][tt], 0, 0, 0);
    };
    constexpr int NMMA = 4 * MT;                                       // matrix instructions per group
    constexpr int VALU_PER = (MODE == MODE_PLAIN ? 24 : 24 + 28 * APER) / NMMA + 1;
    auto interleave = [&](bool with_frags) {
        // (the compiler honours data dependences; the pattern below is a placement request)
        if (with_frags) __builtin_amdgcn_sched_group_barrier(0x100, MT + 4, 0);      // LDS reads first
#pragma unroll
        for (int i = 0; i < NMMA; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                       // one matrix instruction
            __builtin_amdgcn_sched_group_barrier(0x002, VALU_PER, 0);                // a slice of the vector ALU work
            if (i % 4 == 3) __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);       // an LDS write
            if (i % 4 == 1) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);       // a global load
        }
    };
    // kl: tile to load (kt + 2, or the last tile when there is no such tile)
    auto step = [&](int kt, int kl) {
        const int buf = kt & 1, nbuf = buf ^ 1;
        __syncthreads();
        gload_gain(kl);
        gload_b(kl, C1());
        frag_load(buf, 0, C0());
        __builtin_amdgcn_sched_barrier(0);
        frag_load(buf, 1, C1());
        mma(C0());
        sstore_part(nbuf, C0(), C0());
        gload_part(kl, C0());
        interleave(true);
        __builtin_amdgcn_sched_barrier(0);
        frag_load(buf, 2, C0());
        mma(C1());
        sstore_part(nbuf, C0(), C1());
        gload_part(kl, C1());
        interleave(true);
        __builtin_amdgcn_sched_barrier(0);
        frag_load(buf, 3, C1());
        mma(C0());
        sstore_part(nbuf, C0(), C2());
        gload_part(kl, C2());
        interleave(true);
        __builtin_amdgcn_sched_barrier(0);
        mma(C1());
        sstore_part(nbuf, C0(), C3());
        gload_part(kl, C3());
        interleave(false);
        __builtin_amdgcn_sched_barrier(0);
        rg_cur = rg_nxt;
    };
    auto last_step = [&](int kt) {          // nothing left to store or load
        const int buf = kt & 1;
        __syncthreads();
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            frag_load(buf, ks, C0());
            mma(C0());
        }
    };

    // prologue: tile 0 into LDS buffer 0, tile 1 in flight.  Loads past the last
    // tile are redirected to the last tile (always valid memory); what they
    // bring is never stored to LDS.
    gload_gain(0);
    rg_cur = rg_nxt;
    gload_b(0, C0());
    gload_part(0, C0()); gload_part(0, C1()); gload_part(0, C2()); gload_part(0, C3());
    const int t1 = min(1, nk - 1);
    gload_gain(t1);
    gload_b(t1, C1());
    sstore_part(0, C0(), C0()); gload_part(t1, C0());
    sstore_part(0, C0(), C1()); gload_part(t1, C1());
    sstore_part(0, C0(), C2()); gload_part(t1, C2());
    sstore_part(0, C0(), C3()); gload_part(t1, C3());
    rg_cur = rg_nxt;
#pragma unroll
    for (int r = 0; r < 8; ++r) rb[0][r] = rb[1][r];
    // B set 0 always holds tile kt+1, set 1 receives tile kt+2
    for (int kt = 0; kt + 1 < nk; ++kt) {
        step(kt, min(kt + 2, nk - 1));
#pragma unroll
        for (int r = 0; r < 8; ++r) rb[0][r] = rb[1][r];
    }
    last_step(nk - 1);

    // ---- row statistics: finish the sums over the 8 lanes sharing a row
    if (MODE != MODE_PLAIN) {
#pragma unroll
        for (int i = 0; i < AI; ++i) {
            float s2 = ssq[i], s1 = ssum[i];
#pragma unroll
            for (int o = 1; o < 8; o <<= 1) {
                s2 += __shfl_xor(s2, o);
                if (MODE == MODE_LN) s1 += __shfl_xor(s1, o);
            }
            if (kcA == 0) {
                const float invK = 1.0f / (float)p.K;
                if (MODE == MODE_LN) {
                    const float mu = s1 * invK;
                    const float var = fmaxf(s2 * invK - mu * mu, 0.f);
                    sm.stat0[rowA + 32 * i] = rsqrtf(var + p.eps);
                    sm.stat1[rowA + 32 * i] = mu;
                } else {
                    sm.stat0[rowA + 32 * i] = rsqrtf(s2 * invK + p.eps);
                }
            }
        }
        __syncthreads();
    }

    // ---- epilogue.  Accumulator register v of a 32x32 tile belongs to tile
    // row 8 (v / 4) + 4 (lane / 32) + v % 4 and tile column lane % 32.
    if (MODE == MODE_GATEUP) {
        const int fcol = n0 + 64 * wn + 8 * (l32 & 7) + 2 * (l32 >> 3);
        if (fcol < p.N) {
#pragma unroll
            for (int s = 0; s < MT; ++s) {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int rl = wm * (BM / 2) + 32 * s + 8 * (v >> 2) + 4 * lhi + (v & 3);
                    const int m = m0 + rl;
                    if (m < p.M) {
                        const float r = sm.stat0[rl];
                        const float h0 = swiglu(r * acc[s][0][v], r * acc[s][2][v]);
                        const float h1 = swiglu(r * acc[s][1][v], r * acc[s][3][v]);
                        *reinterpret_cast<u32*>(p.C + (size_t)m * p.ldc + fcol) = pack_bf16(h0, h1);
                    }
                }
            }
        }
    } else {
        const int ncol = n0 + 128 * wn + 8 * (l32 & 15) + 4 * (l32 >> 4);
        if (ncol < p.N) {
            float cc[4], cb[4];
            if (MODE == MODE_LN) {
#pragma unroll
                for (int tt = 0; tt < 4; ++tt) { cc[tt] = p.colc[ncol + tt]; cb[tt] = p.colb[ncol + tt]; }
            }
#pragma unroll
            for (int s = 0; s < MT; ++s) {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int rl = wm * (BM / 2) + 32 * s + 8 * (v >> 2) + 4 * lhi + (v & 3);
                    const int m = m0 + rl;
                    if (m < p.M) {
                        float y[4];
#pragma unroll
                        for (int tt = 0; tt < 4; ++tt) y[tt] = acc[s][tt][v];
                        if (MODE == MODE_LN) {
                            const float r = sm.stat0[rl], mu = sm.stat1[rl];
#pragma unroll
                            for (int tt = 0; tt < 4; ++tt) y[tt] = fmaf(r, y[tt] - mu * cc[tt], cb[tt]);
                        }
                        u32x2 o = {pack_bf16(y[0], y[1]), pack_bf16(y[2], y[3])};
                        *reinterpret_cast<u32x2*>(p.C + (size_t)m * p.ldc + ncol) = o;
                    }
                }
            }
        }
    }
}

}  // namespace bb
