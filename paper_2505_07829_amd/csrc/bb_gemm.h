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
// contraction step 64, LDS double buffered with one barrier per step.
//
// B operand.  The weight tile (64 contraction rows x 512 bytes) goes from
// global memory straight into LDS (load-to-LDS instructions, no registers, no
// vector ALU work), row-major as it lies in memory.  The matrix instruction
// wants, per lane, 8 consecutive contraction indices of one column; the
// transposing LDS read (ds_read_b64_tr_b16) delivers exactly that from a
// row-major tile, 4 contraction rows x 16 columns per group of 16 lanes.  Its
// 16 lanes read 4 rows x 32 bytes; the 16-byte chunks of a row are XOR-swizzled
// with the low two row bits (in units of 32 bytes) so that these four rows fall
// on different banks.
//
// A operand.  The activation tile goes global -> registers -> LDS because the
// prologue works on it: the row sums are accumulated and the gain is applied
// (rounded to bf16) on the way.  While step k is multiplied, tile k+1 moves
// from the registers into the idle LDS buffer in four parts, one after each
// group of matrix instructions, and each part's registers are at once refilled
// with tile k+2, so the prologue's vector ALU work and the load latency run in
// the shadow of the matrix cores.
//
// Waiting.  The load-to-LDS instructions are issued from inline assembly: the
// compiler's wait-count pass answers a pending load-to-LDS with "wait for
// every outstanding load" at each later use of a loaded register, which would
// serialise the pipeline.  Unknown to the compiler, they are ordered by hand:
// per step, (1) every register the step consumes is touched first, which makes
// the compiler wait for the A loads of the previous step there; (2) then the
// load-to-LDS instructions of the next B tile are issued, then the A loads of
// the tile after it; (3) the step ends with an explicit wait for all of them
// (a count that spares the A loads would be wrong when a wavefront skips
// out-of-range A rows, and would rely on load-to-LDS and register loads
// retiring in issue order).  The compiler's own counts never force the
// completion of a load-to-LDS early, because none is in flight at (1).
// The main loop is unrolled by two so that LDS buffers and register sets are
// named statically; the parity of the step count is a template parameter so
// that no branch with live accumulators on both sides is needed.
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

// 16 zero bytes in global memory: the source of load-to-LDS lanes that fall
// outside the matrix (the instruction cannot write a constant).
static __device__ const u32x4 gemm_zero_chunk = {0u, 0u, 0u, 0u};

typedef __attribute__((__vector_size__(4 * sizeof(short)))) short s16x4;
typedef const void __attribute__((address_space(1))) * gptr_t;
typedef void __attribute__((address_space(3))) * lptr_t;

// s_waitcnt immediate that waits until at most n vector-memory loads are
// outstanding and leaves the other counters alone (gfx9 encoding).
constexpr int vmcnt_imm(int n) { return 0x0F70 | (n & 15) | ((n >> 4) << 14); }

// One load-to-LDS instruction: lane i of the wavefront copies the 16 bytes at
// its own global address src to LDS byte address lds_base + 16 i (lds_base is
// the same for all lanes and travels in M0).
__device__ __forceinline__ void load_to_lds16(const void* src, u32 lds_base) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
                 :: "s"(lds_base), "v"(src) : "memory");
}
__device__ __forceinline__ u32 lds_addr(const void* q) {
    return (u32)(size_t)((__attribute__((address_space(3))) const char*)q);
}

// 4x4 transposition of bf16 values across the four lanes of a quad.
// In: quad lane e holds d0 = (E[0][e], E[1][e]) and d1 = (E[2][e], E[3][e]),
// low half first.  Out: d0 = (E[e][0], E[e][1]), d1 = (E[e][2], E[e][3]).
// sel is 0x05040100 on even lanes and 0x03020706 on odd lanes.
__device__ __forceinline__ void quad_transpose(u32& d0, u32& d1, bool upper, u32 sel) {
    const u32 send = upper ? d0 : d1, keep = upper ? d1 : d0;
    const u32 recv = (u32)__builtin_amdgcn_update_dpp(0, (int)send, 0x4E, 0xF, 0xF, false);   // lane ^ 2
    const u32 x = upper ? recv : keep, y = upper ? keep : recv;   // rows (2h,2h+1) of columns e&1 and (e&1)+2
    const u32 xp = (u32)__builtin_amdgcn_update_dpp(0, (int)x, 0xB1, 0xF, 0xF, false);        // lane ^ 1
    const u32 yp = (u32)__builtin_amdgcn_update_dpp(0, (int)y, 0xB1, 0xF, 0xF, false);
    d0 = __builtin_amdgcn_perm(xp, x, sel);
    d1 = __builtin_amdgcn_perm(yp, y, sel);
}

// FULL: every tile is complete (M % BM == 0, N % columns-per-tile == 0,
// K % 64 == 0), so the main loop has no bounds checks.
// ODD: the number of contraction steps ceil(K / 64) is odd.
template <int MODE, int BM, bool FULL, bool ODD>
__global__ __launch_bounds__(GEMM_THREADS) void gemm_kernel(const GemmArgs p) {
    constexpr int AI = BM / 32;   // A chunks per thread per step
    constexpr int MT = BM / 64;   // 32-row subtiles per wavefront
    constexpr int NCOL = (MODE == MODE_GATEUP) ? 128 : 256;  // output columns per tile
    __shared__ u32x4 sA0[BM * 8], sA1[BM * 8];       // [row][8 chunks], lds_pos swizzle
    __shared__ u32x4 sB0[64 * 32], sB1[64 * 32];     // [contraction row][32 chunks], swizzled
    __shared__ float stat0[BM];                      // inverse norm / inverse std
    __shared__ float stat1[BM];                      // mean (LN)

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

    // ---- A: global-load role: chunk kcA of rows rowA + 32 i
    const int kcA = t & 7, rowA = t >> 3;

    // ---- B: load-to-LDS role.  One instruction of a wavefront fills 1 KiB =
    // two tile rows, lane i -> byte 16 i.  Wavefront w issues row pairs w, w+4,
    // ..., w+28; this lane therefore always serves tile rows = 2 w + lhi (mod 8)
    // and LDS chunk position l32, which holds source chunk l32 ^ 2 (row & 3).
    // Source chunk c of a tile row is columns n0 + 8 c (PLAIN, LN); in GATEUP
    // it is laid out so that each wavefront's four 32-column subtiles are
    // W1[h..h+32), W1[h+32..h+64), W3[h..h+32), W3[h+32..h+64) of the same 64
    // hidden units: a lane's accumulators then hold the gate and the up
    // product of the same hidden unit.
    const int rowB = 2 * w + lhi;
    const int chunkB = l32 ^ ((rowB & 3) << 1);
    const u16* Bsrc = p.B0;
    int colB;
    if (MODE == MODE_GATEUP) {
        const int ttc = (chunkB >> 2) & 3;
        if (ttc >> 1) Bsrc = p.B1;
        colB = n0 + 64 * (chunkB >> 4) + 32 * (ttc & 1) + 8 * (chunkB & 3);
    } else {
        colB = n0 + 8 * chunkB;
    }
    const bool colB_ok = FULL || colB < p.N;
    const u16* const Blane = Bsrc + (size_t)rowB * p.ldb + (colB_ok ? colB : 0);
    const u16* const zsrc = reinterpret_cast<const u16*>(&gemm_zero_chunk);

    // ---- B: fragment-read role.  Group b = lane / 16 of a transposing read
    // covers contraction rows 8 (b / 2) + 4 h + (0..3) (+ 16 per matrix
    // instruction) and columns 32 tt + 16 (b % 2) + (0..15) of the wavefront's
    // 128; lane i' = lane % 16 supplies the address of row i' / 4, 4-column
    // piece i' % 4.  Byte offsets for tt even / odd (the swizzle XORs bit 2 of
    // the chunk index, which is tt's low bit, so odd tt is not a plain offset).
    int offB[2];
    {
        const int b = lane >> 4, ip = lane & 15;
        const int r = 8 * (b >> 1) + (ip >> 2);
        const int piece = ip & 3;
#pragma unroll
        for (int o = 0; o < 2; ++o) {
            const int chunk = 16 * wn + 4 * o + 2 * (b & 1) + (piece >> 1);
            offB[o] = r * 512 + ((chunk ^ ((r & 3) << 1)) << 4) + 8 * (piece & 1);
        }
    }

    // A register sets: tile j travels in set j % 2 (with its gain chunk)
    u32x4 ra[2][AI], rg[2] = {zero4(), zero4()};
    float ssq[AI], ssum[AI];
#pragma unroll
    for (int i = 0; i < AI; ++i) { ssq[i] = 0.f; ssum[i] = 0.f; }
    constexpr int APER = AI / 4;

    // B tile kt -> LDS array dst (8 load-to-LDS instructions per wavefront)
    auto dma_b = [&](int kt, u32x4* dst) {
        const u16* src = Blane + (size_t)kt * GEMM_BK * p.ldb;
        const u32 base = __builtin_amdgcn_readfirstlane(lds_addr(dst) + (u32)w * 1024u);
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const u16* g = src + (size_t)(8 * q) * p.ldb;
            if (!FULL) {
                const int k = kt * GEMM_BK + 8 * q + rowB;
                g = (colB_ok && k < p.K) ? g : zsrc;
            }
            load_to_lds16(g, base + (u32)q * 4096u);
        }
    };
    // A tile kt and its gain chunk -> register set S
    auto gload_a = [&](int kt, auto SETC) {
        constexpr int S = decltype(SETC)::value;
        const int ka = kt * GEMM_BK + 8 * kcA;
        const bool ka_ok = FULL || ka < p.K;
        if (MODE != MODE_PLAIN) rg[S] = ka_ok ? ldg16(p.gain + ka) : zero4();
#pragma unroll
        for (int i = 0; i < AI; ++i) {
            const int m = m0 + rowA + 32 * i;
            ra[S][i] = (FULL || (ka_ok && m < p.M)) ? ldg16(p.A + (size_t)m * p.lda + ka) : zero4();
        }
    };
    // makes the compiler wait here for everything register set S was loaded with
    auto touch = [&](auto SETC) {
        constexpr int S = decltype(SETC)::value;
#pragma unroll
        for (int i = 0; i < AI; ++i) asm volatile("" : "+v"(ra[S][i]));
        u32x4& gref = rg[S];
        if (MODE != MODE_PLAIN) asm volatile("" : "+v"(gref));
    };
    // part `part` (0..3) of writing register set S into LDS array dst: AI/4
    // chunks, scaled by the gain chunk, rounded, row sums updated
    auto sstore_part = [&](u32x4* dst, auto SETC, auto PARTC) {
        constexpr int S = decltype(SETC)::value;
        constexpr int part = decltype(PARTC)::value;
        const u32x4 gv = rg[S];
#pragma unroll
        for (int ii = 0; ii < APER; ++ii) {
            const int i = part * APER + ii;
            u32x4 v = ra[S][i];
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
            dst[lds_pos(rowA + 32 * i, kcA)] = v;
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

    // fragments of contraction slice ks (16 indices) of one LDS buffer pair
    Chunk fa[2][MT], fb[2][4];
    auto frag_load = [&](const u32x4* bufA, const u32x4* bufB, int ks, auto SETC) {
        constexpr int S = decltype(SETC)::value;
        const int kc = 2 * ks + lhi;
#pragma unroll
        for (int s = 0; s < MT; ++s) fa[S][s].u = bufA[lds_pos(wm * (BM / 2) + 32 * s + l32, kc)];
        const char* bb = reinterpret_cast<const char*>(bufB) + ks * (16 * 512);
#pragma unroll
        for (int tt = 0; tt < 4; ++tt) {
            const char* q = bb + offB[tt & 1] + 128 * (tt >> 1);
            const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(q));
            const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(q + 4 * 512));
            u32x2 l2 = *reinterpret_cast<const u32x2*>(&lo), h2 = *reinterpret_cast<const u32x2*>(&hi);
            fb[S][tt].u = u32x4{l2[0], l2[1], h2[0], h2[1]};
        }
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
    constexpr int VALU_PER = (MODE == MODE_PLAIN ? 4 : 4 + 28 * APER) / NMMA + 1;
    auto interleave = [&](bool with_frags) {
        // (the compiler honours data dependences; the pattern below is a placement request)
        if (with_frags) __builtin_amdgcn_sched_group_barrier(0x100, MT + 8, 0);      // LDS reads first
#pragma unroll
        for (int i = 0; i < NMMA; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                       // one matrix instruction
            __builtin_amdgcn_sched_group_barrier(0x002, VALU_PER, 0);                // a slice of the vector ALU work
            if (i % 8 == 7) __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);       // an LDS write
        }
    };

    // One contraction step on buffer pair PAR (tile kt, kt % 2 == PAR): multiply
    // it; meanwhile B tile kt+1 streams into the other pair's B array, A tile
    // kt+1 goes from register set 1-PAR into the other A array, one part per
    // group of 16 matrix instructions, and register set PAR is refilled with
    // tile kl (kt + 2, or the last tile when there is no such tile: a valid
    // address whose data is never stored).  The scheduling directives spread
    // each part's vector ALU and LDS instructions between the matrix
    // instructions (they issue in order, so only instructions placed between
    // two matrix instructions run in the shadow of the first), and fetch the
    // fragments of the next group while the current one is multiplied.
    auto step = [&](int kt, int kl, auto PARC) {
        constexpr int PAR = decltype(PARC)::value;
        using SN = std::integral_constant<int, 1 - PAR>;      // register set of tile kt + 1
        using SL = std::integral_constant<int, PAR>;          // register set being refilled
        u32x4* const curA = PAR ? sA1 : sA0;
        u32x4* const curB = PAR ? sB1 : sB0;
        u32x4* const nxtA = PAR ? sA0 : sA1;
        u32x4* const nxtB = PAR ? sB0 : sB1;
        __syncthreads();
        touch(SN());
        __builtin_amdgcn_sched_barrier(0);
        dma_b(kt + 1, nxtB);
        gload_a(kl, SL());
        __builtin_amdgcn_sched_barrier(0);
        frag_load(curA, curB, 0, C0());
        __builtin_amdgcn_sched_barrier(0);
        frag_load(curA, curB, 1, C1());
        mma(C0());
        sstore_part(nxtA, SN(), C0());
        interleave(true);
        __builtin_amdgcn_sched_barrier(0);
        frag_load(curA, curB, 2, C0());
        mma(C1());
        sstore_part(nxtA, SN(), C1());
        interleave(true);
        __builtin_amdgcn_sched_barrier(0);
        frag_load(curA, curB, 3, C1());
        mma(C0());
        sstore_part(nxtA, SN(), C2());
        interleave(true);
        __builtin_amdgcn_sched_barrier(0);
        mma(C1());
        sstore_part(nxtA, SN(), C3());
        interleave(false);
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    };
    auto last_step = [&](auto PARC) {          // nothing left to store or load
        constexpr int PAR = decltype(PARC)::value;
        const u32x4* const curA = PAR ? sA1 : sA0;
        const u32x4* const curB = PAR ? sB1 : sB0;
        __syncthreads();
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            frag_load(curA, curB, ks, C0());
            mma(C0());
        }
    };

    // prologue: tile 0 into buffer pair 0, A tile 1 in flight in register set 1
    gload_a(0, C0());
    touch(C0());
    __builtin_amdgcn_sched_barrier(0);
    dma_b(0, sB0);
    gload_a(min(1, nk - 1), C1());
    __builtin_amdgcn_sched_barrier(0);
    sstore_part(sA0, C0(), C0());
    sstore_part(sA0, C0(), C1());
    sstore_part(sA0, C0(), C2());
    sstore_part(sA0, C0(), C3());
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));

    // pairs of steps; the tail depends on the parity of nk only
    {
        int kt = 0;
        for (; kt + 2 < nk; kt += 2) {
            step(kt, kt + 2, C0());
            step(kt + 1, min(kt + 3, nk - 1), C1());
        }
        if (ODD) {
            last_step(C0());
        } else {
            step(kt, kt + 1, C0());
            last_step(C1());
        }
    }

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
                    stat0[rowA + 32 * i] = rsqrtf(var + p.eps);
                    stat1[rowA + 32 * i] = mu;
                } else {
                    stat0[rowA + 32 * i] = rsqrtf(s2 * invK + p.eps);
                }
            }
        }
        __syncthreads();
    }

    // ---- epilogue.  Accumulator register v of a 32x32 subtile belongs to
    // subtile row 8 (v / 4) + 4 (lane / 32) + v % 4 and subtile column
    // lane % 32.  Four registers (4 rows x this lane's column) are finished,
    // rounded to bf16 and transposed within the quad, after which quad lane e
    // holds row e, columns 4 (lane % 32 / 4) + (0..3): an 8-byte store per lane,
    // 64 contiguous bytes per row and instruction.
    const int eq = l32 & 3;
    const u32 tsel = (eq & 1) ? 0x03020706u : 0x05040100u;
    const bool tup = (eq & 2) != 0;
    if (MODE == MODE_GATEUP) {
        const int fcol = n0 + 64 * wn + 4 * (l32 >> 2);       // + 32 u
#pragma unroll
        for (int s = 0; s < MT; ++s) {
#pragma unroll
            for (int vg = 0; vg < 4; ++vg) {
                const int rl = wm * (BM / 2) + 32 * s + 8 * vg + 4 * lhi;
                float r[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) r[i] = stat0[rl + i];
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    float h[4];
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        h[i] = swiglu(r[i] * acc[s][u][4 * vg + i], r[i] * acc[s][u + 2][4 * vg + i]);
                    u32 d0 = pack_bf16(h[0], h[1]), d1 = pack_bf16(h[2], h[3]);
                    quad_transpose(d0, d1, tup, tsel);
                    const int m = m0 + rl + eq, col = fcol + 32 * u;
                    if ((FULL || m < p.M) && (FULL || col < p.N)) {
                        u32x2 o = {d0, d1};
                        *reinterpret_cast<u32x2*>(p.C + (size_t)m * p.ldc + col) = o;
                    }
                }
            }
        }
    } else {
        const int ncol = n0 + 128 * wn + l32;                 // + 32 tt: the column this lane accumulated
        const int scol = n0 + 128 * wn + 4 * (l32 >> 2);      // + 32 tt: first of the 4 columns it stores
        float cc[4], cb[4];
        if (MODE == MODE_LN) {
#pragma unroll
            for (int tt = 0; tt < 4; ++tt) {
                const bool ok = FULL || ncol + 32 * tt < p.N;
                cc[tt] = ok ? p.colc[ncol + 32 * tt] : 0.f;
                cb[tt] = ok ? p.colb[ncol + 32 * tt] : 0.f;
            }
        }
#pragma unroll
        for (int s = 0; s < MT; ++s) {
#pragma unroll
            for (int vg = 0; vg < 4; ++vg) {
                const int rl = wm * (BM / 2) + 32 * s + 8 * vg + 4 * lhi;
                float r[4], mu[4];
                if (MODE == MODE_LN) {
#pragma unroll
                    for (int i = 0; i < 4; ++i) { r[i] = stat0[rl + i]; mu[i] = stat1[rl + i]; }
                }
#pragma unroll
                for (int tt = 0; tt < 4; ++tt) {
                    float y[4];
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        y[i] = acc[s][tt][4 * vg + i];
                        if (MODE == MODE_LN) y[i] = fmaf(r[i], y[i] - mu[i] * cc[tt], cb[tt]);
                    }
                    u32 d0 = pack_bf16(y[0], y[1]), d1 = pack_bf16(y[2], y[3]);
                    quad_transpose(d0, d1, tup, tsel);
                    const int m = m0 + rl + eq, col = scol + 32 * tt;
                    if ((FULL || m < p.M) && (FULL || col < p.N)) {
                        u32x2 o = {d0, d1};
                        *reinterpret_cast<u32x2*>(p.C + (size_t)m * p.ldc + col) = o;
                    }
                }
            }
        }
    }
}

}  // namespace bb
