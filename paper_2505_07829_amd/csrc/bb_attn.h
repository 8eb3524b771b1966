// Attention forward for gfx950: O = softmax(Q K^T / sqrt(d)) V  (Example 1).
//
// This is the loop nest the fusion algorithm ends with for Example 1 (its last
// step, with the feature and value dimensions unsplit, D = L = 1, the setting
// the epilogue names as the original Flash Attention): per block of queries
// one serial loop over key blocks that accumulates the dot with the value
// block and the row sums of the exponentiated scores, and a division by the
// row sums at the end.  Numerical safety is added the way the paper's Appendix
// describes, in its row-wise form: the exponentiated score block of a step is
// a pair (significands, one exponent per query row), accumulators carry a
// running exponent per row and are brought to the larger exponent before a
// block is added.
//
// Layouts: Q [B, M, DK], K [B, N, DK], V [B, N, DV], O [B, M, DV], bf16,
// row-major, B independent problems (heads).
//
// Tiling: one workgroup (4 wavefronts) per 128 queries of one problem, 32
// queries per wavefront; key blocks of 64.  Scores are computed TRANSPOSED,
// S^T = K Q^T, with 32x32x16 matrix instructions: a lane then holds one query
// (column) and 16 of every 32 keys (rows), so the row-wise maximum and sum of
// the softmax are in-lane reductions plus one exchange with lane ^ 32.  The
// second product is computed transposed too, O^T = V^T P^T: the probabilities
// leave the first product already in the register layout the second one wants
// as its B operand (8 consecutive accumulator registers = 8 contraction slots;
// the contraction order is free as long as both operands agree), and V^T comes
// out of LDS with the transposing read, like the weight tiles of the GEMM.
//   Q fragments stay in registers for the whole kernel (loaded from global
// memory in operand layout).  K and V blocks go global -> LDS with load-to-LDS
// instructions, double buffered, one barrier per key block.  The loop is a
// software pipeline: the matrix instructions of block t + 1's scores run
// between the vector instructions that exponentiate block t's scores, and
// those of block t's output product between the maximum of block t + 1.
#pragma once
#include <type_traits>

#include "bb_gemm.h"

namespace bb {

struct AttnArgs {
    const u16* Q;
    const u16* K;
    const u16* V;
    u16* O;
    int B, M, N;
    int tiles_q;        // ceil(M / (32 NW))
    int wgs_per_xcd;    // ceil(B * tiles_q / 8)
    float c;            // log2(e) / sqrt(DK)
    // split keys (KSPLIT kernels): nsplit workgroups per (problem, query block), each over
    // nt_split key blocks; unnormalised outputs and (exponent, row sum) pairs go to part / ml
    int nsplit, nt_split;
    float* part;        // [B M][nsplit][DV]
    float* ml;          // [B M][nsplit][2]
    // attention_decode_kernel: arrival counters, one per problem, zero between launches (the last
    // workgroup of a problem to arrive adds the problem's partial results)
    unsigned* cnt;
};

// a workgroup has NW = 4 or 8 wavefronts of 32 queries each
constexpr int ATTN_BK = 64;       // keys per step
constexpr float ATTN_SLACK = 8.f; // log2 of the largest significand a row keeps before its exponent moves

// chunk position of (row, chunk) in an LDS tile with CPR 16-byte chunks per row,
// for reads that take 16 consecutive rows at one chunk index (128-bit fragment
// reads): 16 different 16-byte slots of the 256-byte bank line
template <int CPR>
__device__ __forceinline__ int attn_pos_rows16(int row, int kc) {
    return CPR == 16 ? row * 16 + (kc ^ (row & 15)) : row * 8 + (kc ^ ((row >> 1) & 7));
}
// swizzle of the chunk index for transposing reads (4 consecutive rows x 64
// bytes per pass): the four rows must take the four 64-byte quarters of a bank line
template <int CPR>
__device__ __forceinline__ int attn_swz_tr(int row) {
    return CPR == 16 ? ((row & 3) << 2) : (((row >> 1) & 1) << 2);
}

// Adds the nsplit partial results of a query row.  Every partial result is a
// pair (significands O_s and l_s, row exponent m_s); two pairs are added by
// bringing both to the larger exponent (Appendix), and the quotient of the
// totals is rounded to bf16.  One wavefront per row: lane = (group of 8 output
// columns, phase); a phase adds every (64 / groups)-th partial result, then the
// phases are added across lanes.  The partial results are read with agent-scope
// loads: they may have been written by other workgroups of the same launch.
template <int DV>
__device__ __forceinline__ void attention_combine_row(const float* part, const float* ml, u16* O, size_t row,
                                                      int nsplit, float c, int lane) {
    constexpr int G = DV / 8, NPH = 64 / G;
    const int cg = lane % G, ph = lane / G;
    float z = -INFINITY, l = 0.f;
    f32x4 a0 = {0, 0, 0, 0}, a1 = a0;
    // (z, l, a) += (z2, l2, b): both to the larger exponent; equal exponents (also -inf = -inf) need no scaling
    auto add = [&](float z2, float l2, const f32x4& b0, const f32x4& b1) {
        const float zn = fmaxf(z, z2);
        const float w1 = (z == zn) ? 1.f : __builtin_amdgcn_exp2f((z - zn) * c);
        const float w2 = (z2 == zn) ? 1.f : __builtin_amdgcn_exp2f((z2 - zn) * c);
        l = l * w1 + l2 * w2;
        a0 = a0 * w1 + b0 * w2;
        a1 = a1 * w1 + b1 * w2;
        z = zn;
    };
    constexpr int NB = 4;                                  // partial results whose loads are in flight together
    for (int sp0 = ph; sp0 < nsplit; sp0 += NB * NPH) {
        u32x2 e[NB];
        f32x4 b0[NB], b1[NB];
#pragma unroll
        for (int u = 0; u < NB; ++u) {
            const int sp = min(sp0 + u * NPH, nsplit - 1);     // (past the end: loaded again, not added)
            const size_t slot = row * nsplit + sp;
            const float* src = part + slot * DV + 8 * cg;
            e[u] = cload8(ml + 2 * slot);
            b0[u] = cload16f(src);
            b1[u] = cload16f(src + 4);
        }
#pragma unroll
        for (int u = 0; u < NB; ++u)
            if (sp0 + u * NPH < nsplit) add(__uint_as_float(e[u][0]), __uint_as_float(e[u][1]), b0[u], b1[u]);
    }
#pragma unroll
    for (int off = G; off < 64; off <<= 1) {
        f32x4 b0, b1;
#pragma unroll
        for (int i = 0; i < 4; ++i) { b0[i] = __shfl_xor(a0[i], off); b1[i] = __shfl_xor(a1[i], off); }
        add(__shfl_xor(z, off), __shfl_xor(l, off), b0, b1);
    }
    if (ph == 0) {
        const float inv = 1.0f / l;
        const u32x4 o = {pack_bf16(a0[0] * inv, a0[1] * inv), pack_bf16(a0[2] * inv, a0[3] * inv),
                         pack_bf16(a1[0] * inv, a1[1] * inv), pack_bf16(a1[2] * inv, a1[3] * inv)};
        *reinterpret_cast<u32x4*>(O + row * DV + 8 * cg) = o;
    }
}

// TAIL: iterations left after the main loop (1 .. 4; the loop takes two
// complete iterations per trip while at least five key blocks remain).  A
// template parameter, so that no branch merges the accumulators and only the
// unrolled tail loads and masks the last key block.
// NW: wavefronts per workgroup (4 or 8).  Eight share every K and V block among
// twice as many queries: half the load-to-LDS instructions per wavefront and
// half the L2 traffic, one workgroup per compute unit instead of two.
// KSPLIT (few queries, e.g. decoding): the serial loop over the key blocks is
// cut into nsplit equal ranges that run in parallel workgroups (Rule 3's
// parallel form); each stores its accumulators as significand-exponent pairs
// (output sums and row sum at its own row exponents) and
// attention_combine_kernel adds them the Appendix's way.
template <int DK, int DV, int TAIL, int NW, bool KSPLIT = false>
__global__ __launch_bounds__(64 * NW, 2) void attention_kernel(const AttnArgs p) {
    constexpr int ATTN_BQ = 32 * NW;
    constexpr int CK = DK / 8, CV = DV / 8;          // 16-byte chunks per K / V row
    constexpr int NKS = DK / 16;                     // contraction slices of the first product
    constexpr int NDS = DV / 32;                     // 32-row subtiles of O^T
    static_assert((DK == 64 || DK == 128) && (DV == 64 || DV == 128), "head dimensions 64 or 128");
    __shared__ u32x4 sK0[ATTN_BK * CK], sK1[ATTN_BK * CK];
    __shared__ u32x4 sV0[ATTN_BK * CV], sV1[ATTN_BK * CV];

    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int l32 = lane & 31, g = lane >> 5;
    // workgroup id -> XCD (id % 8) -> a contiguous range of (problem, query
    // block) pairs per XCD: the workgroups resident on one XCD then work on
    // the same one or two problems and share their K and V blocks in its L2
    const int lin0 = (blockIdx.x & 7) * p.wgs_per_xcd + (blockIdx.x >> 3);
    if (lin0 >= p.B * p.tiles_q * (KSPLIT ? p.nsplit : 1)) return;
    const int split = KSPLIT ? lin0 % p.nsplit : 0, lin = KSPLIT ? lin0 / p.nsplit : lin0;
    const int b = lin / p.tiles_q, qt = lin % p.tiles_q;
    const int q = qt * ATTN_BQ + 32 * w + l32;          // this lane's query
    const int key_first = KSPLIT ? split * p.nt_split * ATTN_BK : 0;       // first key of this workgroup
    const int nkeys = p.N - key_first;                                    // keys from there to the end of the sequence
    const u16* const Kb = p.K + ((size_t)b * p.N + key_first) * DK;
    const u16* const Vb = p.V + ((size_t)b * p.N + key_first) * DV;

    // Q fragments: B operand of S^T = K Q^T: column = query, 8 consecutive features
    Chunk qf[NKS];
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks)
        qf[ks].u = (q < p.M) ? ldg16(p.Q + ((size_t)b * p.M + q) * DK + 16 * ks + 8 * g) : zero4();

    // load-to-LDS roles: an instruction fills 64 chunks = 64 / CPR rows of a
    // tile; instruction j of this wavefront fills LDS chunks (NI w + j) 64 ...
    // Lane offsets inside a complete block are loop constants; the block's base
    // advances as a uniform pointer.  In the last block rows past the end of
    // the sequence load the last valid row instead (their scores are masked,
    // their probabilities exactly zero).
    constexpr int RPK = 64 / CK, NIK = ATTN_BK / RPK / NW;    // rows per instruction, instructions per wavefront
    constexpr int RPV = 64 / CV, NIV = ATTN_BK / RPV / NW;
    static_assert(NIK >= 1 && NIV >= 1, "every wavefront loads part of each block");
    constexpr int NDMA = NIK + NIV;
    int rowKd[NIK], rowVd[NIV];
    u32 offKd[NIK], offVd[NIV];
#pragma unroll
    for (int j = 0; j < NIK; ++j) {
        const int row = RPK * (NIK * w + j) + lane / CK, pos = lane % CK;
        const int chunk = CK == 16 ? (pos ^ (row & 15)) : (pos ^ ((row >> 1) & 7));
        rowKd[j] = row;
        offKd[j] = (u32)(row * DK + 8 * chunk);
    }
#pragma unroll
    for (int j = 0; j < NIV; ++j) {
        const int row = RPV * (NIV * w + j) + lane / CV, pos = lane % CV;
        const int chunk = pos ^ attn_swz_tr<CV>(row);
        rowVd[j] = row;
        offVd[j] = (u32)(row * DV + 8 * chunk);
    }
    // which: 0 nothing, 1 a complete block, 2 the last block
    auto dma_k = [&](int kt, u32x4* dK, auto WHICH) {
        constexpr int W = decltype(WHICH)::value;
        if (W == 0) return;
        const int key0 = kt * ATTN_BK;
        const int rmax = nkeys - 1 - key0;                // last valid row of the block
#pragma unroll
        for (int j = 0; j < NIK; ++j) {
            const u32 off = W == 2 ? offKd[j] - (u32)(max(rowKd[j] - rmax, 0) * DK) : offKd[j];
            (KSPLIT ? load_to_lds16_nt : load_to_lds16)(reinterpret_cast<const char*>(Kb) + (u32)(2 * (off + (u32)(key0 * DK))), dK + (NIK * w + j) * 64);
        }
    };
    auto dma_v = [&](int kt, u32x4* dV, auto WHICH) {
        constexpr int W = decltype(WHICH)::value;
        if (W == 0) return;
        const int key0 = kt * ATTN_BK;
        const int rmax = nkeys - 1 - key0;
#pragma unroll
        for (int j = 0; j < NIV; ++j) {
            const u32 off = W == 2 ? offVd[j] - (u32)(max(rowVd[j] - rmax, 0) * DV) : offVd[j];
            (KSPLIT ? load_to_lds16_nt : load_to_lds16)(reinterpret_cast<const char*>(Vb) + (u32)(2 * (off + (u32)(key0 * DV))), dV + (NIV * w + j) * 64);
        }
    };

    // transposing-read role for V^T fragments: group blk = lane / 16 covers key
    // rows 4 (blk / 2) + (0..3) (+ 8 for the second read) and value columns
    // 16 (blk % 2) + (0..15) of a 32-column subtile; lane i' = lane % 16 supplies
    // the address of row i' / 4, 4-column piece i' % 4.
    const int blk = lane >> 4, ip = lane & 15;
    const int trow = 4 * (blk >> 1) + (ip >> 2);                 // + 32 st + 16 kk (+ 8)
    const int tchunk = 2 * (blk & 1) + ((ip & 3) >> 1);          // + 4 dsub
    const int tbyte = 8 * (ip & 1);

    f32x16 oacc[NDS];
#pragma unroll
    for (int ds = 0; ds < NDS; ++ds)
#pragma unroll
        for (int v = 0; v < 16; ++v) oacc[ds][v] = 0.f;
    float m_run = -INFINITY;      // running exponent of this query's row (in score units)
    float l_run = 0.f;            // this lane's share of the row sum, at exponent m_run

    const int nt = KSPLIT ? p.nt_split : (p.N + ATTN_BK - 1) / ATTN_BK;

    // byte offsets of this lane's fragment reads inside a K / V buffer (the XOR
    // swizzles do not depend on the 32-key subtile or the 16-key slice, which
    // are plain displacements)
    int offK[NKS], offV[NDS];
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) offK[ks] = attn_pos_rows16<CK>(l32, 2 * ks + g) * 16;
#pragma unroll
    for (int ds = 0; ds < NDS; ++ds)
        offV[ds] = trow * (CV * 16) + (((4 * ds + tchunk) ^ attn_swz_tr<CV>(trow)) << 4) + tbyte;

    using I0 = std::integral_constant<int, 0>;
    using I1 = std::integral_constant<int, 1>;
    using I2 = std::integral_constant<int, 2>;
    constexpr int NS = 2 * NKS, NPV = 4 * NDS;        // matrix instructions of the two products
    constexpr int PDK = 2, PDV = 2;                   // fragment reads run this many matrix instructions ahead

    f32x16 sc[2][2];                                  // scores of the blocks of even / odd index, two 32-key subtiles each
    float mloc = -INFINITY;                           // maximum of the block whose scores were computed last
    Chunk pb[2][2];                                   // exponentiated scores of a block as matrix operands
    Chunk vf[NPV];

    auto kread = [&](const char* kb, int i) -> u32x4 {
        return *reinterpret_cast<const u32x4*>(kb + offK[i % NKS] + (i / NKS) * (32 * CK * 16));
    };
    auto vread = [&](const char* vb, int i) {          // fragment of matrix instruction i = (st, kk, ds)
        const char* a0 = vb + offV[i % NDS] + (16 * (i / NDS)) * (CV * 16);
        const char* a1 = a0 + 8 * (CV * 16);
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(a0));
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(a1));
        const u32x2 l2 = *reinterpret_cast<const u32x2*>(&lo), h2 = *reinterpret_cast<const u32x2*>(&hi);
        vf[i].u = u32x4{l2[0], l2[1], h2[0], h2[1]};
    };
    // scores of one block: S^T = K Q^T into sc[PAR]
    auto scores = [&](const char* kb, auto PARC) {
        constexpr int PAR = decltype(PARC)::value;
        Chunk kf[NS];
#pragma unroll
        for (int i = 0; i < NS; ++i) kf[i].u = kread(kb, i);
#pragma unroll
        for (int st = 0; st < 2; ++st) {
#pragma unroll
            for (int v = 0; v < 16; ++v) sc[PAR][st][v] = 0.f;
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks)
                sc[PAR][st] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[st * NKS + ks].v, qf[ks].v, sc[PAR][st], 0, 0, 0);
        }
    };
    // keys past the end of the sequence do not take part
    auto mask = [&](int kt, auto PARC) {
        constexpr int PAR = decltype(PARC)::value;
#pragma unroll
        for (int st = 0; st < 2; ++st)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int key = kt * ATTN_BK + 32 * st + 8 * (v >> 2) + 4 * g + (v & 3);
                if (key >= nkeys) sc[PAR][st][v] = -INFINITY;
            }
    };
    auto block_max = [&](auto PARC) {
        constexpr int PAR = decltype(PARC)::value;
        float m = -INFINITY;
#pragma unroll
        for (int st = 0; st < 2; ++st)
#pragma unroll
            for (int v = 0; v < 16; ++v) m = fmaxf(m, sc[PAR][st][v]);
        mloc = fmaxf(m, __shfl_xor(m, 32));
    };
    // The row exponent moves only when the block maximum exceeds it by more
    // than ATTN_SLACK binary orders of magnitude (significands then stay below
    // 2^ATTN_SLACK, far inside fp32 and bf16 range); a wavefront none of whose
    // rows moves skips the rescaling of its accumulators.
    auto decide = [&]() {
        const bool moves = mloc * p.c > m_run * p.c + ATTN_SLACK;
        const float m_new = moves ? mloc : m_run;
        if (__builtin_amdgcn_ballot_w64(moves) != 0) {
            const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * p.c);   // 1 where the row stays
            l_run *= alpha;
#pragma unroll
            for (int ds = 0; ds < NDS; ++ds)
#pragma unroll
                for (int v = 0; v < 16; ++v) oacc[ds][v] *= alpha;
        }
        m_run = m_new;
    };
    // exponentiate the scores of a block as (significands, row exponent m_run)
    auto exponentiate = [&](auto PARC) {
        constexpr int PAR = decltype(PARC)::value;
        const float mc = m_run * p.c;
        float lsum = 0.f;
#pragma unroll
        for (int st = 0; st < 2; ++st)
#pragma unroll
            for (int kk = 0; kk < 2; ++kk)
#pragma unroll
                for (int h = 0; h < 4; ++h) {
                    const float p0 = __builtin_amdgcn_exp2f(fmaf(sc[PAR][st][8 * kk + 2 * h], p.c, -mc));
                    const float p1 = __builtin_amdgcn_exp2f(fmaf(sc[PAR][st][8 * kk + 2 * h + 1], p.c, -mc));
                    lsum += p0 + p1;
                    pb[st][kk].u[h] = pack_bf16(p0, p1);
                }
        l_run += lsum;
    };
    auto output_mfma = [&]() {
#pragma unroll
        for (int i = 0; i < NPV; ++i)
            oacc[i % NDS] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[i].v, pb[i / (2 * NDS)][(i / NDS) & 1].v,
                                                                    oacc[i % NDS], 0, 0, 0);
    };
    auto sync = [&]() {
        __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
        __syncthreads();
    };

    // One iteration t of the software pipeline (PAR = t % 2).  After the
    // barrier (K block t + 1 and V block t have landed; everyone is done with
    // K block t and V block t - 1, whose buffers the new loads overwrite):
    //   region X: the matrix instructions of the NEXT block's scores,
    //             S(t + 1) = K(t + 1) Q^T, interleaved with the exponentiation
    //             of THIS block's scores (vector arithmetic) and with the
    //             load-to-LDS instructions of K(t + 2) and V(t + 1);
    //   region Y: the matrix instructions of O += P(t) V(t), interleaved with
    //             the maximum of S(t + 1);
    //   then the row exponents take S(t + 1) into account (rarely: rescaling).
    // NEXT: block t + 1 exists; MASKN: it is the last one (keys past the end);
    // KW / VW: what to load (0 nothing, 1 complete block, 2 last block).
    auto iteration = [&](int t, auto PARC, auto NEXTC, auto MASKNC, auto KWC, auto VWC) {
        constexpr int PAR = decltype(PARC)::value;
        constexpr bool NEXT = decltype(NEXTC)::value != 0, MASKN = decltype(MASKNC)::value != 0;
        constexpr int KW = decltype(KWC)::value, VW = decltype(VWC)::value;
        constexpr int ND = (KW ? NIK : 0) + (VW ? NIV : 0);
        using PARN = std::integral_constant<int, PAR ^ 1>;
        const char* const kb = reinterpret_cast<const char*>(PAR ? sK0 : sK1);     // K(t + 1)
        const char* const vb = reinterpret_cast<const char*>(PAR ? sV1 : sV0);     // V(t)
        sync();
        dma_k(t + 2, PAR ? sK1 : sK0, KWC);
        dma_v(t + 1, PAR ? sV0 : sV1, VWC);
        // ---- region X
        if (NEXT) scores(kb, PARN{});
        exponentiate(PARC);
#pragma unroll
        for (int i = 0; i < PDV; ++i) vread(vb, i);
        {
            // 7 vector instructions per matrix instruction: 32 x (fma, exp, add) + 16 conversions
            if (NEXT) __builtin_amdgcn_sched_group_barrier(0x100, PDK, 0);
#pragma unroll
            for (int i = 0; i < NS; ++i) {
                if (NEXT) __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                if (NEXT && i + PDK < NS) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                if ((i * ND) / NS != ((i + 1) * ND) / NS) __builtin_amdgcn_sched_group_barrier(0x010, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x002, 112 / NS, 0);
            }
            __builtin_amdgcn_sched_group_barrier(0x100, 2 * PDV, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
        if (MASKN) mask(t + 1, PARN{});
        // ---- region Y
#pragma unroll
        for (int i = PDV; i < NPV; ++i) vread(vb, i);
        output_mfma();
        if (NEXT) block_max(PARN{});
#pragma unroll
        for (int i = 0; i < NPV; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            if (i + PDV < NPV) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
            if (NEXT) __builtin_amdgcn_sched_group_barrier(0x002, (16 + NPV - 1) / NPV, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
        if (NEXT) decide();
    };

    // ---- prologue: K(0), V(0), K(1); scores, maximum and exponents of block 0
    dma_k(0, sK0, std::integral_constant<int, (TAIL == 1 ? 2 : 1)>{});
    dma_v(0, sV0, std::integral_constant<int, (TAIL == 1 ? 2 : 1)>{});
    dma_k(1, sK1, std::integral_constant<int, (TAIL == 1 ? 0 : (TAIL == 2 ? 2 : 1))>{});
    sync();
    scores(reinterpret_cast<const char*>(sK0), I0{});
    if (TAIL == 1) mask(0, I0{});
    block_max(I0{});
    decide();

    // ---- main loop: complete iterations (blocks t + 1 and t + 2 exist and are
    // not the last one), two per trip so that buffers and score registers are
    // named statically; the last one to four iterations follow unrolled.
    int t = 0;
    for (; t + 5 <= nt; t += 2) {
        iteration(t, I0{}, I1{}, I0{}, I1{}, I1{});
        iteration(t + 1, I1{}, I1{}, I0{}, I1{}, I1{});
    }
    if (TAIL == 1) {
        iteration(t, I0{}, I0{}, I0{}, I0{}, I0{});
    } else if (TAIL == 2) {
        iteration(t, I0{}, I1{}, I1{}, I0{}, I2{});
        iteration(t + 1, I1{}, I0{}, I0{}, I0{}, I0{});
    } else if (TAIL == 3) {
        iteration(t, I0{}, I1{}, I0{}, I2{}, I1{});
        iteration(t + 1, I1{}, I1{}, I1{}, I0{}, I2{});
        iteration(t + 2, I0{}, I0{}, I0{}, I0{}, I0{});
    } else {
        iteration(t, I0{}, I1{}, I0{}, I1{}, I1{});
        iteration(t + 1, I1{}, I1{}, I0{}, I2{}, I1{});
        iteration(t + 2, I0{}, I1{}, I1{}, I0{}, I2{});
        iteration(t + 3, I1{}, I0{}, I0{}, I0{}, I0{});
    }

    // ---- divide by the row sums and store: register v of subtile ds is value
    // column 32 ds + 8 (v / 4) + 4 g + v % 4 of this lane's query
    const float l = l_run + __shfl_xor(l_run, 32);
    if (KSPLIT) {
        if (q < p.M) {
            const size_t slot = ((size_t)b * p.M + q) * p.nsplit + split;
            float* const orow = p.part + slot * DV;
#pragma unroll
            for (int ds = 0; ds < NDS; ++ds)
#pragma unroll
                for (int vg = 0; vg < 4; ++vg)
                    cstore16f(orow + 32 * ds + 8 * vg + 4 * g,
                              f32x4{oacc[ds][4 * vg], oacc[ds][4 * vg + 1], oacc[ds][4 * vg + 2], oacc[ds][4 * vg + 3]});
            if (g == 0) cstore8(p.ml + 2 * slot, __float_as_uint(m_run), __float_as_uint(l));
        }
        return;
    }
    const float inv = 1.0f / l;
    if (q < p.M) {
        u16* const orow = p.O + ((size_t)b * p.M + q) * DV;
#pragma unroll
        for (int ds = 0; ds < NDS; ++ds)
#pragma unroll
            for (int vg = 0; vg < 4; ++vg) {
                const u32x2 o = {pack_bf16(oacc[ds][4 * vg] * inv, oacc[ds][4 * vg + 1] * inv),
                                 pack_bf16(oacc[ds][4 * vg + 2] * inv, oacc[ds][4 * vg + 3] * inv)};
                *reinterpret_cast<u32x2*>(orow + 32 * ds + 8 * vg + 4 * g) = o;
            }
    }
}

// One query per problem (decoding): no matrix product is left, the work is reading K and V once.
// A workgroup of four wavefronts takes 4 nt_split blocks of 64 keys of one problem, wavefront w the
// blocks 4 j + w.  A block's K and V rows are requested together (a lane holds 8 features of a
// row, DK / 8 lanes a row), the scores are fp32 dot products reduced over the lanes of a row, the
// softmax runs online per wavefront with the row exponent in score units (Example 1's running
// maximum and sum; the probabilities stay fp32 here), and the value sums of the lanes' keys are
// added over the lane groups at the end.  The four wavefronts' significand-exponent pairs are
// added in LDS (Appendix), the workgroup's pair goes to slot `split` of part / ml, and the last
// workgroup of the problem to arrive adds the slots (attention_combine_row).  nsplit may be 1.
template <int DK, int DV>
__global__ __launch_bounds__(256) void attention_decode_kernel(const AttnArgs p) {
    constexpr int LK = DK / 8, RK = 64 / LK, NLK = 64 / RK;   // lanes per K row, rows per load instruction, instructions per block
    constexpr int LV = DV / 8, RV = 64 / LV, NLV = 64 / RV;
    __shared__ float s_p[4][64];
    __shared__ float s_o[4][DV];
    __shared__ float s_ml[4][2];
    __shared__ unsigned last_arrival;
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int b = blockIdx.x / p.nsplit, split = blockIdx.x % p.nsplit;
    const u16* const Kb = p.K + (size_t)b * p.N * DK;
    const u16* const Vb = p.V + (size_t)b * p.N * DV;
    const int kl = lane % LK, kr0 = lane / LK;      // this lane's features 8 kl .. 8 kl + 7 of key row kr0 (+ RK i)
    const int vl = lane % LV, vr0 = lane / LV;

    float qf[8];
    {
        const u32x4 qc = ldg16(p.Q + (size_t)b * DK + 8 * kl);
#pragma unroll
        for (int e = 0; e < 4; ++e) { qf[2 * e] = bf_lo(qc[e]); qf[2 * e + 1] = bf_hi(qc[e]); }
    }
    float m_run = -INFINITY, l_run = 0.f;           // l_run: this lane's keys only
    float acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.f;

    for (int j = 0; j < p.nt_split; ++j) {
        const int key0 = ((split * p.nt_split + j) * 4 + w) * ATTN_BK;
        if (key0 >= p.N) break;                      // (the same for the whole wavefront)
        u32x4 kreg[NLK], vreg[NLV];
#pragma unroll
        for (int i = 0; i < NLK; ++i) {
            const int row = min(key0 + RK * i + kr0, p.N - 1);
            kreg[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(Kb + (size_t)row * DK + 8 * kl));
        }
#pragma unroll
        for (int i = 0; i < NLV; ++i) {
            const int row = min(key0 + RV * i + vr0, p.N - 1);
            vreg[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(Vb + (size_t)row * DV + 8 * vl));
        }
        // scores of keys key0 + RK i + kr0 (all lanes of a row hold the row's score); past the end: -inf
        float sc[NLK];
        float mx = -INFINITY;
#pragma unroll
        for (int i = 0; i < NLK; ++i) {
            float d = 0.f;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                d = fmaf(qf[2 * e], bf_lo(kreg[i][e]), d);
                d = fmaf(qf[2 * e + 1], bf_hi(kreg[i][e]), d);
            }
#pragma unroll
            for (int off = 1; off < LK; off <<= 1) d += __shfl_xor(d, off);
            sc[i] = (key0 + RK * i + kr0 < p.N) ? d : -INFINITY;
            mx = fmaxf(mx, sc[i]);
        }
#pragma unroll
        for (int off = LK; off < 64; off <<= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
        const float m_new = fmaxf(m_run, mx);        // finite: key0 < N
        const float scale = __builtin_amdgcn_exp2f((m_run - m_new) * p.c);     // 0 at the first block
        m_run = m_new;
        l_run *= scale;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] *= scale;
        // probabilities through LDS from the K layout (key RK i + kr0) to the V layout (key RV i + vr0)
#pragma unroll
        for (int i = 0; i < NLK; ++i)
            if (kl == 0) s_p[w][RK * i + kr0] = __builtin_amdgcn_exp2f((sc[i] - m_new) * p.c);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
        for (int i = 0; i < NLV; ++i) {
            const float pr = s_p[w][RV * i + vr0];
            l_run += pr;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                acc[2 * e] = fmaf(pr, bf_lo(vreg[i][e]), acc[2 * e]);
                acc[2 * e + 1] = fmaf(pr, bf_hi(vreg[i][e]), acc[2 * e + 1]);
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();             // s_p[w] is rewritten by the next block
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
    // add over the lane groups (keys); group 0 then holds the wavefront's sums for value columns 8 vl .. 8 vl + 7
#pragma unroll
    for (int off = LV; off < 64; off <<= 1) {
        l_run += __shfl_xor(l_run, off);
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] += __shfl_xor(acc[e], off);
    }
    if (vr0 == 0) {
#pragma unroll
        for (int e = 0; e < 8; ++e) s_o[w][8 * vl + e] = acc[e];
    }
    if (lane == 0) { s_ml[w][0] = m_run; s_ml[w][1] = l_run; }
    __syncthreads();
    // the four wavefronts' pairs -> the workgroup's pair (wavefront 0 always has a key: its exponent is finite)
    const size_t slot = (size_t)b * p.nsplit + split;
    {
        float mw[4], ww[4];
        float mm = -INFINITY;
#pragma unroll
        for (int u = 0; u < 4; ++u) { mw[u] = s_ml[u][0]; mm = fmaxf(mm, mw[u]); }
#pragma unroll
        for (int u = 0; u < 4; ++u) ww[u] = (mw[u] == mm) ? 1.f : __builtin_amdgcn_exp2f((mw[u] - mm) * p.c);
        const int t = threadIdx.x;
        if (t < DV) {
            float o = 0.f;
#pragma unroll
            for (int u = 0; u < 4; ++u) o = fmaf(s_o[u][t], ww[u], o);
            __hip_atomic_store(p.part + slot * DV + t, o, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        if (t == 0) {
            float l = 0.f;
#pragma unroll
            for (int u = 0; u < 4; ++u) l = fmaf(s_ml[u][1], ww[u], l);
            cstore8(p.ml + 2 * slot, __float_as_uint(mm), __float_as_uint(l));
        }
    }
    // count the delivery; the last workgroup of the problem adds the slots (in slot order) and
    // puts the counter back to zero
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    if (threadIdx.x == 0) {
        const unsigned old = __hip_atomic_fetch_add(p.cnt + b, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        last_arrival = (old + 1u == (unsigned)p.nsplit) ? 1u : 0u;
    }
    __syncthreads();
    if (last_arrival == 0u || w != 0) return;
    attention_combine_row<DV>(p.part, p.ml, p.O, (size_t)b, p.nsplit, p.c, lane);
    if (lane == 0) __hip_atomic_store(p.cnt + b, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// One wavefront per query row (the launch that follows attention_kernel<..., KSPLIT>).
template <int DV>
__global__ __launch_bounds__(64) void attention_combine_kernel(const float* part, const float* ml, u16* O,
                                                                int nsplit, float c) {
    attention_combine_row<DV>(part, ml, O, blockIdx.x, nsplit, c, threadIdx.x);
}

}  // namespace bb
