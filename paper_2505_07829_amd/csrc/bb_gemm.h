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
//  MODE_GATEUP_PRE  the two products, Swish and Hadamard product of MODE_GATEUP
//               on an A operand that already carries the gain (bf16(x g),
//               written by a row kernel together with the inverse norms):
//               the statistics loop is a loop of its own before the K-map,
//               as in Example 3's first snapshot, and the main loop is the
//               plain one.
//  MODE_LN_PRE  MODE_LN's product and epilogue on an A operand that already
//               carries gamma (bf16(x gamma)), with means and inverse standard
//               deviations from the row kernel that wrote it (Example 2's
//               first snapshot: statistics loop, then the N-map).
//
// Layouts: A [M,K] row-major, B [K,N] row-major (contraction index strided),
// C [M,N] row-major, all bf16.  fp32 accumulation in 32x32x16 matrix
// instructions.
//
// Tiling: 4 or 8 wavefronts, workgroup tile BM x 256 columns (GATEUP:
// 128 hidden units = 128 columns of W1 + the same 128 of W3), contraction step
// 64, LDS double buffered with one barrier per step.  PLAIN, GATEUP_PRE and LN_PRE
// arrange the wavefronts 2x2 or 2x4 (least LDS read traffic; in GATEUP_PRE a
// wavefront takes columns of W1 and the same ones of W3); GATEUP and LN
// arrange them 4x1 or 8x1, so that every wavefront owns its rows of A alone (see
// "A operand").
//
// Both operand tiles go from global memory straight into LDS with load-to-LDS
// instructions: no staging registers, no vector ALU work, no LDS writes.
//
// B operand.  The weight tile (64 contraction rows x 512 bytes) lies in LDS
// row-major as in memory.  The matrix instruction wants, per lane, 8
// consecutive contraction indices of one column; the transposing LDS read
// (ds_read_b64_tr_b16) delivers exactly that from a row-major tile, 4
// contraction rows x 16 columns per group of 16 lanes.  The 16-byte chunks of
// a row are XOR-swizzled with the low two row bits (in units of 64 bytes) so
// that the rows read together fall on different banks.
//
// A operand.  The activation tile lies in LDS as rows of 8 chunks (16 bytes = 8
// contraction indices), chunk index XOR-swizzled with row bits 1..3; one
// 128-bit LDS read is one matrix-instruction operand.  The norm prologue works
// on these operand registers: a fragment is read one group of matrix
// instructions ahead, its squares (LN: and its values) are added to the
// lane's row sums, and it is scaled by the gain (read from a small LDS copy of
// the gain tile) and rounded to bf16 before it enters the matrix instruction.
// With 4x1 wavefronts no fragment is read by two wavefronts, so this costs
// each element one pass through the vector ALU, in the shadow of the matrix
// instructions.
//
// Waiting.  Nothing in the main loop loads into registers from global memory,
// so the only vector-memory waits are the explicit one at the end of a step
// (all load-to-LDS of the next tiles have landed) followed by the barrier.
// Every LDS buffer is its own __shared__ array and the main loop is unrolled
// by two: the compiler tracks outstanding load-to-LDS per array and would
// otherwise make the LDS reads of one buffer wait for the transfer into the
// other.  The parity of the step count is a template parameter so that no
// branch with live accumulators on both sides is needed.
#pragma once
#include <type_traits>

#include "bb_common.h"

namespace bb {

enum { MODE_PLAIN = 0, MODE_GATEUP = 1, MODE_LN = 2, MODE_GATEUP_PRE = 3, MODE_LN_PRE = 4 };

struct GemmArgs {
    const u16* A;        // [M, K]
    const u16* B0;       // [K, N]  (BT kernels: [N, K])
    const u16* B1;       // [K, N]  (GATEUP only: W3; BT kernels: [N, K])
    u16* C;              // [M, N]
    const u16* gain;     // [K]     (GATEUP: g, LN: gamma)
    const float* colc;   // [N]     (LN: gamma^T W)
    const float* colb;   // [N]     (LN: beta^T W)
    int M, N, K;
    int lda, ldb, ldc;
    int tiles_m, tiles_n, tiles_per_xcd;
    int group_m;         // row tiles per group of the tile order (see the kernel's tile coordinates)
    float eps;
    // split contraction (SPLIT kernels): `nsplit` workgroups per tile, each with
    // `nk_split` contraction steps; fp32 partial results part[split][M][ldp]
    // (GATEUP: columns [0,N) the W1 product, [N,2N) the W3 product) and the
    // partial sums of squares ssqpart[split][M]
    int nsplit, nk_split, ldp;
    float* part;
    float* ssqpart;
    const float* rowstat;   // LN_PRE: [M][2] inverse standard deviation and mean per row
    const u16* res;     // PLAIN: residual added to the product before the one rounding ([M, N], row length ldr), or null
    int ldr;
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
// its own global address src to LDS address dst + 16 i (dst is the same for
// all lanes).
__device__ __forceinline__ void load_to_lds16(const void* src, void* dst) {
    __builtin_amdgcn_global_load_lds((gptr_t)src, (lptr_t)dst, 16, 0, 0);
}
// the same with the non-temporal cache policy (data that is read once)
__device__ __forceinline__ void load_to_lds16_nt(const void* src, void* dst) {
    __builtin_amdgcn_global_load_lds((gptr_t)src, (lptr_t)dst, 16, 0, 2);
}

// The same through a buffer resource (base address and size in four scalar registers): lane i copies the 16
// bytes at base + voff (per lane) + soff (wavefront-uniform, a scalar register) to LDS address dst + 16 i.  The
// address needs no vector instruction, and the compiler counts this form as a vector-memory load only:
// next to a pending global_load_lds it makes every wait for an LDS read a wait for ALL LDS reads
// (s_waitcnt lgkmcnt(0)), because that instruction belongs to the FLAT family, whose members may touch LDS
// and memory in one go.
typedef __amdgpu_buffer_rsrc_t rsrc_t;
__device__ __forceinline__ rsrc_t make_rsrc(const void* base, size_t bytes) {
    // (raw buffer: stride 0, size in bytes, 32-bit data format)
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)(u32)bytes, 0x00020000);
}
__device__ __forceinline__ void buffer_to_lds16(rsrc_t r, u32 voff, u32 soff, void* dst) {
    __builtin_amdgcn_raw_ptr_buffer_load_lds(r, (lptr_t)dst, 16, (int)voff, (int)soff, 0, 0);
}

// LDS byte address of a pointer into a __shared__ array
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

// The same transposition for 32-bit values: in, quad lane e holds y[i] = E[i][e];
// out, y[j] = E[e][j].  upper = (e & 2) != 0, odd = (e & 1) != 0.
template <int CTRL>
__device__ __forceinline__ float quad_swap(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, false));
}
__device__ __forceinline__ void quad_transpose_f32(float (&y)[4], bool upper, bool odd) {
    const float r0 = quad_swap<0x4E>(upper ? y[0] : y[2]), r1 = quad_swap<0x4E>(upper ? y[1] : y[3]);   // lane ^ 2
    // rows 2h, 2h + 1 (h = upper) of columns e & 1 (x) and (e & 1) + 2 (z)
    const float x0 = upper ? r0 : y[0], x1 = upper ? r1 : y[1];
    const float z0 = upper ? y[2] : r0, z1 = upper ? y[3] : r1;
    const float q0 = quad_swap<0xB1>(odd ? x0 : x1), q1 = quad_swap<0xB1>(odd ? z0 : z1);               // lane ^ 1
    y[0] = odd ? q0 : x0;
    y[1] = odd ? x1 : q0;
    y[2] = odd ? q1 : z0;
    y[3] = odd ? z1 : q1;
}

// FULL: every tile is complete in the contraction (K % 64 == 0) and A and B are smaller than 4 GiB
// each, so the main loop has no bounds checks and addresses its loads with 32-bit offsets.  The numbers
// of rows and of columns are free: lanes of a ragged last row (column) tile read the last valid row
// (chunk of columns), the epilogue stores only valid elements.
// ODD: the number of contraction steps of a workgroup is odd.
// SPLIT (PLAIN, GATEUP; for shapes with fewer tiles than half the compute
// units, i.e. few rows): nsplit workgroups share a tile, each contracts
// nk_split steps of the contraction range (steps past the end load zeros, so
// SPLIT kernels are built with FULL = false unless the steps divide evenly
// among the workgroups) and stores its fp32 accumulators
// (GATEUP: and its partial row sums of squares) instead of running the
// epilogue; splitk_reduce_kernel adds the partial results in fixed order and
// applies the epilogue.  This is Rule 3's parallel reduction over the
// contraction blocks, with per-workgroup partial results instead of atomics.
// BT: B is given transposed, [N, K] row-major (ldb = its row length): the layout
// of the paper's block programs (W^T) and of linear-layer checkpoints.  Its tile
// then lies in LDS exactly like the A tile (rows of 8 contraction chunks, same
// swizzle, same load-to-LDS role) and its fragments are plain 128-bit reads.
// NW: wavefronts per workgroup.  4 (one per SIMD, a 128 x 128 or 64 x 256 wavefront tile in 256 accumulator registers),
// or, on 256-row tiles, 8 (two per SIMD, 128 x 64 or 32 x 256 each in 128 accumulator registers: while one wavefront's
// LDS reads, load-to-LDS instructions and prologue arithmetic issue, the other's matrix instructions do).
template <int MODE, int BM, bool FULL, bool ODD, bool SPLIT = false, bool BT = false, int NW = 4>
__global__ __launch_bounds__(64 * NW) void gemm_kernel(const GemmArgs p) {
    static_assert(NW == 4 || (NW == 8 && BM == 256), "8 wavefronts: 256-row tiles");
    // (2 x 2 wherever the A fragments need no prologue: least LDS read traffic)
    // wavefronts along the rows (with a prologue: all of them, so that no A fragment is prepared twice)
    constexpr int WM = (MODE == MODE_PLAIN || MODE == MODE_GATEUP_PRE || MODE == MODE_LN_PRE) ? 2 : NW;
    constexpr int WN = NW / WM;                         // and along the columns
    constexpr int WR = BM / WM, WC = 256 / WN;          // wavefront tile
    constexpr int MT = WR / 32, NT = WC / 32;           // 32x32 subtiles per wavefront
    constexpr bool DUAL = MODE == MODE_GATEUP || MODE == MODE_GATEUP_PRE;   // two products per tile, SwiGLU epilogue
    constexpr bool COOK = MODE == MODE_GATEUP || MODE == MODE_LN;           // norm prologue on the A fragments
    constexpr bool LNE = MODE == MODE_LN || MODE == MODE_LN_PRE;            // epilogue r (P - mu c) + b
    constexpr int NCOL = DUAL ? 128 : 256;                   // output columns per tile
    constexpr int ADMA = BM / (8 * NW);   // A load-to-LDS instructions per wavefront and step
    constexpr int BDMA = 32 / NW;         // B load-to-LDS instructions per wavefront and step
    // (the B arrays come first: the many transposing reads of a step then reach
    // their addresses with the 16-bit displacement of the LDS instructions)
    __shared__ u32x4 sB0[64 * 32], sB1[64 * 32];     // [contraction row][32 chunks], swizzled
    __shared__ u32x4 xA0[BM * 8], xA1[BM * 8];       // [row][8 chunks], lds_pos swizzle
    __shared__ u32x4 sG0[64], sG1[64];               // gain tile: chunks 0..7 (stored 8 times)
    __shared__ float stat0[BM];                      // inverse norm / inverse std
    __shared__ float stat1[BM];                      // mean (LN)

    // ---- tile coordinates: workgroup id -> XCD (id % 8) -> contiguous range
    // of the tile order per XCD.  The order runs through groups of `group_m` row
    // tiles, inside a group row tiles fastest: the 32 tiles that an XCD works
    // on together are then a block of about 8 row tiles x 4 column tiles, the
    // shape with the fewest distinct A and B tiles (12 against 18 for 16 x 2 and 33 for
    // 32 x 1), which is what the XCD's L2 has to fetch over the fabric per step.
    const int xcd = blockIdx.x & 7, local = blockIdx.x >> 3;
    const int lin = xcd * p.tiles_per_xcd + local;
    const int ntiles = p.tiles_m * p.tiles_n;
    if (local >= p.tiles_per_xcd || lin >= (SPLIT ? ntiles * p.nsplit : ntiles)) return;
    const int tile = SPLIT ? lin % ntiles : lin, split = SPLIT ? lin / ntiles : 0;
    const int per_group = p.group_m * p.tiles_n;
    const int grp = tile / per_group, in_grp = tile - grp * per_group;
    const int rows_grp = min(p.group_m, p.tiles_m - grp * p.group_m);      // (the last group may be shorter)
    const int tm = grp * p.group_m + in_grp % rows_grp, tn = in_grp / rows_grp;
    const int kt0 = SPLIT ? split * p.nk_split : 0;           // first contraction step of this workgroup
    const int m0 = tm * BM, n0 = tn * NCOL;

    const int t = threadIdx.x, lane = t & 63;
    const int w = __builtin_amdgcn_readfirstlane(t >> 6);        // in a scalar register: what is built from it stays scalar
    const int wm = w / WN, wn = w % WN;
    const int l32 = lane & 31, lhi = lane >> 5;
    const u16* const zsrc = reinterpret_cast<const u16*>(&gemm_zero_chunk);

    // Source addresses of the load-to-LDS instructions.  With FULL set (complete
    // tiles, and every operand smaller than 4 GiB) an address is the matrix
    // pointer (a kernel argument, in scalar registers) plus a 32-bit byte
    // offset = a wavefront-uniform part (scalar arithmetic) + a lane constant:
    // one 32-bit vector add per instruction.  Otherwise the offset is 64-bit and
    // lanes outside the matrix read the zero chunk instead.
    // (FULL: through buffer resources, the uniform part in a scalar register, no vector arithmetic at all)
    const rsrc_t rsA = make_rsrc(p.A, (size_t)p.M * p.lda * 2);
    const rsrc_t rsB0 = make_rsrc(p.B0, (size_t)(BT ? p.N : p.K) * p.ldb * 2);
    const rsrc_t rsB1 = make_rsrc(DUAL ? p.B1 : p.B0, (size_t)(BT ? p.N : p.K) * p.ldb * 2);
    const rsrc_t rsG = make_rsrc(COOK ? p.gain : p.A, (size_t)p.K * 2);
    auto copy16 = [&](const u16* base, rsrc_t rs, size_t uniform_elems, u32 lane_elems, bool ok, void* dst) {
        if (FULL) {
            buffer_to_lds16(rs, lane_elems * 2u, (u32)uniform_elems * 2u, dst);
        } else {
            const u16* g = base + uniform_elems + lane_elems;
            load_to_lds16(ok ? g : zsrc, dst);
        }
    };

    // ---- A: load-to-LDS role.  One instruction fills 64 chunks = 8 tile rows,
    // lane i -> chunk position i % 8 of row i / 8 (+ 8 per instruction), which
    // holds source chunk (i % 8) ^ ((row / 2) % 8): two lane constants, for even
    // and odd instructions.  Wavefront w issues row groups w ADMA .. w ADMA + ADMA-1.
    const int rowA = 8 * ADMA * w + (lane >> 3);                 // + 8 j for instruction j
    int kcA[2];
    u32 laneA[2];
#pragma unroll
    for (int o = 0; o < 2; ++o) {
        kcA[o] = (lane & 7) ^ (((rowA + 8 * o) >> 1) & 7);
        laneA[o] = (u32)((lane >> 3) * p.lda + 8 * kcA[o]);
    }
    // FULL kernels take any number of rows: a lane whose row lies past the last one reads the last row instead (the
    // row tile computes rows that the epilogue does not store).  Per instruction j the wavefront-uniform row base is
    // clamped too, so that the lane part stays non-negative; in every tile but a ragged last one these are the
    // values above.
    int ubaseA[ADMA];
    u32 laneAc[ADMA];
    if (FULL) {
#pragma unroll
        for (int j = 0; j < ADMA; ++j) {
            const int rb = m0 + 8 * ADMA * w + 8 * j;
            ubaseA[j] = min(rb, p.M - 1);
            laneAc[j] = (u32)((min(rb + (lane >> 3), p.M - 1) - ubaseA[j]) * p.lda + 8 * kcA[j & 1]);
        }
    }

    // ---- B: load-to-LDS role.
    // PLAIN, LN: the LDS tile is [64 rows][32 chunks]; one instruction fills two
    // rows, lane i -> byte 16 i.  Wavefront w issues row pairs w, w+4, ..., w+28,
    // so this lane always serves tile rows = 2 w + lhi (mod 8) and chunk position
    // l32, which holds source chunk l32 ^ 4 (row % 4) = columns n0 + 8 chunk.
    // GATEUP: the LDS tile is two half tiles [W1 | W3][64 rows][16 chunks] (the
    // 128 columns of W1, then the same 128 of W3), so that one instruction reads
    // one matrix only: it fills four rows of a half tile, lane i -> row i / 16,
    // chunk position i % 16, which holds source chunk (i % 16) ^ 4 (row % 4).
    // Instructions 0..3 of a wavefront serve W1, 4..7 W3, row groups
    // 4 (q % 4) + w.  Subtiles tt and tt + 4 of the (single-column) wavefront
    // tile are then the gate and the up product of the same hidden units.
    constexpr bool HALF = DUAL;
    // HALF: a wavefront's subtiles 0 .. HT-1 are its columns of W1, HT .. NT-1 the same columns of W3
    // (columns (128 / WN) wn + 32 (tt % HT) + ... of either half tile)
    constexpr int HT = HALF ? NT / 2 : 4;
    constexpr int HWC = 128 / WN;                                // a wavefront's columns within a half tile
    const int rowBl = HALF ? (lane >> 4) : lhi;                  // row of this lane within an instruction
    const int chunkB = HALF ? ((lane & 15) ^ ((lane >> 4) << 2)) : (l32 ^ (((2 * w + lhi) & 3) << 2));
    const int colB = n0 + 8 * chunkB;
    const bool colB_ok = FULL || colB < p.N;
    // (FULL kernels take any number of columns: a lane whose chunk of columns lies past the last one reads the last
    // chunk instead; the ragged last column tile computes columns that the epilogue does not store)
    const u32 laneB = (u32)(rowBl * p.ldb + (FULL ? min(8 * chunkB, p.N - 8 - n0) : (colB_ok ? 8 * chunkB : 0)));
    // BT: like the A tile.  256 tile rows (= output columns; GATEUP: 128 rows of
    // W1^T, then the same 128 of W3^T), BDMA instructions per wavefront, each 8 rows.
    const int rowT = 8 * BDMA * w + (lane >> 3);                 // + 8 j for instruction j
    int kcT[2];
    u32 laneT[2];
#pragma unroll
    for (int o = 0; o < 2; ++o) {
        kcT[o] = (lane & 7) ^ (((rowT + 8 * o) >> 1) & 7);
        laneT[o] = (u32)((lane >> 3) * p.ldb + 8 * kcT[o]);
    }
    // (FULL, transposed weights: the rows of B are output columns; clamped like the rows of A)
    int ubaseT[BDMA];
    u32 laneTc[BDMA];
    if (FULL && BT) {
#pragma unroll
        for (int q = 0; q < BDMA; ++q) {
            const int r0 = 8 * BDMA * w + 8 * q;
            const int nrow = HALF ? n0 + (r0 & 127) : n0 + r0;
            ubaseT[q] = min(nrow, p.N - 1);
            laneTc[q] = (u32)((min(nrow + (lane >> 3), p.N - 1) - ubaseT[q]) * p.ldb + 8 * kcT[q & 1]);
        }
    }

    // ---- B: fragment-read role.  Group b = lane / 16 of a transposing read
    // covers contraction rows 8 (b / 2) + 4 h + (0..3) (+ 16 per matrix
    // instruction) and columns 32 tt + 16 (b % 2) + (0..15) of the wavefront's
    // columns; lane i' = lane % 16 supplies the address of row i' / 4, 4-column
    // piece i' % 4.  The 32 lanes served together read 4 rows x 64 bytes; rows
    // are a multiple of 256 bytes apart, i.e. on the same banks, so the 16-byte
    // chunk index is XOR-swizzled with 4 (row % 4): the four rows then take the
    // four 64-byte quarters of the 256-byte bank line.  The XOR touches the
    // chunk bits that tt % 4 occupies, hence one byte offset per tt % 4 (tt / 4
    // is a plain displacement: 256 bytes, or the other half tile).
    constexpr int BROW = HALF ? 256 : 512;                       // bytes per LDS tile row
    constexpr int BTT4 = HALF ? 64 * 256 : 256;                  // displacement of subtile tt + 4
    int offB[4];
    {
        const int b = lane >> 4, ip = lane & 15;
        const int r = 8 * (b >> 1) + (ip >> 2);
        const int piece = ip & 3;
#pragma unroll
        for (int o = 0; o < 4; ++o) {
            const int chunk = (HALF ? (HWC / 8) * wn : (WC / 8) * wn) + 4 * o + 2 * (b & 1) + (piece >> 1);
            offB[o] = r * BROW + ((chunk ^ ((r & 3) << 2)) << 4) + 8 * (piece & 1);
        }
    }

    // Quarter `part` (0..3) of the load-to-LDS instructions of B tile kt (BDMA per
    // wavefront and tile) into LDS array dB
    auto dma_b = [&](int kt, u32x4* dB, int part) {
        const int k0 = (kt0 + kt) * GEMM_BK;
#pragma unroll
        for (int qq = 0; qq < BDMA / 4; ++qq) {
            const int q = (BDMA / 4) * part + qq;
            if (BT) {
                const int r0 = 8 * BDMA * w + 8 * q;                 // first tile row of the instruction
                const bool second = HALF && r0 >= 128;
                const int nrow = HALF ? n0 + (r0 & 127) : n0 + r0;   // first matrix row (output column)
                if (FULL)
                    copy16(second ? p.B1 : p.B0, second ? rsB1 : rsB0, (size_t)ubaseT[q] * p.ldb + k0, laneTc[q], true,
                           dB + (BDMA * w + q) * 64);
                else
                    copy16(second ? p.B1 : p.B0, second ? rsB1 : rsB0, (size_t)nrow * p.ldb + k0, laneT[q & 1],
                           k0 + 8 * kcT[q & 1] < p.K && nrow + (lane >> 3) < p.N, dB + (BDMA * w + q) * 64);
            } else if (HALF) {
                const int idx = NW * q + w;                          // four-row group of the two half tiles
                const int hf = idx >> 4, rg = idx & 15;
                copy16(hf ? p.B1 : p.B0, hf ? rsB1 : rsB0, (size_t)(k0 + 4 * rg) * p.ldb + n0, laneB,
                       colB_ok && k0 + 4 * rg + rowBl < p.K, dB + hf * 1024 + rg * 64);
            } else {
                const int rp = w + NW * q;                           // row pair of the tile
                copy16(p.B0, rsB0, (size_t)(k0 + 2 * rp) * p.ldb + n0, laneB, colB_ok && k0 + 2 * rp + rowBl < p.K,
                       dB + rp * 64);
            }
        }
    };
    // Quarter `part` of A tile kt (ADMA instructions per wavefront and tile)
    // into dA; the last quarter also brings the gain chunks into dG (every
    // wavefront writes the same bytes there: no branch in the step)
    auto dma_a = [&](int kt, u32x4* dA, u32x4* dG, int part) {
        const int k0 = (kt0 + kt) * GEMM_BK;
#pragma unroll
        for (int jj = 0; jj < ADMA / 4; ++jj) {
            const int j = (ADMA / 4) * part + jj;
            if (FULL)
                copy16(p.A, rsA, (size_t)ubaseA[j] * p.lda + k0, laneAc[j], true, dA + (ADMA * w + j) * 64);
            else
                copy16(p.A, rsA, (size_t)(m0 + 8 * ADMA * w + 8 * j) * p.lda + k0, laneA[j & 1],
                       k0 + 8 * kcA[j & 1] < p.K && m0 + rowA + 8 * j < p.M, dA + (ADMA * w + j) * 64);
        }
        if (COOK && part == 3) {
            copy16(p.gain, rsG, (size_t)k0, (u32)(8 * (lane & 7)), k0 + 8 * (lane & 7) < p.K, dG);
        }
    };

    f32x16 acc[MT][NT];
#pragma unroll
    for (int s = 0; s < MT; ++s)
#pragma unroll
        for (int tt = 0; tt < NT; ++tt)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[s][tt][v] = 0.f;
    // row sums of the fragments this lane has seen: row 32 s + l32 of the
    // wavefront's rows, contraction chunks with (chunk % 2) == lhi
    // (two partial sums each, for the even and the odd elements)
    float ssq[MT][2], ssum[MT][2];
#pragma unroll
    for (int s = 0; s < MT; ++s) { ssq[s][0] = ssq[s][1] = 0.f; ssum[s][0] = ssum[s][1] = 0.f; }

    using C0 = std::integral_constant<int, 0>;
    using C1 = std::integral_constant<int, 1>;

    const int nk = SPLIT ? p.nk_split : (p.K + GEMM_BK - 1) / GEMM_BK;    // steps of this workgroup

    // fragments of contraction slice ks (16 indices) of one LDS buffer set
    Chunk fa[2][MT], fb[2][NT], fg[2];
    auto frag_load = [&](const u32x4* bufA, auto PBC, const u32x4* bufG, int ks, auto SETC) {
        constexpr int S = decltype(SETC)::value;
        constexpr int PB = decltype(PBC)::value;      // which B array
        const int kc = 2 * ks + lhi;
#pragma unroll
        for (int s = 0; s < MT; ++s) fa[S][s].u = bufA[lds_pos(WR * wm + 32 * s + l32, kc)];
        if (COOK) fg[S].u = bufG[kc];
#pragma unroll
        for (int tt = 0; tt < NT; ++tt) {
            if (BT) {
                fb[S][tt].u = (PB ? sB1 : sB0)[lds_pos(
                    (HALF ? 128 * (tt / HT) + HWC * wn + 32 * (tt % HT) : WC * wn + 32 * tt) + l32, kc)];
            } else {
                const char* q = reinterpret_cast<const char*>(PB ? sB1 : sB0) + offB[tt % HT] + ks * (16 * BROW) + BTT4 * (tt / HT);
                const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(q));
                const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(q + 4 * BROW));
                u32x2 l2 = *reinterpret_cast<const u32x2*>(&lo), h2 = *reinterpret_cast<const u32x2*>(&hi);
                fb[S][tt].u = u32x4{l2[0], l2[1], h2[0], h2[1]};
            }
        }
    };
    // norm prologue on the A fragments of set S: row sums, gain, rounding.
    // The MT x 4 (subtile, dword) items are numbered s * 4 + q; one call works
    // on items [lo, hi).
    auto cook = [&](auto SETC, int lo, int hi) {
        constexpr int S = decltype(SETC)::value;
        if (!COOK) return;
        const u32x4 gv = fg[S].u;
#pragma unroll
        for (int s = 0; s < MT; ++s) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int item = 4 * s + q;
                if (item < lo || item >= hi) continue;
                const u32 xw = fa[S][s].u[q];
                const float xl = bf_lo(xw), xh = bf_hi(xw);
                // (plain multiply-adds: the bf16 dot-product instruction does not
                // overlap with matrix instructions and costs ~20 cycles next to them)
                ssq[s][0] = fmaf(xl, xl, ssq[s][0]);
                ssq[s][1] = fmaf(xh, xh, ssq[s][1]);
                if (MODE == MODE_LN) { ssum[s][0] += xl; ssum[s][1] += xh; }
                fa[S][s].u[q] = pack_bf16(xl * bf_lo(gv[q]), xh * bf_hi(gv[q]));
            }
        }
    };
    constexpr int NMMA = MT * NT;          // matrix instructions per group (one contraction slice)
    constexpr int QMMA = NMMA / 4;         // per quarter of a group
    static_assert(NT >= QMMA, "the first quarter must use subtile row 0 only");
    // quarter `part` of the matrix instructions of fragment set S, subtile rows first
    auto mma = [&](auto SETC, int part) {
        constexpr int S = decltype(SETC)::value;
#pragma unroll
        for (int s = 0; s < MT; ++s)
#pragma unroll
            for (int tt = 0; tt < NT; ++tt) {
                const int i = s * NT + tt;
                if (i / QMMA != part) continue;
                acc[s][tt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[S][s].v, fb[S][tt].v, acc[s][tt], 0, 0, 0);
            }
    };
    constexpr int NDSR = MT + 2 * NT + (COOK ? 1 : 0);   // LDS reads per fragment set
    constexpr int ITEMS = 4 * MT;                                      // prologue items per fragment set
    constexpr int P1 = (ITEMS + 2) / 3, P2 = (2 * ITEMS + 2) / 3;      // item ranges of quarters 1, 2, 3
    // Placement request for one group of matrix instructions (the instructions
    // issue in order, so only what stands between two matrix instructions runs
    // in the shadow of the first).  The A and gain reads of the next fragment
    // set come first (the prologue waits for them); then every matrix
    // instruction is followed by its share of the B reads (so that the four
    // wavefronts do not burst into the LDS together), a slice of the vector ALU
    // work and, every second time, one load-to-LDS.
    constexpr int NDSR_A = MT + (COOK ? 1 : 0);
    constexpr int DSR_PER = ((BT ? 1 : 2) * NT + NMMA - 1) / NMMA;
    constexpr int VQ = !COOK ? 2 : ((MODE == MODE_LN ? 9 : 7) * ITEMS + 8) / NMMA + 3;   // vector ALU slice per matrix instruction
    auto pattern = [&](bool with_frags, bool with_dma) {
        if (with_frags) __builtin_amdgcn_sched_group_barrier(0x100, NDSR_A, 0);
#pragma unroll
        for (int i = 0; i < NMMA; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            if (with_frags) __builtin_amdgcn_sched_group_barrier(0x100, DSR_PER, 0);
            __builtin_amdgcn_sched_group_barrier(0x002, VQ, 0);
            if (with_dma && ((i & 1) || NMMA < 16)) __builtin_amdgcn_sched_group_barrier(0x010, 1, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
    };
    auto mma_all = [&](auto SETC) { mma(SETC, 0); mma(SETC, 1); mma(SETC, 2); mma(SETC, 3); };

    // One contraction step on buffer set PAR (tile kt, kt % 2 == PAR, not the
    // last tile): four groups of matrix instructions (one per 16 contraction
    // indices).  Each group reads the next group's fragments and runs the norm
    // prologue on them.  The step is rotated against the tiles: on entry
    // fragment set 0 already holds slice 0 of tile kt; the barrier stands before
    // the last group, which reads slice 0 of tile kt + 1 from the other buffer
    // set, so that no wavefront stands at a barrier or waits for its first
    // fragments with nothing queued for the matrix core.  Loads: group 0 issues
    // the A tile kt + 1 into the other set (free since the previous barrier),
    // the last group issues the B tile kt + 2 into this set (free since this
    // step's barrier; for the last but one tile there is no such tile and the
    // last tile is fetched again into the then unused set).
    auto step = [&](int kt, auto PARC) {
        constexpr int PAR = decltype(PARC)::value;
        using NPAR = std::integral_constant<int, 1 - PAR>;
        const u32x4* const curA = PAR ? xA1 : xA0;
        const u32x4* const curG = PAR ? sG1 : sG0;
        u32x4* const curB = PAR ? sB1 : sB0;
        u32x4* const nxtA = PAR ? xA0 : xA1;
        u32x4* const nxtG = PAR ? sG0 : sG1;
        // group 0
        frag_load(curA, PARC, curG, 1, C1());
        mma_all(C0());
        cook(C1(), 0, ITEMS);
        dma_a(kt + 1, nxtA, nxtG, 0);
        dma_a(kt + 1, nxtA, nxtG, 1);
        pattern(true, true);
        // group 1
        frag_load(curA, PARC, curG, 2, C0());
        mma_all(C1());
        cook(C0(), 0, ITEMS);
        dma_a(kt + 1, nxtA, nxtG, 2);
        dma_a(kt + 1, nxtA, nxtG, 3);
        pattern(true, true);
        // group 2
        frag_load(curA, PARC, curG, 3, C1());
        mma_all(C0());
        cook(C1(), 0, ITEMS);
        pattern(true, false);
        __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
        __syncthreads();
        // group 3
        frag_load(nxtA, NPAR(), nxtG, 0, C0());
        mma_all(C1());
        cook(C0(), 0, ITEMS);
        const int kb = min(kt + 2, nk - 1);
#pragma unroll
        for (int part = 0; part < 4; ++part) dma_b(kb, curB, part);
        pattern(true, true);
    };
    auto last_step = [&](auto PARC) {          // last tile: nothing left to load
        constexpr int PAR = decltype(PARC)::value;
        const u32x4* const curA = PAR ? xA1 : xA0;
        const u32x4* const curG = PAR ? sG1 : sG0;
        frag_load(curA, PARC, curG, 1, C1());
        mma_all(C0());
        cook(C1(), 0, ITEMS);
        pattern(true, false);
        frag_load(curA, PARC, curG, 2, C0());
        mma_all(C1());
        cook(C0(), 0, ITEMS);
        pattern(true, false);
        frag_load(curA, PARC, curG, 3, C1());
        mma_all(C0());
        cook(C1(), 0, ITEMS);
        pattern(true, false);
        mma_all(C1());
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    };

    // prologue: tile 0 into buffer set 0, its slice 0 into fragment set 0, B
    // tile 1 under way
#pragma unroll
    for (int part = 0; part < 4; ++part) {
        dma_b(0, sB0, part);
        dma_a(0, xA0, sG0, part);
    }
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    __syncthreads();
#pragma unroll
    for (int part = 0; part < 4; ++part) dma_b(min(1, nk - 1), sB1, part);
    frag_load(xA0, C0(), sG0, 0, C0());
    cook(C0(), 0, ITEMS);
    __builtin_amdgcn_sched_barrier(0);

    // pairs of steps; the tail depends on the parity of nk only
    {
        int kt = 0;
        for (; kt + 2 < nk; kt += 2) {
            step(kt, C0());
            step(kt + 1, C1());
        }
        if (ODD) {
            last_step(C0());
        } else {
            step(kt, C0());
            last_step(C1());
        }
    }

    // ---- split contraction: store the partial results, no epilogue
    if (SPLIT) {
        static_assert(!SPLIT || MODE == MODE_PLAIN || MODE == MODE_GATEUP, "split kernels: PLAIN or GATEUP");
        float* const part = p.part + (size_t)split * p.M * p.ldp;
        const int eqs = l32 & 3;
#pragma unroll
        for (int s = 0; s < MT; ++s)
#pragma unroll
            for (int tt = 0; tt < NT; ++tt) {
                // GATEUP: subtiles 0..3 are the W1 product of hidden units n0 + 32 tt + ..., 4..7 the W3 product.
                // Four registers (4 rows x this lane's column) are transposed within the quad: the lane then
                // holds 4 consecutive columns of one row, a 16-byte store.
                const int col = (DUAL ? n0 + HWC * wn + 32 * (tt % HT) : n0 + WC * wn + 32 * tt) + 4 * (l32 >> 2);
                const int pcol = (DUAL && tt >= HT) ? p.N + col : col;
#pragma unroll
                for (int vg = 0; vg < 4; ++vg) {
                    float y[4] = {acc[s][tt][4 * vg], acc[s][tt][4 * vg + 1], acc[s][tt][4 * vg + 2], acc[s][tt][4 * vg + 3]};
                    quad_transpose_f32(y, (eqs & 2) != 0, (eqs & 1) != 0);
                    const int m = m0 + WR * wm + 32 * s + 8 * vg + 4 * lhi + eqs;
                    if (m < p.M && col < p.N)           // (N is a multiple of 8: four columns are inside together)
                        *reinterpret_cast<f32x4*>(part + (size_t)m * p.ldp + pcol) = f32x4{y[0], y[1], y[2], y[3]};
                }
            }
        if (MODE == MODE_GATEUP) {
#pragma unroll
            for (int s = 0; s < MT; ++s) {
                const float q2 = ssq[s][0] + ssq[s][1];
                const float s2 = q2 + __shfl_xor(q2, 32);
                const int m = m0 + WR * wm + 32 * s + l32;
                if (lhi == 0 && tn == 0 && m < p.M) p.ssqpart[(size_t)split * p.M + m] = s2;
            }
        }
        return;
    }

    // ---- row statistics: add the two lanes that share a row (lane, lane ^ 32)
    if (MODE == MODE_GATEUP_PRE) {
        // the inverse norms were computed by the row kernel that applied the gain
        for (int i = threadIdx.x; i < BM; i += 64 * NW) stat0[i] = (m0 + i < p.M) ? p.colc[m0 + i] : 0.f;
        __syncthreads();
    }
    if (MODE == MODE_LN_PRE) {
        // row statistics from the row kernel: rowstat[2 m] = inverse standard deviation, [2 m + 1] = mean
        for (int i = threadIdx.x; i < BM; i += 64 * NW) {
            const bool ok = m0 + i < p.M;
            stat0[i] = ok ? p.rowstat[2 * (size_t)(m0 + i)] : 0.f;
            stat1[i] = ok ? p.rowstat[2 * (size_t)(m0 + i) + 1] : 0.f;
        }
        __syncthreads();
    }
    if (COOK) {
#pragma unroll
        for (int s = 0; s < MT; ++s) {
            const float q2 = ssq[s][0] + ssq[s][1], q1 = ssum[s][0] + ssum[s][1];
            const float s2 = q2 + __shfl_xor(q2, 32);
            const float s1 = q1 + __shfl_xor(q1, 32);
            if (lhi == 0) {
                const float invK = 1.0f / (float)p.K;
                const int rl = WR * wm + 32 * s + l32;
                if (MODE == MODE_LN) {
                    const float mu = s1 * invK;
                    const float var = fmaxf(s2 * invK - mu * mu, 0.f);
                    stat0[rl] = rsqrtf(var + p.eps);
                    stat1[rl] = mu;
                } else {
                    stat0[rl] = rsqrtf(s2 * invK + p.eps);
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
    if (DUAL) {
        static_assert(!DUAL || NT % 2 == 0, "gate and up subtiles must share a wavefront");
        const int fcol = n0 + HWC * wn + 4 * (l32 >> 2);       // + 32 u
#pragma unroll
        for (int s = 0; s < MT; ++s) {
#pragma unroll
            for (int vg = 0; vg < 4; ++vg) {
                const int rl = WR * wm + 32 * s + 8 * vg + 4 * lhi;
                float r[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) r[i] = stat0[rl + i];
#pragma unroll
                for (int u = 0; u < NT / 2; ++u) {
                    float h[4];
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        h[i] = swiglu(r[i] * acc[s][u][4 * vg + i], r[i] * acc[s][u + NT / 2][4 * vg + i]);
                    u32 d0 = pack_bf16(h[0], h[1]), d1 = pack_bf16(h[2], h[3]);
                    quad_transpose(d0, d1, tup, tsel);
                    const int m = m0 + rl + eq, col = fcol + 32 * u;
                    if (m < p.M && col < p.N) {
                        u32x2 o = {d0, d1};
                        *reinterpret_cast<u32x2*>(p.C + (size_t)m * p.ldc + col) = o;
                    }
                }
            }
        }
    } else {
        const int ncol = n0 + WC * wn + l32;                 // + 32 tt: the column this lane accumulated
        const int scol = n0 + WC * wn + 4 * (l32 >> 2);      // + 32 tt: first of the 4 columns it stores
        float cc[NT], cb[NT];
        if (LNE) {
#pragma unroll
            for (int tt = 0; tt < NT; ++tt) {
                const bool ok = ncol + 32 * tt < p.N;
                cc[tt] = ok ? p.colc[ncol + 32 * tt] : 0.f;
                cb[tt] = ok ? p.colb[ncol + 32 * tt] : 0.f;
            }
        }
#pragma unroll
        for (int s = 0; s < MT; ++s) {
#pragma unroll
            for (int vg = 0; vg < 4; ++vg) {
                const int rl = WR * wm + 32 * s + 8 * vg + 4 * lhi;
                float r[4], mu[4];
                if (LNE) {
#pragma unroll
                    for (int i = 0; i < 4; ++i) { r[i] = stat0[rl + i]; mu[i] = stat1[rl + i]; }
                }
#pragma unroll
                for (int tt = 0; tt < NT; ++tt) {
                    float y[4];
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        y[i] = acc[s][tt][4 * vg + i];
                        if (LNE) y[i] = fmaf(r[i], y[i] - mu[i] * cc[tt], cb[tt]);
                    }
                    const int m = m0 + rl + eq, col = scol + 32 * tt;
                    const bool inside = m < p.M && col < p.N;
                    if (MODE == MODE_PLAIN && p.res != nullptr) {
                        // residual epilogue: transpose in fp32, add the residual's four values, round once
                        quad_transpose_f32(y, tup, (eq & 1) != 0);
                        if (inside) {
                            const u32x2 rr = *reinterpret_cast<const u32x2*>(p.res + (size_t)m * p.ldr + col);
                            u32x2 o = {pack_bf16(y[0] + bf_lo(rr[0]), y[1] + bf_hi(rr[0])),
                                       pack_bf16(y[2] + bf_lo(rr[1]), y[3] + bf_hi(rr[1]))};
                            *reinterpret_cast<u32x2*>(p.C + (size_t)m * p.ldc + col) = o;
                        }
                        continue;
                    }
                    u32 d0 = pack_bf16(y[0], y[1]), d1 = pack_bf16(y[2], y[3]);
                    quad_transpose(d0, d1, tup, tsel);
                    if (inside) {
                        u32x2 o = {d0, d1};
                        *reinterpret_cast<u32x2*>(p.C + (size_t)m * p.ldc + col) = o;
                    }
                }
            }
        }
    }
}

// Adds the nsplit partial results of a split contraction in fixed order and
// applies the epilogue: PLAIN C = bf16(sum [+ residual]); GATEUP h = SiLU(r P) (r Q) with
// r = (sum of the partial sums of squares / K + eps)^-1/2.  One thread per row
// and 8 consecutive output columns.
template <int MODE>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float* part, const float* ssqpart, u16* C,
                                                            int M, int N, int K, int ldp, int ldc, int nsplit,
                                                            float eps, const u16* res, int ldr) {
    const int groups = N / 8;
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (size_t)M * groups) return;
    const int m = (int)(idx / groups), c0 = 8 * (int)(idx % groups);
    f32x4 a0 = {0, 0, 0, 0}, a1 = a0, b0 = a0, b1 = a0;
    float s2 = 0.f;
    for (int sp = 0; sp < nsplit; ++sp) {
        const float* src = part + ((size_t)sp * M + m) * ldp + c0;
        a0 += *reinterpret_cast<const f32x4*>(src);
        a1 += *reinterpret_cast<const f32x4*>(src + 4);
        if (MODE == MODE_GATEUP) {
            b0 += *reinterpret_cast<const f32x4*>(src + N);
            b1 += *reinterpret_cast<const f32x4*>(src + N + 4);
            s2 += ssqpart[(size_t)sp * M + m];
        }
    }
    u32x4 o;
    if (MODE == MODE_GATEUP) {
        const float r = rsqrtf(s2 / (float)K + eps);
        o = u32x4{pack_bf16(swiglu(r * a0[0], r * b0[0]), swiglu(r * a0[1], r * b0[1])),
                  pack_bf16(swiglu(r * a0[2], r * b0[2]), swiglu(r * a0[3], r * b0[3])),
                  pack_bf16(swiglu(r * a1[0], r * b1[0]), swiglu(r * a1[1], r * b1[1])),
                  pack_bf16(swiglu(r * a1[2], r * b1[2]), swiglu(r * a1[3], r * b1[3]))};
    } else {
        if (res != nullptr) {           // residual added before the one rounding
            const u32x4 rr = ldg16(res + (size_t)m * ldr + c0);
            a0 += f32x4{bf_lo(rr[0]), bf_hi(rr[0]), bf_lo(rr[1]), bf_hi(rr[1])};
            a1 += f32x4{bf_lo(rr[2]), bf_hi(rr[2]), bf_lo(rr[3]), bf_hi(rr[3])};
        }
        o = u32x4{pack_bf16(a0[0], a0[1]), pack_bf16(a0[2], a0[3]), pack_bf16(a1[0], a1[1]), pack_bf16(a1[2], a1[3])};
    }
    *reinterpret_cast<u32x4*>(C + (size_t)m * ldc + c0) = o;
}

}  // namespace bb
