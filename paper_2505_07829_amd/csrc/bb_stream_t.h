// Weight-streaming RMSNorm -> FFN-SwiGLU kernel for few rows (decode) on
// TRANSPOSED weights: W1^T, W3^T [F, D] and W2^T [D, F], the layout of the
// paper's block programs (Example 3 loads tiles of W^T, V^T, U^T) and of
// linear-layer checkpoints.
//
// In this layout the contraction index is the contiguous one, so the work can
// be dealt out by OUTPUT index and every workgroup owns one contiguous range of
// each matrix:
//
//   phase 1 (K-map): workgroup b owns hidden units [b upw, (b+1) upw): rows of
//     W1^T and W3^T, complete dot products over the model dimension.  No
//     partial sums leave the workgroup; sum x^2 is computed by every workgroup
//     for itself while it prepares bf16(x g) in LDS, the inverse norm is applied
//     after the dots (Rule 4), then Swish and the gate; the workgroup's piece of
//     the hidden block (16 x upw, bf16) goes to a scratch in global memory.
//   one grid barrier
//   phase 2 (N-map): workgroup b owns output columns [b cpw, (b+1) cpw): rows of
//     W2^T, complete dot products over the hidden dimension; residual, rounding,
//     store.
//
// Measured on this part: 256 workgroups that each read a contiguous range (in
// pieces of 256 bytes, sixteen rows interleaved) stream at 6.7-6.9 TB/s, the
// same bytes read as 256-byte pieces of rows 22 KB apart (what the row-major
// layout forces on a kernel that wants the contraction in registers) at 4.7.
//
// A wavefront works on groups of 16 rows (hidden units or output columns) and
// on every fourth item of their contraction range (the four wavefronts of a
// workgroup walk along the same 16 rows side by side, 1 KiB of every row at a
// time: few, long streams for the memory).  An item is 16 chunks of 8 elements
// of each of the 16 rows (256 contiguous bytes per row), fetched by four load
// instructions per matrix.  One instruction takes 8 rows x 128 contiguous bytes
// (whole cache lines; with 16 rows x 64 bytes per instruction the same stream
// ran a quarter slower): lane (n = lane % 16, q = lane / 16) loads chunk
// 8 j + 4 (n / 8) + q of row 8 h + n % 8 (h = which 8 rows, j = which 128
// bytes).  Its result is the B operand of TWO 16x16x32 matrix instructions: one
// whose A operand holds chunks 8 j + q of the 16 activation rows - columns 0..7
// of its result are partial dots of rows 8 h + 0..7 over the first 64 bytes -
// and one with chunks 8 j + 4 + q, whose columns 8..15 are the partial dots of
// the same rows over the second 64 bytes.  The other eight columns of either
// result are meaningless and dropped; the matrix cores have time to spare here.
// No transposition anywhere.
#pragma once
#include "bb_stream.h"

// (a timing build of a debugging driver may switch one of the two phase 2 streams off)
#ifndef BB_ST_W2
#define BB_ST_W2 true
#endif
#ifndef BB_ST_H
#define BB_ST_H true
#endif

namespace bb {

constexpr int STREAMT_THREADS = 256;
// cache policy of the weight loads: streamed once, non-temporal (phase 1 runs 4 us shorter than with
// the default policy on the decode workload)
#ifndef BB_ST_WMOD
#define BB_ST_WMOD " nt"
#endif
// cache policy of the hidden-block loads and whether an acquire fence precedes them (see the kernel)
#ifndef BB_ST_HMOD
#define BB_ST_HMOD " sc1"
#endif
#ifndef BB_ST_FENCE
#define BB_ST_FENCE 0
#endif
#ifndef BB_ST_NPF1
#define BB_ST_NPF1 4
#endif
#ifndef BB_ST_NPF2
#define BB_ST_NPF2 6
#endif
constexpr int STREAMT_NPF1 = BB_ST_NPF1;   // phase 1 items (8 KiB per wavefront) in flight
constexpr int STREAMT_NPF2 = BB_ST_NPF2;   // phase 2 items (4 KiB per wavefront) in flight
constexpr int STREAMT_MAXG = 8;      // groups of 16 rows per workgroup the host plans for (LDS for the partial sums)
constexpr int STREAMT_LDS = 160 * 1024;

struct StreamTArgs {
    const u16* X;      // [M, D], M <= 16
    const u16* g;      // [D]
    const u16* W1t;    // [F, D]
    const u16* W3t;    // [F, D]
    const u16* W2t;    // [D, F]
    const u16* R;      // [M, D] residual or null
    u16* Y;            // [M, D]
    u16* H;            // [Fp / 32][16][32] hidden block, bf16 (scratch): blocks of 32 units, so that one load
                       // instruction of phase 2 (16 rows x 64 bytes) reads 1 KiB of contiguous memory
    const u16* zeros;  // 16 zero bytes in global memory: what a lane outside the matrices loads.  (A kernel argument:
                       // of a global variable the compiler would know that it can be read ahead of time, and turn
                       // the loads back into branches around the real ones.)
    unsigned* bar;     // barrier words (see grid_arrive), shared with the row-major streaming kernel
    unsigned* epoch;   // grid barriers completed by earlier launches: the barrier words only ever increase, the count
                       // lives in device memory (workgroup 0 advances it), so the host keeps no state per launch
    unsigned* fault;   // one word of host memory mapped into the device: set when the barrier's bounded wait gives up
    unsigned spin_limit;   // polls after which it gives up
    int M, D, F, Fp;
    int upw, cpw;      // hidden units / output columns per workgroup
    int kblk;          // model channels whose bf16(x g) LDS holds at a time: a multiple of 512
    int cq2;           // chunks of 8 hidden units per wavefront in phase 2: a multiple of 16, 4 cq2 >= F / 8
    int red_off, stat_off;   // byte offsets in LDS of the partial sums and of the 16 row statistics
    float eps;
};

struct StreamTItem1 { u32x4 r1[4], r3[4]; };
struct StreamTItem2 { u32x4 r2[4], h[4]; };

// The weight stream is requested NPF items ahead with loads the compiler does not see as loads
// (it would otherwise move them next to their uses, or wait for all of them before the first
// use in a loop): an asm load leaves its destination registers "in flight", and async_ready()
// is the one place where a wavefront waits until at most N younger loads are outstanding; it
// takes the registers as in-out operands, so every use is ordered after the wait.  Vector
// memory loads of a wavefront return in order.
__device__ __forceinline__ void async_load16(u32x4& dst, const u16* src) {
    asm volatile("global_load_dwordx4 %0, %1, off" BB_ST_WMOD : "=v"(dst) : "v"(src));
}
__device__ __forceinline__ void async_load16_ordered(u32x4& dst, const u16* src) {   // not moved across fences
    asm volatile("global_load_dwordx4 %0, %1, off" BB_ST_HMOD : "=v"(dst) : "v"(src) : "memory");
}
// The four accumulators of a group of 16 rows -> one 16x16 tile in the matrix instruction's result
// layout (lane (n, q) holds rows 4 q .. 4 q + 3 of column n).  acc[h][0] is valid in columns 0..7 (rows
// 8 h + column), acc[h][1] in columns 8..15 (rows 8 h + column - 8); upper = this lane's column is >= 8.
__device__ __forceinline__ f32x4 shfl8(const f32x4 v) {
    f32x4 r;
#pragma unroll
    for (int i = 0; i < 4; ++i) r[i] = __shfl_xor(v[i], 8);
    return r;
}
__device__ __forceinline__ f32x4 fold16(const f32x4 (&acc)[2][2], int upper) {
    const f32x4 c0 = acc[0][0] + shfl8(acc[0][1]);      // columns 0..7: rows 0..7
    const f32x4 c1 = acc[1][0] + shfl8(acc[1][1]);      // columns 0..7: rows 8..15
    const f32x4 c1u = shfl8(c1);                        // ... moved to columns 8..15
    return upper ? c1u : c0;
}

template <int N>
__device__ __forceinline__ void async_wait() {
    asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N) : "memory");
}
__device__ __forceinline__ void async_tie(u32x4 (&a)[4], u32x4 (&b)[4]) {
    asm volatile(""
                 : "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3]), "+v"(b[0]), "+v"(b[1]), "+v"(b[2]), "+v"(b[3]));
}
template <int N>
__device__ __forceinline__ void async_ready(u32x4 (&a)[4], u32x4 (&b)[4]) {
    asm volatile("s_waitcnt vmcnt(%8)"
                 : "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3]), "+v"(b[0]), "+v"(b[1]), "+v"(b[2]), "+v"(b[3])
                 : "n"(N));
}

// The hidden block is written with agent-scope stores (written through, complete when
// acknowledged) and, after the barrier, read with agent-scope loads, which never return a stale
// cached copy.  Measured alternatives for the reads, phase 2 alone with the weight loads off:
// agent-scope loads 10.7 us, ordinary loads behind an agent-scope acquire fence 16 us (the fence
// invalidates the whole L2), ordinary loads without the fence (not coherent) 9.4 us.
#ifndef BB_HOST_ONLY   // (bb_api.hip includes this file for the argument structures only)
__global__ __launch_bounds__(STREAMT_THREADS) void ffn_stream_t_kernel(const StreamTArgs p) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int t = threadIdx.x, lane = t & 63;
    const int w = __builtin_amdgcn_readfirstlane(t >> 6);
    const int n = lane & 15, q4 = lane >> 4;
    const int rn = n & 7, hf = n >> 3;             // load role: row within a group of 8, which 64 bytes of the 128
    const int b = blockIdx.x;
    const u16* const zsrc = p.zeros;

    const int cq = p.kblk / 32;                    // chunks per wavefront and k-block, a multiple of 16
    const int xstride = 32 * cq + 8;               // elements per LDS row: 4 cq chunks and 16 bytes of padding
    u16* const xg = reinterpret_cast<u16*>(smem);                          // [16][xstride] bf16(x g)
    float* const red = reinterpret_cast<float*>(smem + p.red_off);         // [4][groups][2][64][4] / [4][groups][64][4]
    float* const stat = reinterpret_cast<float*>(smem + p.stat_off);       // [16] inverse norms, [4][16] partial sums of squares

    const unsigned bar_base =
        __builtin_amdgcn_readfirstlane(__hip_atomic_load(p.epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));

    BB_STREAM_TRACE(0);
    // =====================  phase 1: hidden units [u0, u1)  =====================
    const int u0 = min(p.F, b * p.upw), u1 = min(p.F, u0 + p.upw);
    const int ng = (u1 - u0 + 15) / 16;
    {
        const int nss = cq / 16;                   // items per group and k-block
        const int total = ng * nss;
        const int nkb = (p.D + p.kblk - 1) / p.kblk;
        float ssq[16];                             // this thread's share of sum x^2 of every row
#pragma unroll
        for (int m = 0; m < 16; ++m) ssq[m] = 0.f;
        for (int kbi = 0; kbi < nkb; ++kbi) {
            const int kb0 = kbi * p.kblk;
            const int nck = min(p.kblk, p.D - kb0) / 8;          // chunks of this k-block
            int gi_i = 0, s_i = 0;                               // position of the next item to request
            // (every load is unconditional: a lane outside the matrix reads the zero chunk instead)
            auto issue = [&](StreamTItem1& r) {
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const int row = u0 + 16 * gi_i + 8 * h + rn;
                    const bool rv = gi_i < ng && row < u1;
                    const int c0 = 16 * (4 * s_i + w) + 4 * hf + q4;    // chunk of instruction j: c0 + 8 j
                    const size_t off = (size_t)row * p.D + kb0 + 8 * c0;
#pragma unroll
                    for (int j = 0; j < 2; ++j) {
                        const bool ok = rv && c0 + 8 * j < nck;
                        async_load16(r.r1[2 * h + j], ok ? p.W1t + off + 64 * j : zsrc);
                        async_load16(r.r3[2 * h + j], ok ? p.W3t + off + 64 * j : zsrc);
                    }
                }
                if (++s_i == nss) { s_i = 0; ++gi_i; }
            };
            StreamTItem1 it[STREAMT_NPF1];
#pragma unroll
            for (int u = 0; u < STREAMT_NPF1; ++u) issue(it[u]);

            // ---- bf16(x g) of this k-block into LDS (zeros past the matrix), sum x^2 on the way.
            // A thread takes chunk columns t, t + 256, ... of all 16 rows: 17 independent loads each.
            if (kbi > 0) __syncthreads();                        // the previous k-block has been consumed
            for (int c = t; c < 4 * cq; c += STREAMT_THREADS) {
                const bool cv = c < nck;
                const size_t co = cv ? (size_t)kb0 + 8 * c : 0;
                const u32x4 gv = ldg16(p.g + co);
                u32x4 xv[16];
#pragma unroll
                for (int m = 0; m < 16; ++m) xv[m] = ldg16(p.X + (size_t)min(m, p.M - 1) * p.D + co);
#pragma unroll
                for (int m = 0; m < 16; ++m) {
                    u32x4 o = zero4();
                    if (cv && m < p.M) {
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const float x0 = bf_lo(xv[m][e]), x1 = bf_hi(xv[m][e]);
                            ssq[m] = fmaf(x0, x0, ssq[m]);
                            ssq[m] = fmaf(x1, x1, ssq[m]);
                            o[e] = pack_bf16(x0 * bf_lo(gv[e]), x1 * bf_hi(gv[e]));
                        }
                    }
                    *reinterpret_cast<u32x4*>(xg + m * xstride + 8 * c) = o;
                }
            }
            __syncthreads();
            BB_STREAM_TRACE(6);

            int gi_c = 0, s_c = 0;                               // position of the item being consumed
            f32x4 accP[2][2], accQ[2][2];                        // [which 8 rows][which 64 bytes]
            // (no load stands inside a branch: past the last item the loop works on dummies - zero
            // operands, results never stored - until the pass through the ring is complete)
            for (int idx0 = 0; idx0 < total; idx0 += STREAMT_NPF1) {
#pragma unroll
                for (int u = 0; u < STREAMT_NPF1; ++u) {
                    if (s_c == 0) {
#pragma unroll
                        for (int h = 0; h < 2; ++h)
#pragma unroll
                            for (int v = 0; v < 2; ++v) { accP[h][v] = f32x4{0, 0, 0, 0}; accQ[h][v] = f32x4{0, 0, 0, 0}; }
                    }
                    const u16* const xa = xg + n * xstride + 8 * (16 * (4 * s_c + w) + q4);
                    async_ready<8 * (STREAMT_NPF1 - 1)>(it[u].r1, it[u].r3);   // the younger items: 8 loads each
#pragma unroll
                    for (int j = 0; j < 2; ++j) {
                        Chunk alo, ahi;
                        alo.u = *reinterpret_cast<const u32x4*>(xa + 64 * j);
                        ahi.u = *reinterpret_cast<const u32x4*>(xa + 64 * j + 32);
#pragma unroll
                        for (int h = 0; h < 2; ++h) {
                            Chunk b1, b3;
                            b1.u = it[u].r1[2 * h + j];
                            b3.u = it[u].r3[2 * h + j];
                            accP[h][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(alo.v, b1.v, accP[h][0], 0, 0, 0);
                            accP[h][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ahi.v, b1.v, accP[h][1], 0, 0, 0);
                            accQ[h][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(alo.v, b3.v, accQ[h][0], 0, 0, 0);
                            accQ[h][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ahi.v, b3.v, accQ[h][1], 0, 0, 0);
                        }
                    }
                    issue(it[u]);
                    if (++s_c == nss) {
                        if (gi_c < ng) {
                            float* const mine = red + ((size_t)((w * ng + gi_c) * 2) * 64 + lane) * 4;   // this lane's partial sums
                            f32x4 oP = fold16(accP, hf), oQ = fold16(accQ, hf);
                            if (kbi > 0) {
                                oP += *reinterpret_cast<const f32x4*>(mine);
                                oQ += *reinterpret_cast<const f32x4*>(mine + 256);
                            }
                            *reinterpret_cast<f32x4*>(mine) = oP;
                            *reinterpret_cast<f32x4*>(mine + 256) = oQ;
                        }
                        s_c = 0;
                        ++gi_c;
                    }
                }
            }
            // the requests past the last item are still in flight: their registers stay reserved until
            // they have landed (a register reused earlier would be overwritten when its load returns)
#pragma unroll
            for (int u = 0; u < STREAMT_NPF1; ++u) async_ready<0>(it[u].r1, it[u].r3);
            BB_STREAM_TRACE(8);
        }
        // ---- inverse norms (rows past M: zero, their hidden values then are exactly zero).
        // Butterfly over the lanes: after the steps with lane bits 0..3 a lane holds one row's sum over its
        // group of 16 lanes, row = 8 b0 + 4 b1 + 2 b2 + b3 (b_k = bit k of the lane number).
        {
#pragma unroll
            for (int st = 0; st < 4; ++st) {
                const int half = 8 >> st;
                const bool up = (lane >> st) & 1;
#pragma unroll
                for (int i = 0; i < half; ++i) {
                    const float keep = up ? ssq[i + half] : ssq[i], send = up ? ssq[i] : ssq[i + half];
                    ssq[i] = keep + __shfl_xor(send, 1 << st);
                }
            }
            float v = ssq[0];
            v += __shfl_xor(v, 16);
            v += __shfl_xor(v, 32);
            const int row = 8 * (lane & 1) + 4 * ((lane >> 1) & 1) + 2 * ((lane >> 2) & 1) + ((lane >> 3) & 1);
            float* const wsum = stat + 16;                       // [4 wavefronts][16 rows]
            if (lane < 16) wsum[16 * w + row] = v;
            __syncthreads();
            if (t < 16) {
                const float q = (wsum[t] + wsum[16 + t]) + (wsum[32 + t] + wsum[48 + t]);
                stat[t] = (t < p.M) ? rsqrtf(q / (float)p.D + p.eps) : 0.f;
            }
        }
        __syncthreads();
        BB_STREAM_TRACE(1);
        // ---- the four wavefronts' partial dots -> inverse norm after the dots, Swish, gate -> hidden block
        const int nu = u1 - u0;
        for (int idx = t; idx < 16 * nu; idx += STREAMT_THREADS) {
            const int m = idx / nu, ul = idx - m * nu;
            const int gi = ul >> 4;
            const int at = ((ul & 15) + 16 * (m >> 2)) * 4 + (m & 3);     // accumulator element (row m, unit ul % 16)
            float P = 0.f, Q = 0.f;
#pragma unroll
            for (int ww = 0; ww < 4; ++ww) {
                const float* src = red + (size_t)((ww * ng + gi) * 2) * 256;
                P += src[at];
                Q += src[256 + at];
            }
            const float r = stat[m];
            const u32 hv = pack_bf16(swiglu(r * P, r * Q), 0.f) & 0xffffu;
            const int un = u0 + ul;                               // hidden unit -> block of 32 units, row m, element
            __hip_atomic_store(p.H + ((size_t)(un >> 5) * 16 + m) * 32 + (un & 31), (u16)hv, __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    BB_STREAM_TRACE(2);
    grid_arrive(p.bar, bar_base + 1u);

    // =====================  phase 2: output columns [c0, c1)  =====================
    const int c0 = min(p.D, b * p.cpw), c1 = min(p.D, c0 + p.cpw);
    const int ng2 = (c1 - c0 + 15) / 16;
    {
        const int nck2 = p.F / 8;
        const int nss2 = p.cq2 / 16;
        const int total2 = ng2 * nss2;
        // Every workgroup walks the hidden dimension from a different starting point: they all read the
        // same hidden block, and in lockstep the compute units of an XCD would ask the same L2 channel
        // for the same lines at the same time (measured: the hidden block alone then takes 16 us).
        const int rot = (b >> 3) % nss2;
        int gi_i = 0, s_i = 0, gi_h = 0, s_h = 0;
        auto issue_w = [&](StreamTItem2& r) {
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int row = c0 + 16 * gi_i + 8 * h + rn;
                const bool rv = gi_i < ng2 && row < c1;
                const int sr = s_i + rot < nss2 ? s_i + rot : s_i + rot - nss2;
                const int cc = 16 * (4 * sr + w) + 4 * hf + q4;        // chunk of instruction j: cc + 8 j
                const size_t off = (size_t)row * p.F + 8 * cc;
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    async_load16(r.r2[2 * h + j], (BB_ST_W2 && rv && cc + 8 * j < nck2) ? p.W2t + off + 64 * j : zsrc);
            }
            if (++s_i == nss2) { s_i = 0; ++gi_i; }
        };
        // hidden values of row n: h[2 j + v] = chunk 8 j + 4 v + q of the item = block (item's first block)
        // + 2 j + v, position q in the block
        auto issue_h = [&](StreamTItem2& r) {
            const int sr = s_h + rot < nss2 ? s_h + rot : s_h + rot - nss2;
            const int cc = 16 * (4 * sr + w) + q4;
            const size_t off = ((size_t)(cc >> 2) * 16 + n) * 32 + 8 * q4;
#pragma unroll
            for (int k = 0; k < 4; ++k)
                async_load16_ordered(r.h[k], (BB_ST_H && gi_h < ng2 && cc + 4 * k < nck2) ? p.H + off + 512 * k : zsrc);
            if (++s_h == nss2) { s_h = 0; ++gi_h; }
        };
        // the first weights are requested before the barrier is through: HBM stays busy
        StreamTItem2 it[STREAMT_NPF2];
#pragma unroll
        for (int u = 0; u < STREAMT_NPF2; ++u) issue_w(it[u]);
        BB_STREAM_TRACE(3);
        if (w == 0) {
            bar_poll_wave(p.bar, bar_base + 1u, p.spin_limit, p.fault);
            if (lane == 0 && b == 0)
                __hip_atomic_store(p.epoch, bar_base + 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        __syncthreads();
        if (BB_ST_FENCE) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
        BB_STREAM_TRACE(4);
#pragma unroll
        for (int u = 0; u < STREAMT_NPF2; ++u) issue_h(it[u]);

        int gi_c = 0, s_c = 0;
        f32x4 acc[2][2];
        for (int idx0 = 0; idx0 < total2; idx0 += STREAMT_NPF2) {
#pragma unroll
            for (int u = 0; u < STREAMT_NPF2; ++u) {
                if (s_c == 0) {
#pragma unroll
                    for (int h = 0; h < 2; ++h) { acc[h][0] = f32x4{0, 0, 0, 0}; acc[h][1] = f32x4{0, 0, 0, 0}; }
                }
                // Younger loads: in the first pass through the ring the hidden values of all items were
                // requested together, after all their weights: at least the 4 (NPF2 - 1) hidden loads of
                // the items behind this one; later, weights and hidden values of an item go out together.
                // (the wait alone in the branch, ONE tie after it: two ties in two branches would be joined
                // by register copies - of registers whose loads are still in flight)
                if (idx0 == 0) async_wait<4 * (STREAMT_NPF2 - 1)>();
                else async_wait<8 * (STREAMT_NPF2 - 1)>();
                async_tie(it[u].r2, it[u].h);
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    Chunk alo, ahi;
                    alo.u = it[u].h[2 * j];
                    ahi.u = it[u].h[2 * j + 1];
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        Chunk bw;
                        bw.u = it[u].r2[2 * h + j];
                        acc[h][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(alo.v, bw.v, acc[h][0], 0, 0, 0);
                        acc[h][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ahi.v, bw.v, acc[h][1], 0, 0, 0);
                    }
                }
                issue_w(it[u]);
                issue_h(it[u]);
                if (++s_c == nss2) {
                    if (gi_c < ng2)
                        *reinterpret_cast<f32x4*>(red + ((size_t)(w * ng2 + gi_c) * 64 + lane) * 4) = fold16(acc, hf);
                    s_c = 0;
                    ++gi_c;
                }
            }
        }
#pragma unroll
        for (int u = 0; u < STREAMT_NPF2; ++u) async_ready<0>(it[u].r2, it[u].h);   // (as after phase 1)
        __syncthreads();
        BB_STREAM_TRACE(5);
        const int nc = c1 - c0;
        for (int idx = t; idx < p.M * nc; idx += STREAMT_THREADS) {
            const int m = idx / nc, cl = idx - m * nc;
            const int gi = cl >> 4;
            const int at = ((cl & 15) + 16 * (m >> 2)) * 4 + (m & 3);
            float y = 0.f;
#pragma unroll
            for (int ww = 0; ww < 4; ++ww) y += red[(size_t)(ww * ng2 + gi) * 256 + at];
            const size_t o = (size_t)m * p.D + c0 + cl;
            if (p.R != nullptr) y += __uint_as_float((u32)p.R[o] << 16);
            p.Y[o] = (u16)(pack_bf16(y, 0.f) & 0xffffu);
        }
    }
    BB_STREAM_TRACE(7);
}
#endif  // BB_HOST_ONLY

}  // namespace bb
