// Weight-streaming RMSNorm -> FFN-SwiGLU kernel for few rows (decode and small batches, up to 32
// rows), row-major weights, gfx950.
//
// With so few rows the operator is a pure stream over the three weight matrices.  One persistent kernel
// (one workgroup per compute unit, all resident at once) runs the maps of Example 3's first fused
// snapshot back to back, separated by grid barriers:
//
//   phase 1 (K-map): work item = (block of 32 model channels, block of 128 hidden units).  Items are dealt
//     out evenly over the workgroups, so the reduction over the model dimension is a PARALLEL reduction
//     (Rule 3): a workgroup sums its consecutive items in registers and LDS and stores its partial
//     pre-activations (X diag(g)) W1, (X diag(g)) W3 and its partial sum x^2 in a slot of its own.
//     Wavefronts 0 and 2 stream W1, wavefronts 1 and 3 stream W3: a wavefront then holds ONE
//     16 MT x 128 accumulator tile, which leaves its registers to the queue of requests.
//   phase 1b: the (at most a few) partial sums per hidden unit are added, the inverse norm is applied
//     AFTER the dots (Rule 4), then Swish and the gate; the hidden block (16 MT x F, bf16) is written
//     once to a cache-resident scratch.
//   phase 2 (N-map): work item = (block of 32 hidden units, block of 128 output columns), again dealt
//     out evenly; partial outputs go to slots.
//   phase 2b: the workgroup that is the last to deliver its partial tile of a block of output columns
//     adds the tiles (in slot order), adds the residual and stores bf16.
//
// Rows come in groups of 16 (MT = 1 or 2 groups: one 16x16x32 matrix instruction per group and 8
// columns), so 17..32 rows stream the weights once as well.
//
// The parallel reductions use per-workgroup slots instead of atomics: fp32 atomics run at about one
// per L2 channel per clock on this part and stall the weight stream behind them (measured), plain
// stores do not.
//
// Every weight element is read from HBM exactly once, by exactly one wavefront, with 16-byte
// non-temporal loads requested several items ahead; the 8x8 in-register transposition turns them into
// matrix-instruction operands without touching LDS.  The grid barrier is a monotonically increasing
// counter in the workspace; its wait is bounded, so the kernel always terminates.
//
// Contracts this file relies on (checked by tests, not language guarantees): (1) data handed from
// one workgroup to another is written with agent-scope stores, the writer waits for their
// acknowledgement (s_waitcnt vmcnt(0)) before its relaxed agent-scope atomic on the barrier word or
// counter, and the reader sees that word through an agent-scope access before it reads the data with
// agent-scope loads; (2) vector memory operations of a wavefront complete in the order they were issued,
// so that "s_waitcnt vmcnt(N)" means "everything but the N youngest has landed"; (3) the weight stream
// is requested ahead with inline-asm loads whose destination registers the compiler must not touch
// before the matching s_waitcnt - check_inflight.py verifies that on the compiled code.
#pragma once
#include "bb_common.h"

// Optional timeline hook: a debugging build may define BB_STREAM_TRACE(slot) to
// record a timestamp per workgroup; it expands to nothing in the library.
#ifndef BB_STREAM_TRACE
#define BB_STREAM_TRACE(slot)
#endif

namespace bb {

constexpr int STREAM_THREADS = 256;
constexpr int STREAM_MAXMT = 2;      // groups of 16 rows (four need more registers than a wavefront has next to the queue)
// items (8 KiB of weights each) a wavefront keeps in flight: as many as its registers hold next to the accumulators
// A queue entry of phase 1 holds a 32 x 128 block of BOTH W1 and W3 when the wavefront accumulates both
// products (16 rows: 16 KiB of weights per load of x), of one of them when it accumulates one (32 rows).
constexpr int stream_nm(int mt) { return mt == 1 ? 2 : 1; }
constexpr int stream_np1(int mt) { return mt == 1 ? 2 : 3; }
constexpr int stream_np2(int mt) { return mt == 1 ? 6 : 4; }

struct StreamArgs {
    const u16* X;      // [M, D], M <= 16 MT
    const u16* g;      // [D]
    const u16* W1;     // [D, F]
    const u16* W3;     // [D, F]
    const u16* W2;     // [F, D]
    u16* Y;            // [M, D]
    const u16* R;      // [M, D] residual added to the output before its one rounding, or null
    float* ppart;      // [nfb][S1][MT][2][16][128] partial pre-activations (P then Q)
    float* spart;      // [S1][16 MT] partial row sums of squares
    u16* H;            // [16 MT][Fp] hidden block, bf16
    float* ypart;      // [nnb][S2][MT][16][128] partial outputs
    unsigned* cnt;     // [nnb] arrivals of partial tiles per block of output columns: zero between launches (the
                       // workgroup that sees a counter complete puts it back)
    const u16* zeros;  // 16 zero bytes in global memory: what a lane outside the matrices loads
    unsigned* bar;     // BAR_WORDS barrier words (see grid_arrive), zero before the first call
    unsigned* epoch;   // one word next to them: grid barriers completed by earlier launches (kept by the kernels)
    unsigned* fault;   // one word of host memory mapped into the device: set when a barrier's bounded wait gives up
    unsigned spin_limit;   // polls after which it gives up
    int M, D, F, Fp;
    int nkb1, nfb, items1, per1, S1;   // phase 1: D/32 blocks, F/128 blocks, items, items per workgroup, slots
    int nkb2, nnb, items2, per2, S2;   // phase 2: F/32 blocks, D/128 blocks, ...
    float eps;
};

struct StreamSmem {
    float red[4][2][16][128];   // per-wavefront partial tiles
    float ssq[4][16 * STREAM_MAXMT];
    unsigned last;              // this workgroup delivered the last partial tile of the block at hand
};

template <int MT>
struct StreamItem1 {
    u32x4 wt[stream_nm(MT)][8], rx[MT], rg;
};
template <int MT>
struct StreamItem2 {
    u32x4 w2[8], h[MT];
};

// acc[c][e] of a wavefront's 16 x 128 tile is row 4*(lane/16)+e, column 8*(lane%16)+c
__device__ __forceinline__ void stash_tile(float (*dst)[128], const f32x4 (&acc)[8], int lane) {
    const int jn = lane & 15, g4 = lane >> 4;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const f32x4 lo = {acc[0][e], acc[1][e], acc[2][e], acc[3][e]};
        const f32x4 hi = {acc[4][e], acc[5][e], acc[6][e], acc[7][e]};
        float* s = &dst[4 * g4 + e][8 * jn];
        *reinterpret_cast<f32x4*>(s) = lo;
        *reinterpret_cast<f32x4*>(s + 4) = hi;
    }
}

// sum of the four wavefronts' tiles, 4 consecutive floats starting at flat index i4*4
__device__ __forceinline__ f32x4 sum4(const float* red0, int stride, int i4) {
    const f32x4 a = *reinterpret_cast<const f32x4*>(red0 + 4 * i4);
    const f32x4 b = *reinterpret_cast<const f32x4*>(red0 + stride + 4 * i4);
    const f32x4 c = *reinterpret_cast<const f32x4*>(red0 + 2 * stride + 4 * i4);
    const f32x4 d = *reinterpret_cast<const f32x4*>(red0 + 3 * stride + 4 * i4);
    return (a + b) + (c + d);
}

// Grid barrier in two halves.  All workgroups of the grid must be resident.
// 256 simultaneous atomics and polls on ONE word serialise at its memory
// channel (measured: > 10 us), so arrivals are counted in 16 groups of
// workgroups (id mod 16), each with an arrival word; the last arriver of a
// group publishes the barrier number in the group's flag word, and a waiting
// wavefront reads all 16 flags with one load (lane j reads flag j).  The
// critical path is one returning atomic, one store and one load (a second
// counting level on top of the groups cost another atomic round trip, about
// 1 us per barrier).  Every word sits in its own 256-byte block.  All words only
// ever increase (the kernels keep the number of completed barriers next to
// them), so nothing needs resetting; the wait gives up after `spin_limit` polls
// (about two seconds by default) and then sets a word in host memory that the
// library looks at when it is called next: the launch runs to its end with an
// invalid output.  Only thread 0 signals, after the whole workgroup's stores have
// been acknowledged.
constexpr int BAR_GROUPS = 16;
constexpr int BAR_STRIDE = 64;                 // words between barrier words (256 bytes)
constexpr int BAR_WORDS = (2 * BAR_GROUPS + 2) * BAR_STRIDE;
// word layout: group arrival g -> g, (16 unused), flag g -> 17 + g (times BAR_STRIDE)

// a bounded wait has given up: tell the host (system-scope store to mapped host memory)
__device__ __forceinline__ void report_fault(unsigned* fault) {
    __hip_atomic_store(fault, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
}

// thread-level half: count this workgroup's arrival at barrier number k (>= 1)
__device__ __forceinline__ void bar_signal(unsigned* bar, unsigned k) {
    const unsigned G = gridDim.x, g = blockIdx.x % BAR_GROUPS;
    const unsigned gsize = (G - g + BAR_GROUPS - 1) / BAR_GROUPS;
    const unsigned old = __hip_atomic_fetch_add(bar + g * BAR_STRIDE, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (old + 1u == gsize * k)
        __hip_atomic_store(bar + (BAR_GROUPS + 1 + g) * BAR_STRIDE, k, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// wavefront-level half (all 64 lanes call it): wait until every group has published barrier number k (bounded)
__device__ __forceinline__ void bar_poll_wave(unsigned* bar, unsigned k, unsigned spin_limit, unsigned* fault) {
    const unsigned G = gridDim.x, ngroups = G < BAR_GROUPS ? G : BAR_GROUPS;
    const unsigned l = threadIdx.x & 63;
    unsigned spins = 0;
    while (true) {
        unsigned v = k;                        // lanes without a group count as done
        if (l < ngroups)
            v = __hip_atomic_load(bar + (BAR_GROUPS + 1 + l) * BAR_STRIDE, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (__all((int)(v - k) >= 0)) break;
        if (++spins > spin_limit) {
            if (l == 0) report_fault(fault);
            break;
        }
        __builtin_amdgcn_s_sleep(2);
    }
}
// whole workgroup: all its stores are complete, then thread 0 signals
__device__ __forceinline__ void grid_arrive(unsigned* bar, unsigned k) {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_s_waitcnt(0);                       // every store of this wavefront has been acknowledged
    __syncthreads();
    if (threadIdx.x == 0) bar_signal(bar, k);
}

// Loads the compiler does not see as loads (it would wait for ALL outstanding loads before the first use
// of any loaded register inside a loop, which empties the queue at every item): an asm load leaves its
// destination registers "in flight"; stream_ready() is the one place where the wavefront waits until at
// most N younger loads are outstanding, and it takes the registers as in-out operands, so that every use
// is ordered after the wait.  The destination is an in-out operand of the load too: a queue entry then is
// one chain of tied operands from request to wait to the next request, which pins it to one set of
// registers.  The queue lives in ACCUMULATION registers (the load instructions write them directly): the
// compiler never picks those as spill candidates, whereas a queue in ordinary vector registers is the
// first thing it moves out of the way when the registers run short - while the loads are in flight.
// Weights are streamed once: non-temporal.
__device__ __forceinline__ void stream_load16_nt(u32x4& dst, const u16* src) {
    asm volatile("global_load_dwordx4 %0, %1, off nt" : "+a"(dst) : "v"(src));
}
__device__ __forceinline__ void stream_load16(u32x4& dst, const u16* src) {
    asm volatile("global_load_dwordx4 %0, %1, off" : "+a"(dst) : "v"(src));
}
// data another workgroup wrote during this launch: agent scope, never a stale cached copy
__device__ __forceinline__ void stream_load16_coherent(u32x4& dst, const u16* src) {
    asm volatile("global_load_dwordx4 %0, %1, off sc1" : "+a"(dst) : "v"(src) : "memory");
}
template <int N>
__device__ __forceinline__ void stream_wait8(u32x4 (&r)[8]) {
    asm volatile("s_waitcnt vmcnt(%8)"
                 : "+a"(r[0]), "+a"(r[1]), "+a"(r[2]), "+a"(r[3]), "+a"(r[4]), "+a"(r[5]), "+a"(r[6]), "+a"(r[7])
                 : "n"(N));
}
template <int N, int MT>
__device__ __forceinline__ void stream_ready(StreamItem1<MT>& r) {
    stream_wait8<N>(r.wt[0]);
    if constexpr (stream_nm(MT) == 2) stream_wait8<N>(r.wt[1]);
#pragma unroll
    for (int m = 0; m < MT; ++m) asm volatile("" : "+a"(r.rx[m]));
    asm volatile("" : "+a"(r.rg));
}
template <int N, int MT>
__device__ __forceinline__ void stream_ready(StreamItem2<MT>& r) {
    stream_wait8<N>(r.w2);
#pragma unroll
    for (int m = 0; m < MT; ++m) asm volatile("" : "+a"(r.h[m]));
}

#ifndef BB_HOST_ONLY   // (bb_api.hip includes this file for the argument structures only)
template <int MT>
__global__ __launch_bounds__(STREAM_THREADS) void ffn_stream_kernel(const StreamArgs p) {
    __shared__ StreamSmem sm;
    constexpr int NP1 = stream_np1(MT), NP2 = stream_np2(MT);
    constexpr int NM = stream_nm(MT);              // matrices a wavefront streams in phase 1
    constexpr int WPI = 2 * NM;                    // wavefronts that share the workgroup's items of a matrix
    constexpr int LOADS1 = 8 * NM + MT + 1, LOADS2 = 8 + MT;     // load instructions per item
    constexpr int RS = 2 * 16 * 128;               // floats of a partial tile of pre-activations (P, Q)
    const int t = threadIdx.x, lane = t & 63;
    const int w = __builtin_amdgcn_readfirstlane(t >> 6);        // in a scalar register: branches on it are scalar
    const int jn = lane & 15, g4 = lane >> 4;
    const int G = gridDim.x, b = blockIdx.x;

    // Grid barriers completed before this launch: the barrier words only ever increase, and the count
    // lives in device memory (workgroup 0 advances it at the end), so the host keeps no state per
    // launch and a launch may be replayed from a captured graph.  Every workgroup reads it before its
    // first arrival; workgroup 0 writes it after the last barrier, i.e. after every arrival.
    const unsigned bar_base =
        __builtin_amdgcn_readfirstlane(__hip_atomic_load(p.epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));

    BB_STREAM_TRACE(0);
    // =====================  phase 1: partial pre-activations  =====================
    {
        // The workgroup's items [i0, i0 + n) lie in one or more blocks of 128 hidden units ("segments", each
        // with its own partial tile and slot).  Wavefronts 0 and 2 stream W1 (their tiles are P), 1 and 3
        // stream W3 (Q); each pair takes the items alternately as ONE stream: the request queue runs on
        // across a segment boundary (draining and refilling it there cost the workgroups with a boundary
        // 3-6 us; they were the last to reach the barrier).  Every wavefront takes part in the flush of
        // every segment, with zeros if it had no item there.
        const int i0 = min(b * p.per1, p.items1);
        const int n = min(i0 + p.per1, p.items1) - i0;
        if (n > 0) {
            const int f0 = i0 / p.nkb1;
            const int nseg = (i0 + n - 1) / p.nkb1 - f0 + 1;
            // NM == 2: every wavefront streams W1 and W3 and takes every fourth item; NM == 1: wavefronts 0 and 2
            // stream W1 (their tiles are P), 1 and 3 stream W3 (Q), each pair takes the items alternately.
            const bool isQ = NM == 1 && (w & 1) != 0;
            const int wv0 = NM == 2 ? w : (w >> 1);
            f32x4 acc[NM][MT][8];
            float ssq[MT];
#pragma unroll
            for (int m = 0; m < MT; ++m) {
                ssq[m] = 0.f;
#pragma unroll
                for (int a = 0; a < NM; ++a)
#pragma unroll
                    for (int c = 0; c < 8; ++c) acc[a][m][c] = f32x4{0, 0, 0, 0};
            }
            StreamItem1<MT> it[NP1];
            int segof[NP1];                        // segment of the item in queue entry u
#pragma unroll
            for (int u = 0; u < NP1; ++u) {
#pragma unroll
                for (int a = 0; a < NM; ++a)
#pragma unroll
                    for (int i = 0; i < 8; ++i) it[u].wt[a][i] = zero4();
#pragma unroll
                for (int m = 0; m < MT; ++m) it[u].rx[m] = zero4();
                it[u].rg = zero4();
                segof[u] = 0;
            }
            // position v of the workgroup's share -> where its operands lie.  Every load is unconditional: a
            // lane outside the matrices or past the last item reads the zero chunk, so no load stands inside a
            // branch.  Returns the item's segment.
            auto issue = [&](int v, StreamItem1<MT>& r) -> int {
                const bool live = v < n;
                const int j = i0 + v;
                const int fb = j / p.nkb1, kb = j - fb * p.nkb1;
                const int col = 128 * fb + 8 * jn;
                const int d0 = 32 * kb + 8 * g4;
                const bool col_ok = live && col < p.F;
#pragma unroll
                for (int a = 0; a < NM; ++a) {
                    const u16* Wm = (NM == 2 ? a == 1 : isQ) ? p.W3 : p.W1;
#pragma unroll
                    for (int i = 0; i < 8; ++i)
                        stream_load16_nt(r.wt[a][i], (col_ok && d0 + i < p.D) ? Wm + (size_t)(d0 + i) * p.F + col : p.zeros);
                }
                const bool ok = live && d0 < p.D;
#pragma unroll
                for (int m = 0; m < MT; ++m)
                    stream_load16(r.rx[m], (ok && jn + 16 * m < p.M) ? p.X + (size_t)(jn + 16 * m) * p.D + d0 : p.zeros);
                stream_load16(r.rg, ok ? p.g + d0 : p.zeros);
                return fb - f0;
            };
            // adds the wavefronts' tiles of segment k in LDS, stores the workgroup's partial tile in its slot,
            // and clears the accumulators (the stores only add to the count the waits look at: they wait longer)
            auto flush = [&](int k) {
                const int fb = f0 + k;
                const int slot = b - (fb * p.nkb1) / p.per1;
                float* dst = p.ppart + (size_t)(fb * p.S1 + slot) * (MT * RS);
#pragma unroll
                for (int m = 0; m < MT; ++m) {
#pragma unroll
                    for (int a = 0; a < NM; ++a) {
                        stash_tile(sm.red[w][a], acc[a][m], lane);
#pragma unroll
                        for (int c = 0; c < 8; ++c) acc[a][m][c] = f32x4{0, 0, 0, 0};
                    }
                    float s = isQ ? 0.f : ssq[m];
                    s += __shfl_xor(s, 16);
                    s += __shfl_xor(s, 32);
                    if (lane < 16) sm.ssq[w][16 * m + lane] = s;
                    ssq[m] = 0.f;
                    __syncthreads();
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const int i4 = t + STREAM_THREADS * j;        // float4 index in [2][16][128]
                        f32x4 v;
                        if (NM == 2) {
                            v = sum4(&sm.red[0][0][0][0], RS, i4);
                        } else {            // P: wavefronts 0 and 2, Q: wavefronts 1 and 3
                            const int which = i4 >> 9, idx = 4 * (i4 & 511);
                            v = *reinterpret_cast<const f32x4*>(&sm.red[which][0][0][0] + idx) +
                                *reinterpret_cast<const f32x4*>(&sm.red[which + 2][0][0][0] + idx);
                        }
                        cstore16f(dst + m * RS + 4 * i4, v);
                    }
                    // sum x^2 is counted once per model channel: by the items of hidden block 0
                    if (fb == 0 && t < 16 && m == MT - 1) {
#pragma unroll
                        for (int mm = 0; mm < MT; ++mm)
                            __hip_atomic_store(p.spart + slot * (16 * MT) + 16 * mm + t,
                                               (sm.ssq[0][16 * mm + t] + sm.ssq[1][16 * mm + t]) +
                                                   (sm.ssq[2][16 * mm + t] + sm.ssq[3][16 * mm + t]),
                                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    }
                    __syncthreads();
                }
            };

            int cur_seg = 0;
#pragma unroll
            for (int u = 0; u < NP1; ++u) segof[u] = issue(wv0 + WPI * u, it[u]);
            for (int v0 = wv0; v0 < n; v0 += WPI * NP1) {
#pragma unroll
                for (int u = 0; u < NP1; ++u) {
                    const int v = v0 + WPI * u;
                    if (v < n)
                        while (cur_seg < segof[u]) flush(cur_seg++);     // (past the last item the entry is all zeros)
                    stream_ready<LOADS1 * (NP1 - 1), MT>(it[u]);
                    // consume the registers of the item, then request the next one into them
                    Chunk xa[MT];
#pragma unroll
                    for (int m = 0; m < MT; ++m) {
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            const float x0 = bf_lo(it[u].rx[m][q]), x1 = bf_hi(it[u].rx[m][q]);
                            ssq[m] = fmaf(x0, x0, ssq[m]);
                            ssq[m] = fmaf(x1, x1, ssq[m]);
                            xa[m].u[q] = pack_bf16(x0 * bf_lo(it[u].rg[q]), x1 * bf_hi(it[u].rg[q]));
                        }
                    }
#pragma unroll
                    for (int a = 0; a < NM; ++a) {
                        u32x4 tt[8];
                        transpose8x8(it[u].wt[a], tt);
                        if (a == NM - 1) segof[u] = issue(v + WPI * NP1, it[u]);
#pragma unroll
                        for (int c = 0; c < 8; ++c) {
                            Chunk bw;
                            bw.u = tt[c];
#pragma unroll
                            for (int m = 0; m < MT; ++m)
                                acc[a][m][c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xa[m].v, bw.v, acc[a][m][c], 0, 0, 0);
                        }
                    }
                }
            }
            // the requests past the last item are still in flight: their registers stay reserved until they
            // have landed (a register reused earlier would be overwritten when its load returns)
#pragma unroll
            for (int u = 0; u < NP1; ++u) stream_ready<0, MT>(it[u]);
            BB_STREAM_TRACE(1);
            while (cur_seg < nseg) flush(cur_seg++);
        }
    }

    BB_STREAM_TRACE(2);
    grid_arrive(p.bar, bar_base + 1u);

    // ---- phase 2 work of this workgroup: positions [i2, iend2) of the (block of output columns, block of
    // 32 hidden units) items.  Wavefronts 1..3 request the weight blocks of their first items now, so HBM
    // stays busy while wavefront 0 runs the short synchronised part (barrier, hidden block, barrier) with
    // nothing in flight that it would have to wait for.
    const int i2 = min(b * p.per2, p.items2);
    const int iend2 = min(i2 + p.per2, p.items2);
    StreamItem2<MT> it2[NP2];
#pragma unroll
    for (int u = 0; u < NP2; ++u) {
#pragma unroll
        for (int i = 0; i < 8; ++i) it2[u].w2[i] = zero4();
#pragma unroll
        for (int m = 0; m < MT; ++m) it2[u].h[m] = zero4();
    }
    // item v of the segment that starts at position q (block nb, first hidden block kb0, nit items)
    auto issue2_w = [&](int nb, int kb0, int nit, int v, StreamItem2<MT>& r) {
        const int col = 128 * nb + 8 * jn;
        const int k0 = 32 * (kb0 + v) + 8 * g4;
        const bool ok = v < nit && col < p.D;
#pragma unroll
        for (int i = 0; i < 8; ++i)
            stream_load16_nt(r.w2[i], (ok && k0 + i < p.F) ? p.W2 + (size_t)(k0 + i) * p.D + col : p.zeros);
    };
    auto issue2_h = [&](int kb0, int nit, int v, StreamItem2<MT>& r) {
        const int k0 = 32 * (kb0 + v) + 8 * g4;
#pragma unroll
        for (int m = 0; m < MT; ++m)
            stream_load16_coherent(r.h[m], v < nit ? p.H + (size_t)(jn + 16 * m) * p.Fp + k0 : p.zeros);
    };
    const int nb_first = i2 / p.nkb2, kb_first = i2 - nb_first * p.nkb2;
    const int nit_first = min(p.nkb2 - kb_first, iend2 - i2);        // (<= 0: no work)
    // (ONE place where the requests are made, after a branch that only wavefront 0 takes: two places would be
    // two sets of registers that the compiler joins with copies - of registers whose loads are in flight)
    if (w == 0) {
        BB_STREAM_TRACE(3);
        bar_poll_wave(p.bar, bar_base + 1u, p.spin_limit, p.fault);
        BB_STREAM_TRACE(4);
        // =====================  phase 1b: hidden block  =====================
        const int groups_per_row = p.Fp / 8;                   // tasks: (row, 8 consecutive hidden units)
        const int total = 16 * MT * groups_per_row;
        const int slots0 = min(G - 1, (p.nkb1 - 1) / p.per1) + 1;   // workgroups that saw hidden block 0
        const float invD = 1.0f / (float)p.D;
        // two tasks per lane and turn, so that all their loads are in flight together
        for (int idx0 = b * 128 + lane; idx0 < total; idx0 += G * 128) {
            f32x4 acc[2][4];
            float ss[2];
            int rowv[2], f0v[2];
            bool live[2];
#pragma unroll
            for (int k = 0; k < 2; ++k) {
                const int idx = idx0 + 64 * k;
                live[k] = idx < total;
                const int row = live[k] ? idx / groups_per_row : 0, f0 = live[k] ? 8 * (idx % groups_per_row) : 0;
                rowv[k] = row;
                f0v[k] = f0;
                const int fb = f0 >> 7, cc = f0 & 127;
                const int first = (fb * p.nkb1) / p.per1;
                const int ns = live[k] ? min(G - 1, ((fb + 1) * p.nkb1 - 1) / p.per1) - first + 1 : 0;
                const int nsq = live[k] ? slots0 : 0;
                const float* src0 = p.ppart + (size_t)fb * p.S1 * (MT * RS) + (row >> 4) * RS + (row & 15) * 128 + cc;
                const f32x4 z = {0, 0, 0, 0};
                acc[k][0] = z; acc[k][1] = z; acc[k][2] = z; acc[k][3] = z;
                ss[k] = 0.f;
                for (int s0 = 0; s0 < max(ns, nsq); s0 += 4) {   // four slots' loads in flight together
                    f32x4 v[4][4];
                    float sq[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const float* src = src0 + (size_t)(s0 + u) * (MT * RS);
                        const bool ok = s0 + u < ns;
                        v[u][0] = ok ? cload16f(src) : z;
                        v[u][1] = ok ? cload16f(src + 4) : z;
                        v[u][2] = ok ? cload16f(src + 2048) : z;
                        v[u][3] = ok ? cload16f(src + 2048 + 4) : z;
                        sq[u] = (s0 + u < nsq) ? cload4f(p.spart + (s0 + u) * (16 * MT) + row) : 0.f;
                    }
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        acc[k][0] += v[u][0]; acc[k][1] += v[u][1]; acc[k][2] += v[u][2]; acc[k][3] += v[u][3];
                        ss[k] += sq[u];
                    }
                }
            }
#pragma unroll
            for (int k = 0; k < 2; ++k) {
                if (!live[k]) continue;
                const float rinv = (rowv[k] < p.M) ? rsqrtf(ss[k] * invD + p.eps) : 0.f;   // rows past M stay exactly zero
                const f32x4 P0 = acc[k][0], P1 = acc[k][1], Q0 = acc[k][2], Q1 = acc[k][3];
                u32x4 h;
#pragma unroll
                for (int q = 0; q < 2; ++q) {
                    h[q] = pack_bf16(swiglu(rinv * P0[2 * q], rinv * Q0[2 * q]),
                                     swiglu(rinv * P0[2 * q + 1], rinv * Q0[2 * q + 1]));
                    h[q + 2] = pack_bf16(swiglu(rinv * P1[2 * q], rinv * Q1[2 * q]),
                                         swiglu(rinv * P1[2 * q + 1], rinv * Q1[2 * q + 1]));
                }
                u16* hd = p.H + (size_t)rowv[k] * p.Fp + f0v[k];
                cstore8(hd, h[0], h[1]);
                cstore8(hd + 4, h[2], h[3]);
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        __builtin_amdgcn_s_waitcnt(0);                    // this wavefront's hidden stores are complete
        BB_STREAM_TRACE(8);
        if (lane == 0) bar_signal(p.bar, bar_base + 2u);
        bar_poll_wave(p.bar, bar_base + 2u, p.spin_limit, p.fault);
        if (lane == 0 && b == 0)       // (every workgroup read the count before its first arrival)
            __hip_atomic_store(p.epoch, bar_base + 2u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
#pragma unroll
    for (int u = 0; u < NP2; ++u) issue2_w(nb_first, kb_first, nit_first, w + 4 * u, it2[u]);
    __syncthreads();
    BB_STREAM_TRACE(5);

    // =====================  phase 2: partial outputs  =====================
    {
        // one segment = one block of 128 output columns; `first`: the segment whose first weight blocks were
        // requested before the barrier.  (The first segment is not the first trip of a loop over segments: the
        // requests in flight would then enter the loop through copies of their registers.)
        auto segment = [&](int i, const bool first) -> int {
            const int nb = i / p.nkb2, kb0 = i - nb * p.nkb2;
            const int nit = min(p.nkb2 - kb0, iend2 - i);
            const int slot = b - (nb * p.nkb2) / p.per2;
            f32x4 acc[MT][8];
#pragma unroll
            for (int m = 0; m < MT; ++m)
#pragma unroll
                for (int c = 0; c < 8; ++c) acc[m][c] = f32x4{0, 0, 0, 0};
            // the queue's first items: of the first segment the weight blocks are on their way (or here) since
            // before the barrier; their hidden fragments are requested behind ALL of them, not item by item, so
            // the counts of the waits in the loop do not hold yet: one full wait
            if (first) {
#pragma unroll
                for (int u = 0; u < NP2; ++u) issue2_h(kb0, nit, w + 4 * u, it2[u]);
#pragma unroll
                for (int u = 0; u < NP2; ++u) stream_ready<0, MT>(it2[u]);
            } else {
#pragma unroll
                for (int u = 0; u < NP2; ++u) {
                    issue2_w(nb, kb0, nit, w + 4 * u, it2[u]);
                    issue2_h(kb0, nit, w + 4 * u, it2[u]);
                }
            }
            for (int v0 = w; v0 < nit; v0 += 4 * NP2) {
#pragma unroll
                for (int u = 0; u < NP2; ++u) {
                    const int v = v0 + 4 * u;
                    stream_ready<LOADS2 * (NP2 - 1), MT>(it2[u]);
                    Chunk ha[MT];
#pragma unroll
                    for (int m = 0; m < MT; ++m) {
                        // (a value of its own in vector registers: the queue entry's old contents must be dead
                        // before the entry is requested again, or the compiler keeps both alive with copies)
                        u32x4 hv = it2[u].h[m];
                        asm volatile("" : "+v"(hv));
                        ha[m].u = hv;
                    }
                    u32x4 tt[8];
                    transpose8x8(it2[u].w2, tt);
                    issue2_w(nb, kb0, nit, v + 4 * NP2, it2[u]);
                    issue2_h(kb0, nit, v + 4 * NP2, it2[u]);
#pragma unroll
                    for (int c = 0; c < 8; ++c) {
                        Chunk bw;
                        bw.u = tt[c];
#pragma unroll
                        for (int m = 0; m < MT; ++m)
                            acc[m][c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ha[m].v, bw.v, acc[m][c], 0, 0, 0);
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < NP2; ++u) stream_ready<0, MT>(it2[u]);
            if (nit <= 0) return iend2;            // (no work at all)
            // ---- the workgroup's partial tile of the block -> its slot
            float* dst = p.ypart + (size_t)(nb * p.S2 + slot) * (MT * 2048);
#pragma unroll
            for (int m = 0; m < MT; ++m) {
                stash_tile(sm.red[w][0], acc[m], lane);
                __syncthreads();
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    const int i4 = t + STREAM_THREADS * j;        // float4 index in [16][128]
                    cstore16f(dst + m * 2048 + 4 * i4, sum4(&sm.red[0][0][0][0], RS, i4));
                }
                __syncthreads();
            }
            // ---- phase 2b.  The partial tile is complete in memory (stores acknowledged), then thread 0
            // counts the delivery; the workgroup whose delivery is the last one of the block adds the
            // tiles of all slots in slot order (so the result does not depend on who is last), adds
            // the residual and stores the block's output.  No grid barrier.
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
            __builtin_amdgcn_s_waitcnt(0);
            __syncthreads();
            const int firstwg = (nb * p.nkb2) / p.per2;
            const int ns = min(G - 1, ((nb + 1) * p.nkb2 - 1) / p.per2) - firstwg + 1;      // slots of this block
            if (t == 0) {
                const unsigned old = __hip_atomic_fetch_add(p.cnt + nb, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                const bool last = old + 1u == (unsigned)ns;
                if (last) __hip_atomic_store(p.cnt + nb, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                sm.last = last ? 1u : 0u;
            }
            __syncthreads();
            if (sm.last) {
#pragma unroll
                for (int m = 0; m < MT; ++m) {
                    const int row = 16 * m + (t >> 4), cc = 8 * (t & 15);   // task: (row, 8 consecutive columns of the block)
                    const int c0 = 128 * nb + cc;
                    if (row < p.M && c0 < p.D) {
                        const float* src0 = p.ypart + (size_t)nb * p.S2 * (MT * 2048) + m * 2048 + (t >> 4) * 128 + cc;
                        f32x4 y0 = {0, 0, 0, 0}, y1 = y0;
                        for (int s0 = 0; s0 < ns; s0 += 8) {              // eight slots' loads in flight together
                            f32x4 v[8][2];
#pragma unroll
                            for (int u = 0; u < 8; ++u) {
                                const float* src = src0 + (size_t)(s0 + u) * (MT * 2048);
                                const bool ok = s0 + u < ns;
                                const f32x4 z = {0, 0, 0, 0};
                                v[u][0] = ok ? cload16f(src) : z;
                                v[u][1] = ok ? cload16f(src + 4) : z;
                            }
#pragma unroll
                            for (int u = 0; u < 8; ++u) { y0 += v[u][0]; y1 += v[u][1]; }
                        }
                        if (p.R != nullptr) {
                            const u32x4 rr = ldg16(p.R + (size_t)row * p.D + c0);
                            y0 += f32x4{bf_lo(rr[0]), bf_hi(rr[0]), bf_lo(rr[1]), bf_hi(rr[1])};
                            y1 += f32x4{bf_lo(rr[2]), bf_hi(rr[2]), bf_lo(rr[3]), bf_hi(rr[3])};
                        }
                        const u32x4 o = {pack_bf16(y0[0], y0[1]), pack_bf16(y0[2], y0[3]), pack_bf16(y1[0], y1[1]),
                                         pack_bf16(y1[2], y1[3])};
                        *reinterpret_cast<u32x4*>(p.Y + (size_t)row * p.D + c0) = o;
                    }
                }
            }
            __syncthreads();
            return i + nit;
        };
        // (a workgroup without work in this phase runs the first segment's queue too, on zero chunks: what it
        // requested before the barrier lands there, on the one path every wavefront takes)
        int i = segment(i2, true);
        while (i < iend2) i = segment(i, false);
    }
    BB_STREAM_TRACE(7);
}
#endif  // BB_HOST_ONLY

}  // namespace bb
