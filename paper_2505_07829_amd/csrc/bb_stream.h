// Weight-streaming RMSNorm -> FFN-SwiGLU kernel for few rows (decode), gfx950.
//
// With at most 16 rows the operator is a pure stream over the three weight
// matrices.  One persistent kernel (one workgroup per compute unit, all
// resident at once) runs the maps of Example 3's first fused snapshot back to
// back, separated by grid barriers:
//
//   phase 1 (K-map): work item = (block of 32 model channels, block of 128
//     hidden units).  Items are dealt out evenly over the workgroups, so the
//     reduction over the model dimension is a PARALLEL reduction (Rule 3): a
//     workgroup sums its consecutive items in registers and LDS and stores its
//     partial pre-activations (X diag(g)) W1, (X diag(g)) W3 and its partial
//     sum x^2 in a slot of its own.
//   phase 1b: the (at most a few) partial sums per hidden unit are added, the
//     inverse norm is applied AFTER the dots (Rule 4), then Swish and the
//     gate; the hidden block (16 x F, bf16) is written once to a cache-
//     resident scratch.
//   phase 2 (N-map): work item = (block of 32 hidden units, block of 128
//     output columns), again dealt out evenly; partial outputs go to slots.
//   phase 2b: the workgroup that is the last to deliver its partial tile of a
//     block of output columns adds the tiles (in slot order) and stores bf16.
//
// The parallel reductions use per-workgroup slots instead of atomics: fp32
// atomics run at about one per L2 channel per clock on this part and stall the
// weight stream behind them (measured), plain stores do not.  No scratch needs
// to be zero on entry except the barrier word.
//
// Every weight element is read from HBM exactly once, by exactly one
// wavefront, with 16-byte loads; the 8x8 in-register transposition turns them
// into matrix-instruction operands without touching LDS.  The grid barrier is
// a monotonically increasing counter in the workspace; its wait is bounded, so
// the kernel always terminates.
//
// Contracts this file relies on (both checked by tests, neither a language
// guarantee): (1) data handed from one workgroup to another is written with
// agent-scope stores, the writer waits for their acknowledgement
// (s_waitcnt vmcnt(0)) before its relaxed agent-scope atomic on the barrier
// word, and the reader polls the flag with agent-scope loads before it reads the
// data with agent-scope loads; (2) the weight stream is requested ahead with
// inline-asm loads whose destination registers the compiler must not touch
// before the matching s_waitcnt - check_inflight.py verifies that on the
// compiled code.
#pragma once
#include "bb_common.h"

// Optional timeline hook: a debugging build may define BB_STREAM_TRACE(slot) to
// record a timestamp per workgroup; it expands to nothing in the library.
#ifndef BB_STREAM_TRACE
#define BB_STREAM_TRACE(slot)
#endif

namespace bb {

constexpr int STREAM_THREADS = 256;

struct StreamArgs {
    const u16* X;      // [M, D], M <= 16
    const u16* g;      // [D]
    const u16* W1;     // [D, F]
    const u16* W3;     // [D, F]
    const u16* W2;     // [F, D]
    u16* Y;            // [M, D]
    const u16* R;      // [M, D] residual added to the output before its one rounding, or null
    float* ppart;      // [nfb][S1][2][16][128] partial pre-activations (P then Q)
    float* spart;      // [S1][16] partial row sums of squares
    u16* H;            // [16][Fp] hidden block, bf16
    float* ypart;      // [nnb][S2][16][128] partial outputs
    unsigned* cnt;     // [nnb] arrival counters of the output blocks (any initial values: used relative to their
                       // value at the start of the launch)
    const u16* zeros;  // 16 zero bytes in global memory: what a lane outside the matrices loads in phase 1
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
    unsigned segbase[64];       // arrival counters of this workgroup's output blocks at the start of the launch
    unsigned last;              // this workgroup delivered the last partial tile of the block at hand
};

// loads the 8 rows x 8 columns block of a row-major matrix this lane owns
__device__ __forceinline__ void load_block(const u16* base, int ld, int row0, int nrows, int col,
                                           bool col_ok, u32x4 (&r)[8]) {
#pragma unroll
    for (int i = 0; i < 8; ++i)
        r[i] = (col_ok && row0 + i < nrows) ? ldg16(base + (size_t)(row0 + i) * ld + col) : zero4();
}

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

constexpr int STREAM_NP1 = 2;   // phase 1 items (16 KiB each) a wavefront keeps in flight
constexpr int STREAM_NP2 = 6;   // phase 2 items (8 KiB each) a wavefront keeps in flight

struct StreamItem1 {
    u32x4 r1[8], r3[8], rx, rg;
};

// Phase 1 requests its weights STREAM_NP1 items ahead with loads the compiler does not see as
// loads (it waits for ALL outstanding loads before the first use of any loaded register inside
// a loop, which empties the queue at every item): an asm load leaves its destination registers
// "in flight"; stream_ready() is the one place where the wavefront waits until at most N younger
// loads are outstanding, and it takes the registers as in-out operands, so that every use is
// ordered after the wait.  Vector memory loads of a wavefront return in order.  Weights are
// streamed once: non-temporal.
__device__ __forceinline__ void stream_load16_nt(u32x4& dst, const u16* src) {
    asm volatile("global_load_dwordx4 %0, %1, off nt" : "=v"(dst) : "v"(src));
}
__device__ __forceinline__ void stream_load16(u32x4& dst, const u16* src) {
    asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(dst) : "v"(src));
}
template <int N>
__device__ __forceinline__ void stream_ready(StreamItem1& r) {
    asm volatile("s_waitcnt vmcnt(%8)"
                 : "+v"(r.r1[0]), "+v"(r.r1[1]), "+v"(r.r1[2]), "+v"(r.r1[3]), "+v"(r.r1[4]), "+v"(r.r1[5]),
                   "+v"(r.r1[6]), "+v"(r.r1[7])
                 : "n"(N));
    asm volatile(""
                 : "+v"(r.r3[0]), "+v"(r.r3[1]), "+v"(r.r3[2]), "+v"(r.r3[3]), "+v"(r.r3[4]), "+v"(r.r3[5]),
                   "+v"(r.r3[6]), "+v"(r.r3[7]));
    asm volatile("" : "+v"(r.rx), "+v"(r.rg));
}
constexpr int STREAM_ITEM1_LOADS = 18;

#ifndef BB_HOST_ONLY   // (bb_api.hip includes this file for the argument structures only)
__global__ __launch_bounds__(STREAM_THREADS) void ffn_stream_kernel(const StreamArgs p) {
    __shared__ StreamSmem sm;
    const int t = threadIdx.x, lane = t & 63;
    const int w = __builtin_amdgcn_readfirstlane(t >> 6);        // in a scalar register: branches on it are scalar
    const int jn = lane & 15, g4 = lane >> 4;
    const int G = gridDim.x, b = blockIdx.x;
    constexpr int RS = 2 * 16 * 128;               // floats per wavefront in sm.red

    // Grid barriers completed before this launch: the barrier words only ever increase, and the count
    // lives in device memory (workgroup 0 advances it at the end), so the host keeps no state per
    // launch and a launch may be replayed from a captured graph.  Every workgroup reads it before its
    // first arrival; workgroup 0 writes it after the last barrier, i.e. after every arrival.
    const unsigned bar_base =
        __builtin_amdgcn_readfirstlane(__hip_atomic_load(p.epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));

    BB_STREAM_TRACE(0);
    // =====================  phase 1: partial pre-activations  =====================
    {
        // The workgroup's items [i0, iend) lie in one or more blocks of 128 hidden units ("segments", each
        // with its own partial tile and slot).  Wavefront w takes items i0 + w, i0 + w + 4, ... as ONE stream:
        // the request queue runs on across a segment boundary (draining and refilling it there cost the
        // workgroups with a boundary 3-6 us; they were the last to reach the barrier).  Every wavefront takes
        // part in the flush of every segment, with zeros if it had no item there.
        const int i0 = b * p.per1;
        const int iend = min(i0 + p.per1, p.items1);
        if (i0 < iend) {
            const int fb_last = (iend - 1) / p.nkb1;
            int cur_fb = i0 / p.nkb1;
            f32x4 accP[8], accQ[8];
#pragma unroll
            for (int c = 0; c < 8; ++c) { accP[c] = f32x4{0, 0, 0, 0}; accQ[c] = f32x4{0, 0, 0, 0}; }
            float ssq = 0.f;
            StreamItem1 it[STREAM_NP1];
            // (every load is unconditional: a lane outside the matrices or past the last item reads the
            // zero chunk instead, so no load stands inside a branch)
            auto issue = [&](int id, StreamItem1& r) {
                const bool live = id < iend;
                const int fb = id / p.nkb1, kb = id - fb * p.nkb1;
                const int col = 128 * fb + 8 * jn;
                const bool col_ok = col < p.F;
                const int d0 = 32 * kb + 8 * g4;
#pragma unroll
                for (int i2 = 0; i2 < 8; ++i2) {
                    const bool ok = col_ok && live && d0 + i2 < p.D;
                    const size_t off = (size_t)(d0 + i2) * p.F + col;
                    stream_load16_nt(r.r1[i2], ok ? p.W1 + off : p.zeros);
                    stream_load16_nt(r.r3[i2], ok ? p.W3 + off : p.zeros);
                }
                const bool ok = live && d0 < p.D;
                stream_load16(r.rx, (ok && jn < p.M) ? p.X + (size_t)jn * p.D + d0 : p.zeros);
                stream_load16(r.rg, ok ? p.g + d0 : p.zeros);
            };
            // adds the 4 wavefronts' tiles of segment fb in LDS, stores the workgroup's partial tile in its
            // slot, and clears the accumulators
            auto flush = [&](int fb) {
                const int slot = b - (fb * p.nkb1) / p.per1;
                stash_tile(sm.red[w][0], accP, lane);
                stash_tile(sm.red[w][1], accQ, lane);
                __syncthreads();
                float* dst = p.ppart + (size_t)(fb * p.S1 + slot) * RS;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int i4 = t + STREAM_THREADS * j;        // float4 index in [2][16][128]
                    cstore16f(dst + 4 * i4, sum4(&sm.red[0][0][0][0], RS, i4));
                }
                if (fb == 0) {   // sum x^2 is counted once per model channel: by the items of hidden block 0
                    ssq += __shfl_xor(ssq, 16);
                    ssq += __shfl_xor(ssq, 32);
                    __syncthreads();
                    if (lane < 16) sm.red[w][0][0][lane] = ssq;
                    __syncthreads();
                    if (t < 16)
                        __hip_atomic_store(p.spart + slot * 16 + t,
                                           sm.red[0][0][0][t] + sm.red[1][0][0][t] + sm.red[2][0][0][t] + sm.red[3][0][0][t],
                                           __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
                __syncthreads();
#pragma unroll
                for (int c = 0; c < 8; ++c) { accP[c] = f32x4{0, 0, 0, 0}; accQ[c] = f32x4{0, 0, 0, 0}; }
                ssq = 0.f;
            };
#pragma unroll
            for (int u = 0; u < STREAM_NP1; ++u) issue(i0 + w + 4 * u, it[u]);
            for (int id0 = i0 + w; id0 < iend; id0 += 4 * STREAM_NP1) {
#pragma unroll
                for (int u = 0; u < STREAM_NP1; ++u) {
                    // (past the last item the item is all zeros and adds nothing)
                    const int id = id0 + 4 * u;
                    if (id < iend) {
                        const int fbi = id / p.nkb1;
                        while (cur_fb < fbi) flush(cur_fb++);     // (the stores of a flush only add to the count
                    }                                             //  the wait below looks at: it waits longer)
                    stream_ready<STREAM_ITEM1_LOADS * (STREAM_NP1 - 1)>(it[u]);
                    // consume the registers of the item, then refill them
                    Chunk xa;
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const float x0 = bf_lo(it[u].rx[q]), x1 = bf_hi(it[u].rx[q]);
                        ssq = fmaf(x0, x0, ssq);
                        ssq = fmaf(x1, x1, ssq);
                        xa.u[q] = pack_bf16(x0 * bf_lo(it[u].rg[q]), x1 * bf_hi(it[u].rg[q]));
                    }
                    u32x4 t1[8], t3[8];
                    transpose8x8(it[u].r1, t1);
                    transpose8x8(it[u].r3, t3);
                    issue(id + 4 * STREAM_NP1, it[u]);
#pragma unroll
                    for (int c = 0; c < 8; ++c) {
                        Chunk b1, b3;
                        b1.u = t1[c];
                        b3.u = t3[c];
                        accP[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xa.v, b1.v, accP[c], 0, 0, 0);
                        accQ[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xa.v, b3.v, accQ[c], 0, 0, 0);
                    }
                }
            }
            // the requests past the last item are still in flight: their registers stay reserved until they
            // have landed (a register reused earlier would be overwritten when its load returns)
#pragma unroll
            for (int u = 0; u < STREAM_NP1; ++u) stream_ready<0>(it[u]);
            BB_STREAM_TRACE(1);
            while (cur_fb <= fb_last) flush(cur_fb++);
        }
    }

    BB_STREAM_TRACE(2);
    grid_arrive(p.bar, bar_base + 1u);

    // ---- phase 2 work of this workgroup.  Wavefronts 1..3 request their first
    // weight blocks now, so HBM stays busy while wavefront 0 runs the short
    // synchronised part (barrier, hidden block, barrier) with nothing in flight
    // that it would have to wait for.
    const int i2 = b * p.per2;
    const int iend2 = min(i2 + p.per2, p.items2);
    u32x4 pre[STREAM_NP2][8];
    auto issue2 = [&](int nb, int kb, int kb1, u32x4 (&r)[8]) {
        const int col = 128 * nb + 8 * jn;
        load_block(p.W2, p.D, 32 * kb + 8 * g4, p.F, col, col < p.D && kb < kb1, r);
    };
    auto prefetch2 = [&]() {
        if (i2 < iend2) {
            const int nb = i2 / p.nkb2, kb0 = i2 % p.nkb2;
            const int kb1 = min(p.nkb2, kb0 + (iend2 - i2));
#pragma unroll
            for (int u = 0; u < STREAM_NP2; ++u) issue2(nb, kb0 + w + 4 * u, kb1, pre[u]);
        }
    };
    if (w != 0) {
        prefetch2();
    } else {
        BB_STREAM_TRACE(3);
        bar_poll_wave(p.bar, bar_base + 1u, p.spin_limit, p.fault);
        BB_STREAM_TRACE(4);
        // =====================  phase 1b: hidden block  =====================
        const int groups_per_row = p.Fp / 8;                   // tasks: (row, 8 consecutive hidden units)
        const int total = 16 * groups_per_row;
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
                const float* src0 = p.ppart + (size_t)fb * p.S1 * RS + row * 128 + cc;
                const f32x4 z = {0, 0, 0, 0};
                acc[k][0] = z; acc[k][1] = z; acc[k][2] = z; acc[k][3] = z;
                ss[k] = 0.f;
                for (int s0 = 0; s0 < max(ns, nsq); s0 += 4) {   // four slots' loads in flight together
                    f32x4 v[4][4];
                    float sq[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const float* src = src0 + (size_t)(s0 + u) * RS;
                        const bool ok = s0 + u < ns;
                        v[u][0] = ok ? cload16f(src) : z;
                        v[u][1] = ok ? cload16f(src + 4) : z;
                        v[u][2] = ok ? cload16f(src + 2048) : z;
                        v[u][3] = ok ? cload16f(src + 2048 + 4) : z;
                        sq[u] = (s0 + u < nsq) ? cload4f(p.spart + (s0 + u) * 16 + row) : 0.f;
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
        // Where the output blocks' arrival counters stand before any workgroup can arrive in this launch
        // (arrivals come after barrier 2, which this workgroup has not signalled yet): lane j reads the
        // counter of this workgroup's j-th block of output columns.
        if (i2 < iend2) {
            const int nb_first = i2 / p.nkb2, nseg = (iend2 - 1) / p.nkb2 - nb_first + 1;     // (the host made sure nseg <= 64)
            if (lane < nseg)
                sm.segbase[lane] = __hip_atomic_load(p.cnt + nb_first + lane, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        if (lane == 0) bar_signal(p.bar, bar_base + 2u);
        bar_poll_wave(p.bar, bar_base + 2u, p.spin_limit, p.fault);
        if (lane == 0 && b == 0)       // (every workgroup read the count before its first arrival)
            __hip_atomic_store(p.epoch, bar_base + 2u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
    if (w == 0) prefetch2();
    const bool had_prefetch = i2 < iend2;
    bool preloaded = had_prefetch;
    BB_STREAM_TRACE(5);

    // =====================  phase 2: partial outputs  =====================
    {
        int i = i2;
        while (i < iend2) {                        // one segment = one block of 128 output columns
            const int nb = i / p.nkb2, kb0 = i % p.nkb2;
            const int kb1 = min(p.nkb2, kb0 + (iend2 - i));
            const int slot = b - (nb * p.nkb2) / p.per2;
            f32x4 acc[8];
#pragma unroll
            for (int c = 0; c < 8; ++c) acc[c] = f32x4{0, 0, 0, 0};
            // hidden fragments: row jn, hidden units 32 kb + 8 g4 .. +7
            auto hfrag = [&](int kb) -> u32x4 {
                if (kb >= kb1) return zero4();
                const u16* hsrc = p.H + (size_t)jn * p.Fp + 32 * kb + 8 * g4;
                const u32x2 lo = cload8(hsrc), hi = cload8(hsrc + 4);
                const u32x4 r = {lo[0], lo[1], hi[0], hi[1]};
                return r;
            };
            u32x4 hp[STREAM_NP2];
#pragma unroll
            for (int u = 0; u < STREAM_NP2; ++u) {
                if (!preloaded) issue2(nb, kb0 + w + 4 * u, kb1, pre[u]);
                hp[u] = hfrag(kb0 + w + 4 * u);
            }
            preloaded = false;
            for (int kbb = kb0 + w; kbb < kb1; kbb += 4 * STREAM_NP2) {
#pragma unroll
                for (int u = 0; u < STREAM_NP2; ++u) {
                    const int kb = kbb + 4 * u;
                    if (kb < kb1) {
                        Chunk ha;
                        ha.u = hp[u];
                        u32x4 tt[8];
                        transpose8x8(pre[u], tt);
                        issue2(nb, kb + 4 * STREAM_NP2, kb1, pre[u]);
                        hp[u] = hfrag(kb + 4 * STREAM_NP2);
#pragma unroll
                        for (int c = 0; c < 8; ++c) {
                            Chunk bw;
                            bw.u = tt[c];
                            acc[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ha.v, bw.v, acc[c], 0, 0, 0);
                        }
                    }
                }
            }
            stash_tile(sm.red[w][0], acc, lane);
            __syncthreads();
            float* dst = p.ypart + (size_t)(nb * p.S2 + slot) * 2048;
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int i4 = t + STREAM_THREADS * j;        // float4 index in [16][128]
                cstore16f(dst + 4 * i4, sum4(&sm.red[0][0][0][0], RS, i4));
            }
            // ---- phase 2b.  The partial tile is complete in memory (stores acknowledged), then thread 0
            // counts the delivery; the workgroup whose delivery is the last one of the block adds the
            // tiles of all slots in slot order (so the result does not depend on who is last), adds
            // the residual and stores the block's output.  No grid barrier.
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
            __builtin_amdgcn_s_waitcnt(0);
            __syncthreads();
            const int first = (nb * p.nkb2) / p.per2;
            const int ns = min(G - 1, ((nb + 1) * p.nkb2 - 1) / p.per2) - first + 1;      // slots of this block
            if (t == 0) {
                const unsigned old = __hip_atomic_fetch_add(p.cnt + nb, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                sm.last = (old + 1u - sm.segbase[nb - i2 / p.nkb2] == (unsigned)ns) ? 1u : 0u;
            }
            __syncthreads();
            if (sm.last) {
                const int row = t >> 4, cc = 8 * (t & 15);            // task: (row, 8 consecutive columns of the block)
                const int c0 = 128 * nb + cc;
                if (row < p.M && c0 < p.D) {
                    const float* src0 = p.ypart + (size_t)nb * p.S2 * 2048 + row * 128 + cc;
                    f32x4 y0 = {0, 0, 0, 0}, y1 = y0;
                    for (int s0 = 0; s0 < ns; s0 += 8) {              // eight slots' loads in flight together
                        f32x4 v[8][2];
#pragma unroll
                        for (int u = 0; u < 8; ++u) {
                            const float* src = src0 + (size_t)(s0 + u) * 2048;
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
            __syncthreads();
            i += kb1 - kb0;
        }
    }
    BB_STREAM_TRACE(7);
}
#endif  // BB_HOST_ONLY

}  // namespace bb
