// Shared device helpers for the gfx950 kernels: vector types, bf16 packing,
// the LDS swizzle and the register transposition used to turn row-major
// (contraction-strided) weight tiles into matrix-instruction operands.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace bb {

typedef unsigned short u16;
typedef unsigned int u32;
typedef __attribute__((__vector_size__(4 * sizeof(u32)))) u32 u32x4;
typedef __attribute__((__vector_size__(2 * sizeof(u32)))) u32 u32x2;
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
typedef __attribute__((__vector_size__(2 * sizeof(float)))) float f32x2;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

union Chunk {          // 16 bytes = 8 bf16 = one matrix-instruction operand
    u32x4 u;
    bf16x8 v;
};

__device__ __forceinline__ float bf_lo(u32 w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf_hi(u32 w) { return __uint_as_float(w & 0xffff0000u); }

// two floats -> packed bf16 pair (round to nearest even), low half = a
__device__ __forceinline__ u32 pack_bf16(float a, float b) {
    f32x2 v = {a, b};
    bf16x2 r = __builtin_convertvector(v, bf16x2);
    return *reinterpret_cast<u32*>(&r);
}

// (lo16(a), lo16(b)) and (hi16(a), hi16(b)) as one dword, a in the low half
__device__ __forceinline__ u32 pack_lo(u32 a, u32 b) { return __builtin_amdgcn_perm(b, a, 0x05040100u); }
__device__ __forceinline__ u32 pack_hi(u32 a, u32 b) { return __builtin_amdgcn_perm(b, a, 0x07060302u); }

// In-register transposition of an 8x8 block of bf16.
// in[r] holds row r (8 consecutive columns of one contraction index);
// out[c] holds column c (8 consecutive contraction indices of one column),
// which is what a lane must supply to a 16x16x32 / 32x32x16 matrix instruction.
__device__ __forceinline__ void transpose8x8(const u32x4 (&in)[8], u32x4 (&out)[8]) {
#pragma unroll
    for (int c = 0; c < 8; ++c) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const u32 a = in[2 * q][c >> 1], b = in[2 * q + 1][c >> 1];
            out[c][q] = (c & 1) ? pack_hi(a, b) : pack_lo(a, b);
        }
    }
}

// LDS tiles of the A operand are arrays of 16-byte chunks, 8 chunks (64
// contraction indices) per row.  The LDS of gfx950 has 64 four-byte banks and
// serves a 128-bit read of a wavefront sixteen lanes at a time (measured: 256
// bytes per clock when these sixteen chunks fall on sixteen different 16-byte
// bank groups, half of that with a swizzle that only separates eight).  A
// fragment read has 16 consecutive lanes on 16 consecutive rows at one chunk
// index; two rows are one pass through the banks, so the chunk index is
// XOR-swizzled with bits 1..3 of the row.
__device__ __forceinline__ int lds_pos(int row, int kc) { return row * 8 + (kc ^ ((row >> 1) & 7)); }

__device__ __forceinline__ u32x4 zero4() { u32x4 z = {0u, 0u, 0u, 0u}; return z; }

__device__ __forceinline__ u32x4 ldg16(const u16* p) { return *reinterpret_cast<const u32x4*>(p); }

// x / (1 + exp(-x)) * gate, fp32
__device__ __forceinline__ float swiglu(float p, float q) {
    const float e = __expf(-p);
    return p * __builtin_amdgcn_rcpf(1.0f + e) * q;
}

// Data exchanged between workgroups inside a kernel is written with
// agent-scope stores (written through, complete when acknowledged) and read
// with agent-scope loads (never a stale cached copy).  So neither side needs a
// cache write-back or invalidation around the barrier or the arrival
// counter, and nothing waits on other loads that are in flight.
__device__ __forceinline__ void cstore8(void* p, u32 lo, u32 hi) {
    __hip_atomic_store(reinterpret_cast<unsigned long long*>(p), ((unsigned long long)hi << 32) | lo,
                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void cstore16f(float* p, const f32x4 v) {
    cstore8(p, __float_as_uint(v[0]), __float_as_uint(v[1]));
    cstore8(p + 2, __float_as_uint(v[2]), __float_as_uint(v[3]));
}
__device__ __forceinline__ u32x2 cload8(const void* p) {
    const unsigned long long v =
        __hip_atomic_load(reinterpret_cast<const unsigned long long*>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    u32x2 r = {(u32)v, (u32)(v >> 32)};
    return r;
}
__device__ __forceinline__ f32x4 cload16f(const float* p) {
    const u32x2 a = cload8(p), b = cload8(p + 2);
    f32x4 r = {__uint_as_float(a[0]), __uint_as_float(a[1]), __uint_as_float(b[0]), __uint_as_float(b[1])};
    return r;
}
__device__ __forceinline__ float cload4f(const float* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

}  // namespace bb
