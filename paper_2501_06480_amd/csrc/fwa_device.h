// Device-side helpers for the gfx950 kernels: matrix-core operand types,
// wave-level reductions over the four 16-lane rows, bf16 packing.
//
// Lane naming used throughout: a 64-lane wave is seen as 4 rows of 16 lanes,
//     n = lane & 15  (position inside the row),  g = lane >> 4  (which row).
// For v_mfma_f32_16x16x32_bf16 (and 16x16x4_f32) lane (g, n) supplies
//     A[m = n][k-slots owned by g]   and   B[k-slots owned by g][col = n],
// and receives the four accumulators  D[row = 4g + r][col = n], r = 0..3.
// Which contraction index a k-slot stands for is free as long as A and B agree,
// which the kernels use to feed operands straight from row-major global memory.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fwa {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

constexpr float kLog2e = 1.4426950408889634f;

__device__ __forceinline__ f32x4 mfma_bf16(bf16x8 a, bf16x8 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ f32x4 mfma_f32(float a, float b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}

// two fp32 -> packed bf16 pair (lo = a, hi = b), round to nearest even
__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
    f32x2 t = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(t, bf16x2));
}

__device__ __forceinline__ bf16x8 as_bf16x8(uint4 u) { return __builtin_bit_cast(bf16x8, u); }

// max / sum over the 4 lanes (g = 0..3) that share the same n
__device__ __forceinline__ float max_over_g(float x) {
    x = fmaxf(x, __shfl_xor(x, 16));
    x = fmaxf(x, __shfl_xor(x, 32));
    return x;
}
__device__ __forceinline__ float sum_over_g(float x) {
    x += __shfl_xor(x, 16);
    x += __shfl_xor(x, 32);
    return x;
}
// sum over the 16 lanes (n = 0..15) that share the same g
__device__ __forceinline__ float sum_over_n(float x) {
    x += __shfl_xor(x, 1);
    x += __shfl_xor(x, 2);
    x += __shfl_xor(x, 4);
    x += __shfl_xor(x, 8);
    return x;
}

// Split 8 dwords, each holding the bf16 pair (channel 2n, channel 2n+1) of one
// row, into the operand of the even channel (low halves) and of the odd one.
__device__ __forceinline__ void split_pairs(const uint32_t (&d)[8], bf16x8& even, bf16x8& odd) {
    uint4 e, o;
    e.x = (d[0] & 0xffffu) | (d[1] << 16);
    e.y = (d[2] & 0xffffu) | (d[3] << 16);
    e.z = (d[4] & 0xffffu) | (d[5] << 16);
    e.w = (d[6] & 0xffffu) | (d[7] << 16);
    o.x = (d[0] >> 16) | (d[1] & 0xffff0000u);
    o.y = (d[2] >> 16) | (d[3] & 0xffff0000u);
    o.z = (d[4] >> 16) | (d[5] & 0xffff0000u);
    o.w = (d[6] >> 16) | (d[7] & 0xffff0000u);
    even = as_bf16x8(e);
    odd = as_bf16x8(o);
}

// Row index (inside a 32-row group) that k-slot e of lane row g stands for when
// the A operand is built from two 16x16 accumulator tiles: slots 0..3 are rows
// 4g..4g+3 of the first tile, slots 4..7 the same rows of the second.
__device__ __forceinline__ int slot_row(int g, int e) { return (e & 3) + 4 * g + 16 * (e >> 2); }

}  // namespace fwa
