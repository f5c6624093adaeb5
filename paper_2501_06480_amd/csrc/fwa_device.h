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
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef int i32x4 __attribute__((ext_vector_type(4)));

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

// The 16-bit operand types share one carrier: kernels that take bf16 or IEEE half data (template flag F16)
// keep their operands in the bf16 vector types as raw bits and pick the matrix instruction and the
// conversion here.  Half products have 11 significant bits in each operand, bf16 products 8.
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
template <bool F16>
__device__ __forceinline__ f32x4 mfma_e(bf16x8 a, bf16x8 b, f32x4 c) {
    if constexpr (F16)
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}
// two fp32 -> a packed pair of the 16-bit type (lo = a, hi = b), round to nearest even
template <bool F16>
__device__ __forceinline__ uint32_t pack_e(float a, float b) {
    f32x2 t = {a, b};
    if constexpr (F16)
        return __builtin_bit_cast(uint32_t, __builtin_convertvector(t, f16x2));
    else
        return __builtin_bit_cast(uint32_t, __builtin_convertvector(t, bf16x2));
}

__device__ __forceinline__ bf16x8 as_bf16x8(uint4 u) { return __builtin_bit_cast(bf16x8, u); }
__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 u) { return __builtin_bit_cast(bf16x8, u); }

// Raw buffer descriptor over `bytes` bytes at `base`.  Loads whose offset lies
// beyond `bytes` return zero and such stores are dropped by the hardware, which
// is how rows past the end of a tile are padded without branches.  Every access
// made through it is either entirely inside or entirely outside the range.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base, uint32_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, 0x00020000);
}

// NOTE: never write __builtin_bit_cast(T, vec[i]) on a vector element: this
// compiler reads element 0 whatever i is.  Cast whole vectors, or copy the
// element into a scalar first.
__device__ __forceinline__ f32x4 load_f32x4(__amdgpu_buffer_rsrc_t r, uint32_t voffset) {
    return __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(r, voffset, 0, 0));
}
__device__ __forceinline__ void store_f32x4(f32x4 v, __amdgpu_buffer_rsrc_t r, uint32_t voffset) {
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, v), r, voffset, 0, 0);
}
__device__ __forceinline__ float load_f32(__amdgpu_buffer_rsrc_t r, uint32_t voffset) {
    return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(r, voffset, 0, 0));
}
// one bf16 element (2-byte load) as fp32
__device__ __forceinline__ float load_bf16(__amdgpu_buffer_rsrc_t r, uint32_t voffset) {
    return __builtin_bit_cast(float, (uint32_t)(uint16_t)__builtin_amdgcn_raw_buffer_load_b16(r, voffset, 0, 0) << 16);
}
__device__ __forceinline__ i32x4 load_i32x4(__amdgpu_buffer_rsrc_t r, uint32_t voffset) {
    return __builtin_bit_cast(i32x4, __builtin_amdgcn_raw_buffer_load_b128(r, voffset, 0, 0));
}
__device__ __forceinline__ int load_i32(__amdgpu_buffer_rsrc_t r, uint32_t voffset) {
    return (int)__builtin_amdgcn_raw_buffer_load_b32(r, voffset, 0, 0);
}

// Unsigned division by a runtime constant with a host-made multiplier
// (round-up method): n / d == (mulhi(n, mul) + n) >> shift for n < 2^31.
struct FastDiv {
    uint32_t mul, shift, d;
};
__host__ inline FastDiv make_fastdiv(uint32_t d) {
    FastDiv f;
    f.d = d;
    uint32_t l = 0;
    while ((1u << l) < d) ++l;
    f.shift = l;
    f.mul = (uint32_t)((((uint64_t)1 << 32) * (((uint64_t)1 << l) - d)) / d + 1);
    return f;
}
__device__ __forceinline__ uint32_t fastdiv(uint32_t n, const FastDiv& f) {
    return (uint32_t)(((uint64_t)__umulhi(n, f.mul) + n) >> f.shift);
}

// Workgroups are handed to the 8 XCDs (each with its own L2) round-robin by
// index.  This maps the hardware index to a logical one such that logical
// neighbours run on the same XCD: XCD x owns the contiguous logical range
// [x*q + min(x, r), ...) where q, r = nblocks / 8, nblocks % 8.
__device__ __forceinline__ uint32_t xcd_logical_block(uint32_t bid, uint32_t q, uint32_t r) {
    const uint32_t x = bid & 7u, idx = bid >> 3;
    return x * q + (x < r ? x : r) + idx;
}

// max / sum over the 4 lanes (g = 0..3) that share the same n.  The gfx950
// lane-swap instructions exchange 16-lane rows between two registers
// (v_permlane16_swap: odd rows of the first with even rows of the second;
// v_permlane32_swap: upper half of the first with lower half of the second).
// Fed two copies of x, one swap leaves (x of rows 0,0,2,2 | x of rows 1,1,3,3)
// resp. (x of the low half | x of the high half) in the two registers, so a
// swap plus one max/add per step reduces across rows without the LDS crossbar.
__device__ __forceinline__ float max_over_g(float x) {
    uint32_t u = __builtin_bit_cast(uint32_t, x);
    auto s16 = __builtin_amdgcn_permlane16_swap(u, u, false, false);
    uint32_t a = s16[0], b = s16[1];
    x = fmaxf(__builtin_bit_cast(float, a), __builtin_bit_cast(float, b));
    u = __builtin_bit_cast(uint32_t, x);
    auto s32 = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    a = s32[0];
    b = s32[1];
    return fmaxf(__builtin_bit_cast(float, a), __builtin_bit_cast(float, b));
}
__device__ __forceinline__ float sum_over_g(float x) {
    uint32_t u = __builtin_bit_cast(uint32_t, x);
    auto s16 = __builtin_amdgcn_permlane16_swap(u, u, false, false);
    uint32_t a = s16[0], b = s16[1];
    x = __builtin_bit_cast(float, a) + __builtin_bit_cast(float, b);
    u = __builtin_bit_cast(uint32_t, x);
    auto s32 = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    a = s32[0];
    b = s32[1];
    return __builtin_bit_cast(float, a) + __builtin_bit_cast(float, b);
}
// sum over the 16 lanes (n = 0..15) that share the same g
__device__ __forceinline__ float sum_over_n(float x) {
    x += __shfl_xor(x, 1);
    x += __shfl_xor(x, 2);
    x += __shfl_xor(x, 4);
    x += __shfl_xor(x, 8);
    return x;
}

// (lo16(a), lo16(b)) and (hi16(a), hi16(b)) as one byte-permute each
__device__ __forceinline__ uint32_t lower_halves(uint32_t a, uint32_t b) { return __builtin_amdgcn_perm(b, a, 0x05040100u); }
__device__ __forceinline__ uint32_t upper_halves(uint32_t a, uint32_t b) { return __builtin_amdgcn_perm(b, a, 0x07060302u); }

typedef short bf16x4 __attribute__((ext_vector_type(4)));  // raw bf16 bits, operand of the K=16 matrix op
__device__ __forceinline__ f32x4 mfma16(bf16x4 a, bf16x4 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ bf16x4 as_bf16x4(uint2 u) { return __builtin_bit_cast(bf16x4, u); }

// fp32 values that are exactly bf16 (results of a product with a 0/1 matrix) -> packed bf16
__device__ __forceinline__ uint2 pack_exact_u2(const f32x4& x) {
    uint32_t u[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        const float xc = x[c];
        u[c] = __builtin_bit_cast(uint32_t, xc);
    }
    uint2 h;
    h.x = upper_halves(u[0], u[1]);
    h.y = upper_halves(u[2], u[3]);
    return h;
}
__device__ __forceinline__ bf16x4 pack_exact(const f32x4& x) { return as_bf16x4(pack_exact_u2(x)); }

// x = hi + lo with hi the upper 16 bits of x (a bf16 by truncation) and lo the
// remainder rounded to bf16: together 16 significant bits.
__device__ __forceinline__ void split_hi_lo(const f32x4& x, bf16x4& hi, bf16x4& lo) {
    uint32_t u[4];
    float rem[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        const float xc = x[c];
        u[c] = __builtin_bit_cast(uint32_t, xc);
        rem[c] = xc - __builtin_bit_cast(float, u[c] & 0xffff0000u);
    }
    uint2 h, l;
    h.x = upper_halves(u[0], u[1]);
    h.y = upper_halves(u[2], u[3]);
    l.x = pack_bf16(rem[0], rem[1]);
    l.y = pack_bf16(rem[2], rem[3]);
    hi = as_bf16x4(h);
    lo = as_bf16x4(l);
}

// B operand of the K=16 matrix op that is the 16x16 identity: slot e of lane (g, n) is 1.0 iff
// 4g + e == n.  X (as A operand) times it returns X in the accumulator layout, i.e. with the
// other index on the lane: lane (g', n') <- X[row 4g' + r][column n'].
__device__ __forceinline__ bf16x4 identity_operand(int g, int n) {
    uint2 u;
    u.x = (4 * g + 0 == n ? 0x3f80u : 0u) | (4 * g + 1 == n ? 0x3f800000u : 0u);
    u.y = (4 * g + 2 == n ? 0x3f80u : 0u) | (4 * g + 3 == n ? 0x3f800000u : 0u);
    return as_bf16x4(u);
}

// A operand of the K=32 matrix op that is all ones: times the probability operand of a pair of key blocks it
// returns, in every component of every lane (g, n), the sum over the pair's 32 keys of the (rounded)
// probabilities of query n.  Accumulated over the pairs this is the row sum the output is divided by -- the sum of
// the very weights the output was formed with -- at the price of one matrix instruction per pair instead of one
// addition per score and the reduction over the four lanes of a row.
__device__ __forceinline__ bf16x8 ones_operand() {
    const u32x4 s = {0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u};
    return as_bf16x8(s);
}

// B operand of the K=32 matrix op that picks every second channel: slot e of lane (g, n)
// stands for channel 8g + e; the product rows x selector puts channel 2n + parity of each
// row into column n, i.e. returns lane (g', n') <- X[row 4g' + r][channel 2n' + parity].
// This turns a row operand (channels on the k-slots) into the operand with the rows on the
// k-slots without touching memory.
__device__ __forceinline__ bf16x8 channel_selector(int g, int n, int parity) {
    u32x4 s = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int e = 0; e < 8; ++e)
        if (8 * g + e == 2 * n + parity) s[e >> 1] |= (e & 1) ? 0x3f800000u : 0x3f80u;
    return as_bf16x8(s);
}

// Transposing LDS read (ds_read_b64_tr_b16): lane r of a row of 16 lanes passes the address of
// 4 consecutive bf16, lane t receives element (t & 3) of the rows passed by lanes (t >> 2) + 4 e,
// e = 0..3.  With lane r pointing at X[i0 + (r >> 2)][j0 + 4 (r & 3)] lane t receives
// X[i0 + e][j0 + t]: the k-slots of an operand whose lane index is the column of a row-major tile.
typedef short v4i16 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint2 lds_read_tr(const uint16_t* p) {
    typedef __attribute__((address_space(3))) v4i16 lds_v4i16;
    const v4i16 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4i16*)(p));
    return __builtin_bit_cast(uint2, v);
}
// Operand whose 8 k-slots are rows i0 + 4g + e (e < 4) and i0 + 16 + 4g + (e - 4) of a row-major
// bf16 tile and whose lane index is column j0 + n; `p` = &X[i0 + 4g + (n >> 2)][j0 + 4 (n & 3)],
// `rows16` = elements between row i and row i + 16.  `two` = the second 16 rows exist.
__device__ __forceinline__ bf16x8 operand_tr(const uint16_t* p, uint32_t rows16, bool two) {
    const uint2 a = lds_read_tr(p);
    uint2 b = {0u, 0u};
    if (two) b = lds_read_tr(p + rows16);
    return as_bf16x8(u32x4{a.x, a.y, b.x, b.y});
}

}  // namespace fwa
