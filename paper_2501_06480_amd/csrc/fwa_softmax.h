// Row softmax of one 16-query block in the "query on the lane" layout, shared by the
// forward and backward kernels.  Lane (g, n) holds s[jb][r] = <q_i, k_j> for query row i = i0 + n and
// key j = 16 jb + 4g + r; a row is spread over the 4 lanes that share n.
#pragma once

#include "fwa_device.h"

namespace fwa {

// Where the additive term of the scores (bias + mask, in log2 units) comes from.
// AddendGlobal: two buffer descriptors (absent tensor = null descriptor = zeros); every load
// takes 4 consecutive columns of one row: 16 bytes, only dword aligned; the range check is per
// dword, rows beyond L fall outside the descriptor and read as zero.
struct AddendGlobal {
    __amdgpu_buffer_rsrc_t rb, rm;
    uint32_t off;  // byte offset of element [i0 + n][4g] of the tile
    __device__ __forceinline__ f32x4 operator()(int jb) const {
        return (load_f32x4(rb, off + 16 * jb * 4u) + load_f32x4(rm, off + 16 * jb * 4u)) * kLog2e;
    }
};
// AddendRegs: the term is already in registers (one f32x4 per key block), times log2e.
template <int NB>
struct AddendRegs {
    const f32x4 (&a)[NB];
    __device__ __forceinline__ f32x4 operator()(int jb) const { return a[jb]; }
};
struct AddendNone {
    __device__ __forceinline__ f32x4 operator()(int) const { return f32x4{0.f, 0.f, 0.f, 0.f}; }
};

// On entry s holds the raw products.  On exit s holds exp(score - rowmax), not yet
// normalised; the return value is 1 / rowsum.  Scores are scale * s + addend (BM) or
// scale * s (no bias/mask), and columns j >= L are excluded.
template <int NB, bool BM, class Addend>
__device__ __forceinline__ float softmax_block(f32x4 (&s)[NB], float sl2, const Addend& addend, int L, int g) {
    float mul, mb;  // p = exp2(s * mul - mb)
    if (BM) {
        // Columns beyond L are overwritten with -inf below, whatever was fetched for them.
#pragma unroll
        for (int jb = 0; jb < NB; ++jb) {
            const f32x4 add = addend(jb);
#pragma unroll
            for (int r = 0; r < 4; ++r) s[jb][r] = fmaf(s[jb][r], sl2, add[r]);
        }
#pragma unroll
        for (int r = 0; r < 4; ++r)
            if (16 * (NB - 1) + 4 * g + r >= L) s[NB - 1][r] = -INFINITY;
        float m = s[0][0];
#pragma unroll
        for (int jb = 0; jb < NB; ++jb) {
            m = fmaxf(fmaxf(m, s[jb][0]), s[jb][1]);
            m = fmaxf(fmaxf(m, s[jb][2]), s[jb][3]);
        }
        mul = 1.0f;
        mb = max_over_g(m);
    } else {
        // No bias: keep the raw products and fold the scale into the exponent,
        // p = exp2(s*sl2 - max(s*sl2)).  For sl2 >= 0 the maximum of the scaled scores is
        // sl2 * max(s); a negative scale uses the minimum instead.
        const float pad = sl2 >= 0.f ? -INFINITY : INFINITY;
#pragma unroll
        for (int r = 0; r < 4; ++r)
            if (16 * (NB - 1) + 4 * g + r >= L) s[NB - 1][r] = pad;
        float m = s[0][0];
        if (sl2 >= 0.f) {
#pragma unroll
            for (int jb = 0; jb < NB; ++jb) {
                m = fmaxf(fmaxf(m, s[jb][0]), s[jb][1]);
                m = fmaxf(fmaxf(m, s[jb][2]), s[jb][3]);
            }
            m = max_over_g(m);
        } else {
#pragma unroll
            for (int jb = 0; jb < NB; ++jb) {
                m = fminf(fminf(m, s[jb][0]), s[jb][1]);
                m = fminf(fminf(m, s[jb][2]), s[jb][3]);
            }
            m = -max_over_g(-m);
        }
        mul = sl2;
        mb = m * sl2;
    }
    float sum = 0.f;
#pragma unroll
    for (int jb = 0; jb < NB; ++jb)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const float e = __builtin_amdgcn_exp2f(fmaf(s[jb][r], mul, -mb));
            s[jb][r] = e;
            sum += e;
        }
    sum = sum_over_g(sum);
    return __builtin_amdgcn_rcpf(sum);
}

// The probabilities of key blocks 2 kp and 2 kp + 1 of a lane as one bf16 operand
// (k-slots 0..3 = keys 4g..4g+3 of the first block, 4..7 = the same keys of the second).
template <int NB>
__device__ __forceinline__ bf16x8 prob_operand(const f32x4 (&s)[NB], int kp) {
    u32x4 a;
    a.x = pack_bf16(s[2 * kp][0], s[2 * kp][1]);
    a.y = pack_bf16(s[2 * kp][2], s[2 * kp][3]);
    const int j1 = 2 * kp + 1 < NB ? 2 * kp + 1 : 0;  // odd NB: the last pair has no second block
    a.z = 2 * kp + 1 < NB ? pack_bf16(s[j1][0], s[j1][1]) : 0u;
    a.w = 2 * kp + 1 < NB ? pack_bf16(s[j1][2], s[j1][3]) : 0u;
    return as_bf16x8(a);
}

}  // namespace fwa
