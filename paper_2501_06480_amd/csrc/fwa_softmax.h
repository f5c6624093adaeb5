// Row softmax of one 16-query block in the "query on the lane" layout, shared by the
// forward and backward kernels.  Lane (g, n) holds s[jb][r] = <q_i, k_j> for query row i = i0 + n and
// key j = 16 jb + 4g + r; a row is spread over the 4 lanes that share n.
#pragma once

#include "fwa_device.h"

namespace fwa {

// The shift mask of one window comes in one of two forms: a dense fp32 tile [L, L], or the int32
// region labels [L] of its tokens, from which M[i][j] = labels[i] == labels[j] ? 0 : value is formed
// on the fly (L * 4 bytes per window instead of L * L * 4).  An absent mask is a dense one over a
// null descriptor: every load returns zero.
struct MaskSrc {
    __amdgpu_buffer_rsrc_t r;
    float value;  // what the scores of tokens with different labels receive; labels only
    bool labels;
};

template <class Args>
__device__ __forceinline__ MaskSrc mask_of_window(const Args& p, uint32_t w) {
    const uint32_t L = (uint32_t)p.L;
    if (p.labels) return MaskSrc{make_rsrc(p.labels + (size_t)(w % (uint32_t)p.nW) * L, L * 4u), p.mask_value, true};
    if (p.mask) return MaskSrc{make_rsrc(p.mask + (size_t)(w % (uint32_t)p.nW) * L * L, L * L * 4u), 0.f, false};
    return MaskSrc{make_rsrc(nullptr, 0), 0.f, false};
}

// Mask values of 4 consecutive columns of a row from the labels: lq = label of the row,
// lk = labels of the columns.
__device__ __forceinline__ f32x4 mask_of_labels(int lq, const i32x4& lk, float value) {
    return f32x4{lk[0] == lq ? 0.f : value, lk[1] == lq ? 0.f : value, lk[2] == lq ? 0.f : value,
                 lk[3] == lq ? 0.f : value};
}

// "Key on the lane": mask values M[i0 .. i0 + 3][j] for a lane that owns column j and 4 consecutive
// rows (i0 a multiple of 4).  Dense tiles cost 4 dword loads, labels one dword and one 16-byte load.
__device__ __forceinline__ f32x4 mask_rows4(const MaskSrc& m, uint32_t i0, uint32_t j, uint32_t L) {
    if (m.labels) return mask_of_labels(load_i32(m.r, 4u * j), load_i32x4(m.r, 4u * i0), m.value);
    const uint32_t off = (i0 * L + j) * 4u;
    return f32x4{load_f32(m.r, off), load_f32(m.r, off + 4u * L), load_f32(m.r, off + 8u * L), load_f32(m.r, off + 12u * L)};
}

// The bias tile of a head: fp32 through a descriptor over the head's [L, L] tile (rows beyond L read
// as zero), or bf16 through a descriptor over the whole [heads, L, L] tensor with the head's first
// element in `hbase` (a head's tile may start at an odd element, i.e. not on a dword, so loads are
// addressed from the tensor's aligned base; rows beyond L then read the next head's values, which
// are discarded like every padded row).  An absent bias is an fp32 one over a null descriptor.
struct BiasSrc {
    __amdgpu_buffer_rsrc_t r;
    uint32_t hbase;
    bool bf16;
};
__device__ __forceinline__ BiasSrc no_bias() { return BiasSrc{make_rsrc(nullptr, 0), 0u, false}; }
template <class Args>
__device__ __forceinline__ BiasSrc bias_of_head(const Args& p, uint32_t h) {
    const uint32_t L = (uint32_t)p.L;
    if (!p.bias) return no_bias();
    // size rounded up to whole dwords: with an odd element count the last dword holds the last element and
    // two bytes past the tensor, which lie in the same (aligned) dword and hence in the same page
    if (p.bias_bf16) return BiasSrc{make_rsrc(p.bias, ((uint32_t)p.heads * L * L * 2u + 3u) & ~3u), h * L * L, true};
    return BiasSrc{make_rsrc(static_cast<const float*>(p.bias) + (size_t)h * L * L, L * L * 4u), 0u, false};
}
// One element of the tile (idx = i L + j) and four consecutive ones out of a 16-byte load that
// started at the dword holding element idx (bf16: `odd` = idx is odd, the quad then starts in the
// upper half of the first dword).
__device__ __forceinline__ float bias_elem(const BiasSrc& b, uint32_t idx) {
    if (b.bf16) return load_bf16(b.r, 2u * (b.hbase + idx));
    return load_f32(b.r, 4u * idx);
}
__device__ __forceinline__ f32x4 bf16_quad(const f32x4& raw, bool odd) {
    const u32x4 r = __builtin_bit_cast(u32x4, raw);
    const uint32_t sh = odd ? 16u : 0u;
    const uint32_t lo = __builtin_amdgcn_alignbit(r.y, r.x, sh), hi = __builtin_amdgcn_alignbit(r.z, r.y, sh);
    const u32x4 e = {lo << 16, lo & 0xffff0000u, hi << 16, hi & 0xffff0000u};
    return __builtin_bit_cast(f32x4, e);
}

// Where the additive term of the scores (bias + mask) comes from.
// AddendGlobal: the bias tile of the head and the mask of the window; every load takes 4
// consecutive columns of the lane's row i: 16 bytes, only dword aligned; the range check is per
// dword, rows beyond L fall outside the descriptors and read as zero (label 0 for the mask).
struct AddendGlobal {
    BiasSrc rb;
    MaskSrc m;
    uint32_t off;     // byte offset of element [i][j0] of an [L, L] fp32 tile, j0 = 4g
    uint32_t i4, j4;  // 4 i and 4 j0: byte offsets of the labels of the row and of its first column
    // BF16_BIAS = false promises an fp32 (or absent) bias and leaves the bf16 path out of the code
    template <int NB, bool BF16_BIAS = true>
    __device__ __forceinline__ void fill(f32x4 (&add)[NB], float mul) const;
};
// The addend of row i (beyond L: zeros), first column j0, of the given bias tile and mask.
__device__ __forceinline__ AddendGlobal addend_at(const BiasSrc& rb, const MaskSrc& m, uint32_t i, uint32_t j0,
                                                  uint32_t L) {
    return AddendGlobal{rb, m, (i * L + j0) * 4u, 4u * i, 4u * j0};
}

// add[t][jb] = (bias + mask)[i_t][j0 + 16 jb ..+3] * mul for the NQ rows described by `rows`
// (same bias tile and mask).  Both forms of the mask issue the same loads, back to back and with
// nothing waiting on them: 16 bytes per key block from the mask descriptor (tile values, or the
// labels of the 4 columns) next to the bias loads, plus the row's own label.  Only the label form
// then passes through a uniform branch that turns labels into mask values in place; a dense mask
// skips it, so that the sums below can be scheduled as late as their consumer allows, as if there
// were no branch at all.
template <int NQ, int NB, bool BF16_BIAS = true>
__device__ __forceinline__ void fill_rows(f32x4 (&add)[NQ][NB], const AddendGlobal (&rows)[NQ], float mul) {
    const MaskSrc& m = rows[0].m;
    const BiasSrc& b = rows[0].rb;
    const bool bbf = BF16_BIAS && b.bf16;
    f32x4 mk[NQ][NB];
    int lq[NQ];
#pragma unroll
    for (int t = 0; t < NQ; ++t) {
        const uint32_t moff = m.labels ? rows[t].j4 : rows[t].off;
        // bf16 bias: the dword that holds element hbase + i L + j0, then 32 bytes per key block
        const uint32_t boff = bbf ? ((2u * b.hbase + (rows[t].off >> 1)) & ~3u) : rows[t].off;
        const uint32_t bstep = bbf ? 32u : 64u;
#pragma unroll
        for (int jb = 0; jb < NB; ++jb) {
            add[t][jb] = load_f32x4(b.r, boff + bstep * jb);
            mk[t][jb] = load_f32x4(m.r, moff + 16 * jb * 4u);
        }
        lq[t] = load_i32(m.r, rows[t].i4);  // dense: some element of the tile, unused
    }
    if (bbf) {  // uniform, like the label branch below: fp32 biases skip it
#pragma unroll
        for (int t = 0; t < NQ; ++t) {
            const bool odd = ((b.hbase + (rows[t].off >> 2)) & 1u) != 0;
#pragma unroll
            for (int jb = 0; jb < NB; ++jb) add[t][jb] = bf16_quad(add[t][jb], odd);
        }
    }
    if (m.labels) {
#pragma unroll
        for (int t = 0; t < NQ; ++t)
#pragma unroll
            for (int jb = 0; jb < NB; ++jb)
                mk[t][jb] = mask_of_labels(lq[t], __builtin_bit_cast(i32x4, mk[t][jb]), m.value);
    }
#pragma unroll
    for (int t = 0; t < NQ; ++t)
#pragma unroll
        for (int jb = 0; jb < NB; ++jb) add[t][jb] = (add[t][jb] + mk[t][jb]) * mul;
}
// The rows i0, i0 + 16, ... of one bias tile and mask.
template <int NQ, int NB>
__device__ __forceinline__ void fill_rows(f32x4 (&add)[NQ][NB], const BiasSrc& rb, const MaskSrc& m, uint32_t i0,
                                          uint32_t j0, uint32_t L, float mul) {
    AddendGlobal rows[NQ];
#pragma unroll
    for (int t = 0; t < NQ; ++t) rows[t] = addend_at(rb, m, i0 + 16 * t, j0, L);
    fill_rows<NQ, NB>(add, rows, mul);
}
template <int NB, bool BF16_BIAS>
__device__ __forceinline__ void AddendGlobal::fill(f32x4 (&add)[NB], float mul) const {
    f32x4 one[1][NB];
    const AddendGlobal rows[1] = {*this};
    fill_rows<1, NB, BF16_BIAS>(one, rows, mul);
#pragma unroll
    for (int jb = 0; jb < NB; ++jb) add[jb] = one[0][jb];
}
// AddendRegs: the term is already in registers (one f32x4 per key block), times log2e.
template <int NB>
struct AddendRegs {
    const f32x4 (&a)[NB];
    __device__ __forceinline__ void fill(f32x4 (&add)[NB], float) const {
#pragma unroll
        for (int jb = 0; jb < NB; ++jb) add[jb] = a[jb];
    }
};
// AddendRegsLabels: the bias (times log2e) in registers as above, the mask formed per score from the
// labels of the current window, which the kernel has staged in LDS: 0 where the label of the lane's
// query row equals that of the key, `mv` (mask value times log2e) elsewhere.  For persistent kernels
// whose workgroups cannot keep one mask tile for life (a mask period that does not divide their
// stride over the windows): the bias still stays in registers.  Keys beyond L read whatever the
// staging left there; their columns are overwritten with -inf afterwards.
template <int NB>
struct AddendRegsLabels {
    const f32x4 (&a)[NB];
    const int* lab;  // LDS: labels of tokens 0 .. 16 NB - 1 of the window
    int tq;          // label of the lane's query row
    float mv;
    int g;
    // the term of key block jb (one block at a time keeps the labels out of the register file)
    __device__ __forceinline__ f32x4 block(int jb) const {
        const i32x4 tk = *reinterpret_cast<const i32x4*>(lab + 16 * jb + 4 * g);
        f32x4 t;
#pragma unroll
        for (int r = 0; r < 4; ++r) t[r] = a[jb][r] + (tk[r] == tq ? 0.f : mv);
        return t;
    }
    __device__ __forceinline__ void fill(f32x4 (&add)[NB], float) const {
#pragma unroll
        for (int jb = 0; jb < NB; ++jb) add[jb] = block(jb);
    }
};
template <class A>
struct addend_per_block { static constexpr bool value = false; };
template <int NB>
struct addend_per_block<AddendRegsLabels<NB>> { static constexpr bool value = true; };
struct AddendNone {
    template <int NB>
    __device__ __forceinline__ void fill(f32x4 (&add)[NB], float) const {
#pragma unroll
        for (int jb = 0; jb < NB; ++jb) add[jb] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
};

// On entry s holds the raw products.  On exit s holds exp(score - rowmax), not yet
// normalised; the return value is 1 / rowsum.  Scores are scale * s + addend (BM) or
// scale * s (no bias/mask), and columns j >= L are excluded.
// KT < 4 promises L <= 16 (NB - 1) + KT: of the last key block only the components r < KT can be
// real columns (e.g. KT = 1 for L = 49), the others are set to zero without any arithmetic.
template <int NB, bool BM, class Addend, int KT = 4>
__device__ __forceinline__ float softmax_block(f32x4 (&s)[NB], float sl2, const Addend& addend, int L, int g) {
    float mul, mb;  // p = exp2(s * mul - mb)
    if (BM) {
        // Columns beyond L are overwritten with -inf below, whatever was fetched for them.
        f32x4 add[NB];
        addend.fill(add, kLog2e);
#pragma unroll
        for (int jb = 0; jb < NB; ++jb)
#pragma unroll
            for (int r = 0; r < (jb == NB - 1 ? KT : 4); ++r) s[jb][r] = fmaf(s[jb][r], sl2, add[jb][r]);
#pragma unroll
        for (int r = 0; r < KT; ++r)
            if (16 * (NB - 1) + 4 * g + r >= L) s[NB - 1][r] = -INFINITY;
        float m = s[0][0];
#pragma unroll
        for (int jb = 0; jb < NB; ++jb)
#pragma unroll
            for (int r = 0; r < (jb == NB - 1 ? KT : 4); ++r) m = fmaxf(m, s[jb][r]);
        mul = 1.0f;
        mb = max_over_g(m);
    } else {
        // No bias: keep the raw products and fold the scale into the exponent,
        // p = exp2(s*sl2 - max(s*sl2)).  For sl2 >= 0 the maximum of the scaled scores is
        // sl2 * max(s); a negative scale uses the minimum instead.  A zero scale makes every
        // score zero: the products are replaced by zeros and the multiplier by one (an infinite
        // pad times a zero multiplier would be NaN); the branch is uniform.
        const bool flat = sl2 == 0.f;
        if (flat) {
#pragma unroll
            for (int jb = 0; jb < NB; ++jb) s[jb] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
        const float pad = sl2 >= 0.f ? -INFINITY : INFINITY;
#pragma unroll
        for (int r = 0; r < KT; ++r)
            if (16 * (NB - 1) + 4 * g + r >= L) s[NB - 1][r] = pad;
        float m = s[0][0];
        if (sl2 >= 0.f) {
#pragma unroll
            for (int jb = 0; jb < NB; ++jb)
#pragma unroll
                for (int r = 0; r < (jb == NB - 1 ? KT : 4); ++r) m = fmaxf(m, s[jb][r]);
            m = max_over_g(m);
        } else {
#pragma unroll
            for (int jb = 0; jb < NB; ++jb)
#pragma unroll
                for (int r = 0; r < (jb == NB - 1 ? KT : 4); ++r) m = fminf(m, s[jb][r]);
            m = -max_over_g(-m);
        }
        mul = flat ? 1.0f : sl2;
        mb = m * mul;
    }
    float sum = 0.f;
#pragma unroll
    for (int jb = 0; jb < NB; ++jb)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            if (jb == NB - 1 && r >= KT) {
                s[jb][r] = 0.f;
                continue;
            }
            const float e = __builtin_amdgcn_exp2f(fmaf(s[jb][r], mul, -mb));
            s[jb][r] = e;
            sum += e;
        }
    sum = sum_over_g(sum);
    return __builtin_amdgcn_rcpf(sum);
}

// The first half of softmax_block on its own: scores scaled (with an additive term) and padded, the
// row maximum reduced.  Afterwards p = exp2(s * mul - mb), which softmax_exp_pair applies to two key
// blocks at a time, so that a kernel can issue the loads of the matching V operands first and let
// their latency pass behind the exponentials instead of in front of every matrix instruction.
template <int NB, bool BM, class Addend>
__device__ __forceinline__ float softmax_scale_max(f32x4 (&s)[NB], float sl2, const Addend& addend, int L, int g, float& mul) {
    if (BM) {
        if constexpr (addend_per_block<Addend>::value) {
#pragma unroll
            for (int jb = 0; jb < NB; ++jb) {
                const f32x4 t = addend.block(jb);
#pragma unroll
                for (int r = 0; r < 4; ++r) s[jb][r] = fmaf(s[jb][r], sl2, t[r]);
            }
        } else {
            f32x4 add[NB];
            addend.fill(add, kLog2e);
#pragma unroll
            for (int jb = 0; jb < NB; ++jb)
#pragma unroll
                for (int r = 0; r < 4; ++r) s[jb][r] = fmaf(s[jb][r], sl2, add[jb][r]);
        }
#pragma unroll
        for (int r = 0; r < 4; ++r)
            if (16 * (NB - 1) + 4 * g + r >= L) s[NB - 1][r] = -INFINITY;
        float m = s[0][0];
#pragma unroll
        for (int jb = 0; jb < NB; ++jb)
#pragma unroll
            for (int r = 0; r < 4; ++r) m = fmaxf(m, s[jb][r]);
        mul = 1.0f;
        return max_over_g(m);
    }
    // a zero scale: all scores are zero (see softmax_block)
    const bool flat = sl2 == 0.f;
    if (flat) {
#pragma unroll
        for (int jb = 0; jb < NB; ++jb) s[jb] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    const float pad = sl2 >= 0.f ? -INFINITY : INFINITY;
#pragma unroll
    for (int r = 0; r < 4; ++r)
        if (16 * (NB - 1) + 4 * g + r >= L) s[NB - 1][r] = pad;
    float m = s[0][0];
    if (sl2 >= 0.f) {
#pragma unroll
        for (int jb = 0; jb < NB; ++jb)
#pragma unroll
            for (int r = 0; r < 4; ++r) m = fmaxf(m, s[jb][r]);
        m = max_over_g(m);
    } else {
#pragma unroll
        for (int jb = 0; jb < NB; ++jb)
#pragma unroll
            for (int r = 0; r < 4; ++r) m = fminf(m, s[jb][r]);
        m = -max_over_g(-m);
    }
    mul = flat ? 1.0f : sl2;
    return m * mul;
}

// exponentials of key blocks 2 kp and 2 kp + 1, added to the lane's partial row sum (SUM = false: not
// added; the caller takes the row sum from the matrix core, see ones_operand)
template <int NB, bool SUM = true>
__device__ __forceinline__ void softmax_exp_pair(f32x4 (&s)[NB], int kp, float mul, float mb, float& sum) {
#pragma unroll
    for (int b = 0; b < 2; ++b) {
        const int jb = 2 * kp + b;
        if (jb >= NB) break;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const float e = __builtin_amdgcn_exp2f(fmaf(s[jb][r], mul, -mb));
            s[jb][r] = e;
            if (SUM) sum += e;
        }
    }
}

// The probabilities of key blocks 2 kp and 2 kp + 1 of a lane as one 16-bit operand (bf16, or half with F16)
// (k-slots 0..3 = keys 4g..4g+3 of the first block, 4..7 = the same keys of the second).
template <int NB, bool F16 = false>
__device__ __forceinline__ bf16x8 prob_operand(const f32x4 (&s)[NB], int kp) {
    u32x4 a;
    a.x = pack_e<F16>(s[2 * kp][0], s[2 * kp][1]);
    a.y = pack_e<F16>(s[2 * kp][2], s[2 * kp][3]);
    const int j1 = 2 * kp + 1 < NB ? 2 * kp + 1 : 0;  // odd NB: the last pair has no second block
    a.z = 2 * kp + 1 < NB ? pack_e<F16>(s[j1][0], s[j1][1]) : 0u;
    a.w = 2 * kp + 1 < NB ? pack_e<F16>(s[j1][2], s[j1][3]) : 0u;
    return as_bf16x8(a);
}

}  // namespace fwa
