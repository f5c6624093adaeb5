// Forward kernels: O = softmax(scale*QK^T + B + M) V per (window, head) tile.
//
// Paper Algorithm 1 keeps the L x L score tile on chip and touches Q, K, V, O
// once; it walks the feature dimension in chunks because its target GPU has
// little on-chip memory.  Here the head width is 32, which is exactly one
// k-step of the gfx950 bf16 matrix instruction, so the chunk loop has a single
// iteration (r = 1) and the whole tile lives in one wave's registers:
//
//   * one wave owns one (window, head) tile (or a slice of its query rows);
//   * K rows go from global memory straight into A operands (16 B per lane),
//     Q rows into B operands, so the accumulators hold S^T:
//         lane (g, n), tile jb, slot r  <->  S[i = n][j = 16 jb + 4 g + r];
//     a query row is spread over the 4 lanes sharing n, so max and sum need
//     two cross-row shuffles each and no LDS;
//   * in that layout the probabilities of a lane are already a B operand of
//     O^T = V^T P^T (its k-slots are keys 4g..4g+3 of two neighbouring tiles);
//     V is loaded as rows like K and turned by the matrix core (rows times a
//     0/1 channel selector) into an even-channel and an odd-channel A operand
//     with the keys on the k-slots.  The two
//     accumulators of lane (g, n) then hold channels 8g..8g+7 of query row n:
//     the row's softmax sum is in the same lane and the result leaves as one
//     16-byte store, mirroring the Q load;
//   * all global traffic goes through raw buffer descriptors sized to the tile:
//     rows beyond L (L is padded to a multiple of 16 on chip only) load as
//     zero and their stores are dropped by the address range check, so there
//     are no branches and nothing is touched outside [N, L, C]; padded score
//     columns are set to -inf.  The range check covers the vector offset and
//     the immediate only, NOT the scalar offset operand, so every offset goes
//     into the vector operand and the scalar one stays 0.
#include "fwa_device.h"
#include "fwa_internal.h"
#include "fwa_softmax.h"

namespace fwa {
namespace {

// How a launch is cut into workgroups and waves (all wave-uniform).
struct FwdGeom {
    FastDiv groups;        // workgroups per window
    uint32_t heads_per_block;
    uint32_t qsplit_log2;  // waves sharing the query blocks of one tile = 1 << qsplit_log2
    uint32_t xcd_remap;    // use the XCD-aware block order
    uint32_t xcd_q, xcd_r; // nblocks / 8, nblocks % 8 for that order
};

template <int NB>
struct Tiling {
    static constexpr int kQSplitLog2 = NB <= 4 ? 0 : (NB <= 8 ? 1 : 2);
    static constexpr int kQSplit = 1 << kQSplitLog2;
    static constexpr int kQPerWave = (NB + kQSplit - 1) / kQSplit;  // query blocks per wave
};

struct TileCoord {
    uint32_t w, h, qs;
    bool valid;
};
__device__ __forceinline__ TileCoord tile_of_wave(const FwdGeom& gm, int heads) {
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t lb = gm.xcd_remap ? xcd_logical_block(blockIdx.x, gm.xcd_q, gm.xcd_r) : blockIdx.x;
    TileCoord t;
    t.w = fastdiv(lb, gm.groups);
    const uint32_t hg = lb - t.w * gm.groups.d;
    t.h = hg * gm.heads_per_block + (wave >> gm.qsplit_log2);
    t.qs = wave & ((1u << gm.qsplit_log2) - 1u);
    t.valid = t.h < (uint32_t)heads;
    return t;
}

// ---------------------------------------------------------------- bf16 ----
// NB = ceil(L / 16) key/query blocks; BM = a bias and/or mask is present.
template <int NB, bool BM>
__global__ void __launch_bounds__(64 * kWavesPerBlock) fwd_bf16_kernel(FwdArgs p, FwdGeom gm) {
    constexpr int NB2 = (NB + 1) / 2;
    constexpr int QPW = Tiling<NB>::kQPerWave;
    const int lane = threadIdx.x & 63;
    const int n = lane & 15, g = lane >> 4;
    const TileCoord tc = tile_of_wave(gm, p.heads);
    if (!tc.valid) return;  // wave-uniform; the kernel has no barriers
    const int L = p.L;
    // token rows are p.ldq (q, k, v) resp. p.ldo (o) elements apart; window w starts at row w L
    const uint32_t row_bytes = (uint32_t)p.ldq * 2u, row_out = (uint32_t)p.ldo * 2u;
    const uint32_t tile_bytes = (uint32_t)(L - 1) * row_bytes + 2u * kHeadDim;
    const size_t tile = ((size_t)tc.w * L * p.ldq + (size_t)tc.h * kHeadDim) * 2u;
    const __amdgpu_buffer_rsrc_t rq = make_rsrc((const char*)p.q + tile, tile_bytes);
    const __amdgpu_buffer_rsrc_t rk = make_rsrc((const char*)p.k + tile, tile_bytes);
    const __amdgpu_buffer_rsrc_t rv = make_rsrc((const char*)p.v + tile, tile_bytes);
    const __amdgpu_buffer_rsrc_t ro = make_rsrc((char*)p.o + ((size_t)tc.w * L * p.ldo + (size_t)tc.h * kHeadDim) * 2u,
                                                (uint32_t)(L - 1) * row_out + 2u * kHeadDim);
    const uint32_t off_row = (uint32_t)n * row_bytes + 16u * g;  // 16 B of row n (plus a block offset)

    // K: A operands of S^T, lane (g, n) = K[16 jb + n][8g .. 8g+7]
    bf16x8 kop[NB];
#pragma unroll
    for (int jb = 0; jb < NB; ++jb)
        kop[jb] = as_bf16x8(__builtin_amdgcn_raw_buffer_load_b128(rk, off_row + 16 * jb * row_bytes, 0, 0));
    // Q: B operands, one per query block of this wave
    bf16x8 qop[QPW];
#pragma unroll
    for (int t = 0; t < QPW; ++t)
        qop[t] = as_bf16x8(__builtin_amdgcn_raw_buffer_load_b128(rq, off_row + 16 * (tc.qs * QPW + t) * row_bytes, 0, 0));
    // V: A operands of O^T per pair of key blocks (keys on the k-slots, even resp. odd
    // channels on the lane).
    bf16x8 vop[NB2][2];
    {
        // V is loaded as rows like K and turned into the operands by the matrix core
        // (rows x channel selector): 16-byte loads only.
        bf16x8 vrow[NB];
#pragma unroll
        for (int jb = 0; jb < NB; ++jb)
            vrow[jb] = as_bf16x8(__builtin_amdgcn_raw_buffer_load_b128(rv, off_row + 16 * jb * row_bytes, 0, 0));
        const bf16x8 sel[2] = {channel_selector(g, n, 0), channel_selector(g, n, 1)};
        const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kp = 0; kp < NB2; ++kp)
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                const uint2 a = pack_exact_u2(mfma_bf16(vrow[2 * kp], sel[c], zero));
                uint2 b = {0u, 0u};
                if (2 * kp + 1 < NB) b = pack_exact_u2(mfma_bf16(vrow[2 * kp + 1 < NB ? 2 * kp + 1 : 0], sel[c], zero));
                const u32x4 v = {a.x, a.y, b.x, b.y};
                vop[kp][c] = as_bf16x8(v);
            }
    }

    const float sl2 = p.scale * kLog2e;
    BiasSrc rb = no_bias();
    MaskSrc msk = {make_rsrc(nullptr, 0), 0.f, false};
    if (BM) {
        rb = bias_of_head(p, tc.h);
        msk = mask_of_window(p, tc.w);
    }

#pragma unroll
    for (int t = 0; t < QPW; ++t) {
        const int qb = tc.qs * QPW + t;
        if (16 * qb >= L) break;  // wave-uniform

        f32x4 s[NB];
#pragma unroll
        for (int jb = 0; jb < NB; ++jb) {
            const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
            s[jb] = mfma_bf16(kop[jb], qop[t], zero);  // s[jb][r] = S[16 qb + n][16 jb + 4g + r]
        }
        const AddendGlobal addend = addend_at(rb, msk, (uint32_t)(16 * qb + n), 4u * g, (uint32_t)L);
        const float inv = softmax_block<NB, BM>(s, sl2, addend, L, g);

        f32x4 oe = {0.f, 0.f, 0.f, 0.f}, oo = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kp = 0; kp < NB2; ++kp) {
            const bf16x8 pop = prob_operand<NB>(s, kp);
            oe = mfma_bf16(vop[kp][0], pop, oe);  // oe[r] = O[16 qb + n][2 (4g + r)]
            oo = mfma_bf16(vop[kp][1], pop, oo);  // oo[r] = O[16 qb + n][2 (4g + r) + 1]
        }
        u32x4 out;
        out.x = pack_bf16(oe[0] * inv, oo[0] * inv);
        out.y = pack_bf16(oe[1] * inv, oo[1] * inv);
        out.z = pack_bf16(oe[2] * inv, oo[2] * inv);
        out.w = pack_bf16(oe[3] * inv, oo[3] * inv);
        __builtin_amdgcn_raw_buffer_store_b128(out, ro, (uint32_t)(16 * qb + n) * row_out + 16u * g, 0, 0);
    }
}

// ---------------------------------------------------------------- fp32 ----
// Same tile ownership and layouts with v_mfma_f32_16x16x4_f32 (true fp32
// products): k-slot g of step kk stands for channel 8g + kk in QK^T and for
// key 16 jb + 4g + r in step (jb, r) of O^T = V^T P^T.  V is streamed from
// cache per query block instead of being held in registers.
template <int NB, bool BM>
__global__ void __launch_bounds__(64 * kWavesPerBlock) fwd_f32_kernel(FwdArgs p, FwdGeom gm) {
    constexpr int QPW = Tiling<NB>::kQPerWave;
    const int lane = threadIdx.x & 63;
    const int n = lane & 15, g = lane >> 4;
    const TileCoord tc = tile_of_wave(gm, p.heads);
    if (!tc.valid) return;
    const int L = p.L;
    const uint32_t row_bytes = (uint32_t)p.ldq * 4u, row_out = (uint32_t)p.ldo * 4u;
    const uint32_t tile_bytes = (uint32_t)(L - 1) * row_bytes + 4u * kHeadDim;
    const size_t tile = ((size_t)tc.w * L * p.ldq + (size_t)tc.h * kHeadDim) * 4u;
    const __amdgpu_buffer_rsrc_t rq = make_rsrc((const char*)p.q + tile, tile_bytes);
    const __amdgpu_buffer_rsrc_t rk = make_rsrc((const char*)p.k + tile, tile_bytes);
    const __amdgpu_buffer_rsrc_t rv = make_rsrc((const char*)p.v + tile, tile_bytes);
    const __amdgpu_buffer_rsrc_t ro = make_rsrc((char*)p.o + ((size_t)tc.w * L * p.ldo + (size_t)tc.h * kHeadDim) * 4u,
                                                (uint32_t)(L - 1) * row_out + 4u * kHeadDim);
    const uint32_t off_row = (uint32_t)n * row_bytes + 32u * g;  // channels 8g..8g+7 of row n
    const uint32_t off_v = 4u * g * row_bytes + 4u * n;          // channel n of row 4g

    float kop[NB][8];
#pragma unroll
    for (int jb = 0; jb < NB; ++jb) {
        const f32x4 a = load_f32x4(rk, off_row + 16 * jb * row_bytes);
        const f32x4 b = load_f32x4(rk, off_row + 16 + 16 * jb * row_bytes);
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            kop[jb][c] = a[c];
            kop[jb][4 + c] = b[c];
        }
    }
    BiasSrc rb = no_bias();
    MaskSrc msk = {make_rsrc(nullptr, 0), 0.f, false};
    if (BM) {
        rb = bias_of_head(p, tc.h);
        msk = mask_of_window(p, tc.w);
    }

    for (int t = 0; t < QPW; ++t) {
        const int qb = tc.qs * QPW + t;
        if (16 * qb >= L) break;
        float qop[8];
        {
            const f32x4 a = load_f32x4(rq, off_row + 16 * qb * row_bytes);
            const f32x4 b = load_f32x4(rq, off_row + 16 + 16 * qb * row_bytes);
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                qop[c] = a[c];
                qop[4 + c] = b[c];
            }
        }
        f32x4 s[NB], add[NB];
        if (BM) addend_at(rb, msk, (uint32_t)(16 * qb + n), 4u * g, (uint32_t)L).fill(add, 1.0f);
        float m = -INFINITY;
#pragma unroll
        for (int jb = 0; jb < NB; ++jb) {
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kk = 0; kk < 8; ++kk) acc = mfma_f32(kop[jb][kk], qop[kk], acc);
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                float x = BM ? acc[r] * p.scale + add[jb][r] : acc[r] * p.scale;
                if (jb == NB - 1 && 16 * jb + 4 * g + r >= L) x = -INFINITY;
                acc[r] = x;
                m = fmaxf(m, x);
            }
            s[jb] = acc;
        }
        m = max_over_g(m);
        float sum = 0.f;
#pragma unroll
        for (int jb = 0; jb < NB; ++jb)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float e = __builtin_amdgcn_exp2f((s[jb][r] - m) * kLog2e);
                s[jb][r] = e;
                sum += e;
            }
        sum = sum_over_g(sum);

        f32x4 o0 = {0.f, 0.f, 0.f, 0.f}, o1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int jb = 0; jb < NB; ++jb)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const uint32_t so = (uint32_t)(16 * jb + r) * row_bytes;
                const float v0 = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rv, off_v + so, 0, 0));
                const float v1 = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rv, off_v + 64 + so, 0, 0));
                o0 = mfma_f32(v0, s[jb][r], o0);  // o0[r'] = O[16 qb + n][4g + r']
                o1 = mfma_f32(v1, s[jb][r], o1);  // o1[r'] = O[16 qb + n][16 + 4g + r']
            }
        const uint32_t off_o = (uint32_t)(16 * qb + n) * row_out + 16u * g;
        store_f32x4(o0 / sum, ro, off_o);
        store_f32x4(o1 / sum, ro, off_o + 64);
    }
}

// Heads are 64 B (bf16) slices of a row, so neighbouring heads share 128 B
// memory lines: the waves of a workgroup take neighbouring heads (all heads of
// the window when there are at most 4).  Only when line-sharing heads still end
// up in different workgroups (an odd number of heads per workgroup) is the
// XCD-aware block order used, to keep them on one L2; otherwise the plain order
// is faster (it spreads neighbouring windows over all XCDs and HBM channels).
template <int NB>
FwdGeom make_geom(const FwdArgs& a, unsigned* grid, unsigned* block) {
    FwdGeom gm;
    const int qsplit = Tiling<NB>::kQSplit;
    int hpb = kWavesPerBlock / qsplit;  // heads per workgroup
    if (a.heads < hpb) hpb = a.heads;
    const uint32_t groups = (uint32_t)((a.heads + hpb - 1) / hpb);
    gm.groups = make_fastdiv(groups);
    gm.heads_per_block = (uint32_t)hpb;
    gm.qsplit_log2 = Tiling<NB>::kQSplitLog2;
    const uint32_t nblocks = (uint32_t)(a.N * groups);
    gm.xcd_remap = (groups > 1 && hpb % 2 == 1) ? 1u : 0u;
    gm.xcd_q = nblocks / 8u;
    gm.xcd_r = nblocks % 8u;
    *grid = nblocks;
    *block = 64u * (unsigned)(hpb * qsplit);
    return gm;
}

template <int NB>
hipError_t launch_bf16_nb(const FwdArgs& a, hipStream_t st) {
    unsigned grid, block;
    const FwdGeom gm = make_geom<NB>(a, &grid, &block);
    if (a.bias || has_mask(a))
        hipLaunchKernelGGL((fwd_bf16_kernel<NB, true>), dim3(grid), dim3(block), 0, st, a, gm);
    else
        hipLaunchKernelGGL((fwd_bf16_kernel<NB, false>), dim3(grid), dim3(block), 0, st, a, gm);
    return hipGetLastError();
}

template <int NB>
hipError_t launch_f32_nb(const FwdArgs& a, hipStream_t st) {
    unsigned grid, block;
    const FwdGeom gm = make_geom<NB>(a, &grid, &block);
    if (a.bias || has_mask(a))
        hipLaunchKernelGGL((fwd_f32_kernel<NB, true>), dim3(grid), dim3(block), 0, st, a, gm);
    else
        hipLaunchKernelGGL((fwd_f32_kernel<NB, false>), dim3(grid), dim3(block), 0, st, a, gm);
    return hipGetLastError();
}

}  // namespace

#define FWA_NB_SWITCH(FN, NBV, ...)                                   \
    switch (NBV) {                                                    \
        case 1: return FN<1>(__VA_ARGS__);                            \
        case 2: return FN<2>(__VA_ARGS__);                            \
        case 3: return FN<3>(__VA_ARGS__);                            \
        case 4: return FN<4>(__VA_ARGS__);                            \
        case 5: return FN<5>(__VA_ARGS__);                            \
        case 6: return FN<6>(__VA_ARGS__);                            \
        case 7: return FN<7>(__VA_ARGS__);                            \
        case 8: return FN<8>(__VA_ARGS__);                            \
        case 9: return FN<9>(__VA_ARGS__);                            \
        case 10: return FN<10>(__VA_ARGS__);                          \
        case 11: return FN<11>(__VA_ARGS__);                          \
        case 12: return FN<12>(__VA_ARGS__);                          \
        case 13: return FN<13>(__VA_ARGS__);                          \
        case 14: return FN<14>(__VA_ARGS__);                          \
        case 15: return FN<15>(__VA_ARGS__);                          \
        case 16: return FN<16>(__VA_ARGS__);                          \
        default: return hipErrorInvalidValue;                         \
    }

// bf16 dispatch: windows of up to 64 tokens whose heads form whole 128-byte lines per
// workgroup take the LDS-staged kernel, longer windows the LDS row-blocked kernel (both in
// fwa_forward_staged.hip).  The direct kernel above remains for L <= 64 with an odd number of
// heads greater than 4, where no such grouping exists.
hipError_t launch_forward_bf16(const FwdArgs& a, hipStream_t s) {
    if (staged_heads_per_block(a.L, a.heads) > 0) return launch_forward_bf16_staged(a, s);
    switch ((a.L + 15) / 16) {
        case 1: return launch_bf16_nb<1>(a, s);
        case 2: return launch_bf16_nb<2>(a, s);
        case 3: return launch_bf16_nb<3>(a, s);
        case 4: return launch_bf16_nb<4>(a, s);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_forward_f32(const FwdArgs& a, hipStream_t s) {
    const int nb = (a.L + 15) / 16;
    FWA_NB_SWITCH(launch_f32_nb, nb, a, s)
}

}  // namespace fwa
