// Cooperative backward kernel (paper Algorithm 2) for L <= 64: four waves per
// (window, head) tile, several heads per workgroup, persistent over windows.
//
// The single-wave kernel (fwa_backward.hip) needs the whole register file for one tile and
// runs two waves per SIMD.  Here the tile is split:
//
//   phase A, wave qb (16 queries, "query on the lane"):
//       S^T = K Q^T, softmax, dP^T = V dO^T, delta, dS          (K, V rows read from LDS)
//       dQ rows of its block (contraction over keys: dS is already the B operand)
//       dBias rows of its block, accumulated in registers across windows
//       P and dS blocks moved to "key on the lane" by an identity product on the matrix core,
//       as hi + lo bf16, and left in an LDS exchange area
//   phase B, wave jb (16 keys):
//       dV, dK rows of its block = contraction over all queries of the exchanged blocks with
//       dO^T resp. Q^T (row operands times a channel selector on the matrix core)
//
// The workgroup loads the Q, K, V, dO slabs of its heads (whole 128-byte lines per row) with
// coalesced 16-byte loads into LDS once per window and requests the next window's slabs before
// computing.  A workgroup keeps its heads and walks the windows bw, bw + G, ...; G is a
// multiple of nW, so (bias[h] + mask[bw % nW]) * log2e is loaded once, into registers.
#include "fwa_device.h"
#include "fwa_internal.h"

namespace fwa {
namespace {

constexpr int kCoopWavesPerTile = 4;
constexpr int kCoopMaxHeads = 3;  // heads per workgroup: 12 waves, 3 per SIMD, <= 170 VGPRs each

struct CoopGeom {
    FastDiv groups;         // workgroups per window position
    FastDiv lanes_per_row;  // 4 * heads_per_block
    uint32_t heads_per_block;
    uint32_t G;             // window positions walked in parallel (= dBias slots)
};

template <int NB, bool BM, bool DB>
__global__ void __launch_bounds__(64 * kCoopWavesPerTile * kCoopMaxHeads) bwd_bf16_coop_kernel(BwdArgs p, CoopGeom gm) {
    constexpr int NB2 = (NB + 1) / 2;
    constexpr int ROWS = 16 * NB;
    extern __shared__ __attribute__((aligned(16))) uint4 lds[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int n = lane & 15, g = lane >> 4;
    const uint32_t wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const uint32_t hl = wv >> 2;            // head inside the workgroup
    const int role = (int)(wv & 3u);        // query block in phase A, key block in phase B
    const uint32_t bw = fastdiv(blockIdx.x, gm.groups);
    const uint32_t hg = blockIdx.x - bw * gm.groups.d;
    const uint32_t hpb = gm.heads_per_block;
    const uint32_t h = hg * hpb + hl;
    const int L = p.L;
    const uint32_t row_bytes = (uint32_t)p.C * 2u;
    const uint32_t stride = 4u * hpb + 1u;  // slab row stride in 16-byte units
    const float sl2 = p.scale * kLog2e;
    const bool active = role < NB;

    // LDS: slabs [K][V][Q][dO], each [ROWS][stride] uint4; then per head the exchange area
    // [jb][qb][P_hi, P_lo, dS_hi, dS_lo][lane] of 8 bytes.
    uint4* const lk = lds;
    uint4* const lv = lds + ROWS * stride;
    uint4* const lq = lds + 2 * ROWS * stride;
    uint4* const lg = lds + 3 * ROWS * stride;
    uint2* const ex = reinterpret_cast<uint2*>(lds + 4 * ROWS * stride) + (size_t)hl * (NB * NB * 4 * 64) + lane;
    const uint32_t opd = (uint32_t)n * stride + 4u * hl + g;  // operand of row block b: slab[opd + 16 b stride]

    // additive score term of this wave's query rows, in registers (see the file comment)
    f32x4 add[NB];
    if (BM && active) {
        const uint32_t ll = (uint32_t)L * L * 4u;
        const __amdgpu_buffer_rsrc_t rb = p.bias ? make_rsrc(p.bias + (size_t)h * L * L, ll) : make_rsrc(nullptr, 0);
        const __amdgpu_buffer_rsrc_t rm =
            p.mask ? make_rsrc(p.mask + (size_t)(bw % (uint32_t)p.nW) * L * L, ll) : make_rsrc(nullptr, 0);
        const uint32_t off = (((uint32_t)(16 * role + n)) * L + 4u * g) * 4u;
#pragma unroll
        for (int jb = 0; jb < NB; ++jb)
            add[jb] = (load_f32x4(rb, off + 16 * jb * 4u) + load_f32x4(rm, off + 16 * jb * 4u)) * kLog2e;
    }
    f32x4 dbacc[NB];
#pragma unroll
    for (int jb = 0; jb < NB; ++jb) dbacc[jb] = f32x4{0.f, 0.f, 0.f, 0.f};

    const bf16x4 ident = identity_operand(g, n);
    const bf16x8 sel_even = channel_selector(g, n, 0), sel_odd = channel_selector(g, n, 1);
    const f32x4 zero = {0.f, 0.f, 0.f, 0.f};

    // slab movement: thread -> (row, 16-byte column); one pass covers 64 rows
    const uint32_t rip = fastdiv((uint32_t)tid, gm.lanes_per_row);
    const uint32_t col = (uint32_t)tid - rip * gm.lanes_per_row.d;
    const uint32_t slab_bytes = (uint32_t)(L - 1) * row_bytes + hpb * 2u * kHeadDim;
    const uint32_t goff = rip * row_bytes + col * 16u;
    const uint32_t loff = rip * stride + col;
    u32x4 pk, pv, pq, pg;
    auto request = [&](uint32_t w) {
        const size_t slab = ((size_t)w * L * p.C + (size_t)hg * hpb * kHeadDim) * 2u;
        // rows beyond L lie outside the descriptors and arrive as zeros
        pk = __builtin_amdgcn_raw_buffer_load_b128(make_rsrc((const char*)p.k + slab, slab_bytes), goff, 0, 0);
        pv = __builtin_amdgcn_raw_buffer_load_b128(make_rsrc((const char*)p.v + slab, slab_bytes), goff, 0, 0);
        pq = __builtin_amdgcn_raw_buffer_load_b128(make_rsrc((const char*)p.q + slab, slab_bytes), goff, 0, 0);
        pg = __builtin_amdgcn_raw_buffer_load_b128(make_rsrc((const char*)p.d_o + slab, slab_bytes), goff, 0, 0);
    };
    if (bw < (uint32_t)p.N) request(bw);

    const uint32_t tile_bytes = (uint32_t)(L - 1) * row_bytes + 2u * kHeadDim;
    const uint32_t off_row = (uint32_t)n * row_bytes + 16u * g;

    for (uint32_t w = bw; w < (uint32_t)p.N; w += gm.G) {
        if (rip < (uint32_t)ROWS) {
            lk[loff] = __builtin_bit_cast(uint4, pk);
            lv[loff] = __builtin_bit_cast(uint4, pv);
            lq[loff] = __builtin_bit_cast(uint4, pq);
            lg[loff] = __builtin_bit_cast(uint4, pg);
        }
        if (w + gm.G < (uint32_t)p.N) request(w + gm.G);  // in flight while this window is computed
        __syncthreads();

        const size_t tile = ((size_t)w * L * p.C + (size_t)h * kHeadDim) * 2u;
        // ---------------- phase A: query block `role` ----------------
        if (active) {
            const int qb = role;
            const bf16x8 qop = __builtin_bit_cast(bf16x8, lq[opd + 16 * qb * stride]);
            const bf16x8 gop = __builtin_bit_cast(bf16x8, lg[opd + 16 * qb * stride]);
            f32x4 s[NB], dp[NB];
#pragma unroll
            for (int jb = 0; jb < NB; ++jb) {
                s[jb] = mfma_bf16(__builtin_bit_cast(bf16x8, lk[opd + 16 * jb * stride]), qop, zero);
                dp[jb] = mfma_bf16(__builtin_bit_cast(bf16x8, lv[opd + 16 * jb * stride]), gop, zero);
            }
#pragma unroll
            for (int jb = 0; jb < NB; ++jb) {
                if (BM) {
#pragma unroll
                    for (int r = 0; r < 4; ++r) s[jb][r] = fmaf(s[jb][r], sl2, add[jb][r]);
                } else {
                    s[jb] *= sl2;
                }
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
            m = max_over_g(m);
            float sum = 0.f;
#pragma unroll
            for (int jb = 0; jb < NB; ++jb)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const float e = __builtin_amdgcn_exp2f(s[jb][r] - m);
                    s[jb][r] = e;
                    sum += e;
                }
            sum = sum_over_g(sum);
            const float inv = __builtin_amdgcn_rcpf(sum);
            float delta = 0.f;
#pragma unroll
            for (int jb = 0; jb < NB; ++jb)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    s[jb][r] *= inv;  // P
                    delta = fmaf(s[jb][r], dp[jb][r], delta);
                }
            delta = sum_over_g(delta);
#pragma unroll
            for (int jb = 0; jb < NB; ++jb) {
#pragma unroll
                for (int r = 0; r < 4; ++r) dp[jb][r] = s[jb][r] * (dp[jb][r] - delta);  // dS
                if (DB) dbacc[jb] += dp[jb];
            }
            // hi + lo bf16 parts; the blocks with the key on the lane go to the exchange area
            bf16x4 ds_hi[NB], ds_lo[NB];
#pragma unroll
            for (int jb = 0; jb < NB; ++jb) {
                bf16x4 p_hi, p_lo;
                split_hi_lo(s[jb], p_hi, p_lo);
                split_hi_lo(dp[jb], ds_hi[jb], ds_lo[jb]);
                uint2* slot = ex + ((jb * NB + qb) * 4) * 64;
                slot[0 * 64] = pack_exact_u2(mfma16(p_hi, ident, zero));
                slot[1 * 64] = pack_exact_u2(mfma16(p_lo, ident, zero));
                slot[2 * 64] = pack_exact_u2(mfma16(ds_hi[jb], ident, zero));
                slot[3 * 64] = pack_exact_u2(mfma16(ds_lo[jb], ident, zero));
            }
            // dQ^T = K^T dS^T over pairs of key blocks
            f32x4 qe = zero, qo = zero;
#pragma unroll
            for (int kp = 0; kp < NB2; ++kp) {
                const bool two = 2 * kp + 1 < NB;
                const int j1 = two ? 2 * kp + 1 : 0;
                const bf16x8 k0 = __builtin_bit_cast(bf16x8, lk[opd + 16 * (2 * kp) * stride]);
                const bf16x8 k1 = __builtin_bit_cast(bf16x8, lk[opd + 16 * j1 * stride]);
                const uint2 e0 = pack_exact_u2(mfma_bf16(k0, sel_even, zero)), o0 = pack_exact_u2(mfma_bf16(k0, sel_odd, zero));
                uint2 e1 = {0u, 0u}, o1 = {0u, 0u};
                if (two) {
                    e1 = pack_exact_u2(mfma_bf16(k1, sel_even, zero));
                    o1 = pack_exact_u2(mfma_bf16(k1, sel_odd, zero));
                }
                const uint2 h0 = __builtin_bit_cast(uint2, ds_hi[2 * kp]), l0 = __builtin_bit_cast(uint2, ds_lo[2 * kp]);
                uint2 h1 = {0u, 0u}, l1 = {0u, 0u};
                if (two) {
                    h1 = __builtin_bit_cast(uint2, ds_hi[j1]);
                    l1 = __builtin_bit_cast(uint2, ds_lo[j1]);
                }
                const bf16x8 ke = as_bf16x8(u32x4{e0.x, e0.y, e1.x, e1.y}), ko = as_bf16x8(u32x4{o0.x, o0.y, o1.x, o1.y});
                const bf16x8 dh = as_bf16x8(u32x4{h0.x, h0.y, h1.x, h1.y}), dl = as_bf16x8(u32x4{l0.x, l0.y, l1.x, l1.y});
                qe = mfma_bf16(ke, dh, qe);
                qo = mfma_bf16(ko, dh, qo);
                qe = mfma_bf16(ke, dl, qe);
                qo = mfma_bf16(ko, dl, qo);
            }
            u32x4 out;
            out.x = pack_bf16(qe[0] * p.scale, qo[0] * p.scale);
            out.y = pack_bf16(qe[1] * p.scale, qo[1] * p.scale);
            out.z = pack_bf16(qe[2] * p.scale, qo[2] * p.scale);
            out.w = pack_bf16(qe[3] * p.scale, qo[3] * p.scale);
            __builtin_amdgcn_raw_buffer_store_b128(out, make_rsrc((char*)p.dq + tile, tile_bytes),
                                                   off_row + 16 * qb * row_bytes, 0, 0);
        }
        __syncthreads();
        // ---------------- phase B: key block `role` ----------------
        if (active) {
            const int jb = role;
            f32x4 ve = zero, vo = zero, ke = zero, ko = zero;
#pragma unroll
            for (int qp = 0; qp < NB2; ++qp) {
                const bool two = 2 * qp + 1 < NB;
                const int q1 = two ? 2 * qp + 1 : 0;
                // dO^T and Q^T of the 32 queries: row operands times the channel selectors
                const bf16x8 g0 = __builtin_bit_cast(bf16x8, lg[opd + 16 * (2 * qp) * stride]);
                const bf16x8 g1 = __builtin_bit_cast(bf16x8, lg[opd + 16 * q1 * stride]);
                const bf16x8 x0 = __builtin_bit_cast(bf16x8, lq[opd + 16 * (2 * qp) * stride]);
                const bf16x8 x1 = __builtin_bit_cast(bf16x8, lq[opd + 16 * q1 * stride]);
                const uint2 ge0 = pack_exact_u2(mfma_bf16(g0, sel_even, zero)), go0 = pack_exact_u2(mfma_bf16(g0, sel_odd, zero));
                const uint2 xe0 = pack_exact_u2(mfma_bf16(x0, sel_even, zero)), xo0 = pack_exact_u2(mfma_bf16(x0, sel_odd, zero));
                uint2 ge1 = {0u, 0u}, go1 = {0u, 0u}, xe1 = {0u, 0u}, xo1 = {0u, 0u};
                const uint2* s0 = ex + ((jb * NB + 2 * qp) * 4) * 64;
                const uint2 ph0 = s0[0 * 64], pl0 = s0[1 * 64], sh0 = s0[2 * 64], sl0 = s0[3 * 64];
                uint2 ph1 = {0u, 0u}, pl1 = {0u, 0u}, sh1 = {0u, 0u}, sl1 = {0u, 0u};
                if (two) {
                    ge1 = pack_exact_u2(mfma_bf16(g1, sel_even, zero));
                    go1 = pack_exact_u2(mfma_bf16(g1, sel_odd, zero));
                    xe1 = pack_exact_u2(mfma_bf16(x1, sel_even, zero));
                    xo1 = pack_exact_u2(mfma_bf16(x1, sel_odd, zero));
                    const uint2* s1 = ex + ((jb * NB + q1) * 4) * 64;
                    ph1 = s1[0 * 64];
                    pl1 = s1[1 * 64];
                    sh1 = s1[2 * 64];
                    sl1 = s1[3 * 64];
                }
                const bf16x8 ge = as_bf16x8(u32x4{ge0.x, ge0.y, ge1.x, ge1.y}), go = as_bf16x8(u32x4{go0.x, go0.y, go1.x, go1.y});
                const bf16x8 xe = as_bf16x8(u32x4{xe0.x, xe0.y, xe1.x, xe1.y}), xo = as_bf16x8(u32x4{xo0.x, xo0.y, xo1.x, xo1.y});
                const bf16x8 ph = as_bf16x8(u32x4{ph0.x, ph0.y, ph1.x, ph1.y}), pl = as_bf16x8(u32x4{pl0.x, pl0.y, pl1.x, pl1.y});
                const bf16x8 sh = as_bf16x8(u32x4{sh0.x, sh0.y, sh1.x, sh1.y}), sl = as_bf16x8(u32x4{sl0.x, sl0.y, sl1.x, sl1.y});
                ve = mfma_bf16(ge, ph, ve);  // dV[16 jb + n][2 (4g + r)]
                vo = mfma_bf16(go, ph, vo);
                ke = mfma_bf16(xe, sh, ke);  // dK[16 jb + n][2 (4g + r)]
                ko = mfma_bf16(xo, sh, ko);
                ve = mfma_bf16(ge, pl, ve);
                vo = mfma_bf16(go, pl, vo);
                ke = mfma_bf16(xe, sl, ke);
                ko = mfma_bf16(xo, sl, ko);
            }
            u32x4 ov, ok;
            ov.x = pack_bf16(ve[0], vo[0]);
            ov.y = pack_bf16(ve[1], vo[1]);
            ov.z = pack_bf16(ve[2], vo[2]);
            ov.w = pack_bf16(ve[3], vo[3]);
            ok.x = pack_bf16(ke[0] * p.scale, ko[0] * p.scale);
            ok.y = pack_bf16(ke[1] * p.scale, ko[1] * p.scale);
            ok.z = pack_bf16(ke[2] * p.scale, ko[2] * p.scale);
            ok.w = pack_bf16(ke[3] * p.scale, ko[3] * p.scale);
            __builtin_amdgcn_raw_buffer_store_b128(ov, make_rsrc((char*)p.dv + tile, tile_bytes),
                                                   off_row + 16 * jb * row_bytes, 0, 0);
            __builtin_amdgcn_raw_buffer_store_b128(ok, make_rsrc((char*)p.dk + tile, tile_bytes),
                                                   off_row + 16 * jb * row_bytes, 0, 0);
        }
        __syncthreads();  // slabs and exchange area are rewritten by the next window
    }

    if (DB && active) {
        float* dst = p.partial + ((size_t)bw * p.heads + h) * L * L;
#pragma unroll
        for (int jb = 0; jb < NB; ++jb)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int i = 16 * role + n, j = 16 * jb + 4 * g + r;
                if (i < L && j < L) dst[(size_t)i * L + j] = dbacc[jb][r];
            }
    }
}

template <int NB, bool BM, bool DB>
hipError_t launch_coop_one(const BwdArgs& a, const CoopGeom& gm, unsigned grid, unsigned block, size_t lds,
                           hipStream_t st) {
    if (lds > 64 * 1024) {
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&bwd_bf16_coop_kernel<NB, BM, DB>),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL((bwd_bf16_coop_kernel<NB, BM, DB>), dim3(grid), dim3(block), lds, st, a, gm);
    return hipGetLastError();
}

template <int NB>
hipError_t launch_coop_nb(const BwdArgs& a, int hpb, hipStream_t st) {
    CoopGeom gm;
    const uint32_t groups = (uint32_t)(a.heads / hpb);
    gm.groups = make_fastdiv(groups);
    gm.lanes_per_row = make_fastdiv(4u * (uint32_t)hpb);
    gm.heads_per_block = (uint32_t)hpb;
    gm.G = (uint32_t)a.slots;
    const unsigned grid = gm.G * groups, block = 64u * kCoopWavesPerTile * (unsigned)hpb;
    const size_t lds = (size_t)4 * 16 * NB * (4 * hpb + 1) * 16 + (size_t)hpb * NB * NB * 4 * 64 * 8;
    const bool bm = a.bias || a.mask, db = a.dbias != nullptr;
    if (bm)
        return db ? launch_coop_one<NB, true, true>(a, gm, grid, block, lds, st)
                  : launch_coop_one<NB, true, false>(a, gm, grid, block, lds, st);
    return db ? launch_coop_one<NB, false, true>(a, gm, grid, block, lds, st)
              : launch_coop_one<NB, false, false>(a, gm, grid, block, lds, st);
}

}  // namespace

// Heads per workgroup of the cooperative kernel: a divisor of `heads` whose slab is whole
// 128-byte lines per row (an even count) or the whole row; 0 = not applicable.
int coop_heads_per_block(int heads) {
    if (heads <= kCoopMaxHeads) return heads;
    if (heads % 2 == 0) return 2;
    if (heads % 3 == 0) return 3;
    return 0;
}

// Window positions walked in parallel: about one workgroup per CU (LDS allows no more), a
// multiple of nW so that every workgroup keeps one mask tile; 0 = the kernel does not apply.
int coop_slots(long long N, int heads, int nW) {
    const int hpb = coop_heads_per_block(heads);
    if (hpb == 0 || nW < 1) return 0;
    const int groups = heads / hpb;
    const int per_cu = hpb == 3 ? 1 : (hpb == 2 ? 1 : 3);
    long long G = (256LL * per_cu / groups) / nW * nW;
    if (G > N) G = N / nW * nW;
    if (G < nW || G <= 0) return 0;
    return (int)G;
}

hipError_t launch_backward_bf16_coop(const BwdArgs& a, hipStream_t s) {
    const int hpb = coop_heads_per_block(a.heads);
    switch ((a.L + 15) / 16) {
        case 1: return launch_coop_nb<1>(a, hpb, s);
        case 2: return launch_coop_nb<2>(a, hpb, s);
        case 3: return launch_coop_nb<3>(a, hpb, s);
        case 4: return launch_coop_nb<4>(a, hpb, s);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace fwa
