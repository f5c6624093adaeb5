// Backward (paper Algorithm 2) for 64 < L <= 256: the score matrix of a tile no longer fits
// the registers of a few waves, so it is produced twice, block by block, in the two
// orientations the two kinds of output need, and never leaves the registers.
//
// A workgroup of W = ceil(NB / 2) waves (NB = ceil(L / 16) blocks of 16 rows) owns one head,
// parks the K, V, Q, dO slabs of the current window in LDS and walks the windows
// bw, bw + G, ...  Per window:
//
//   pass 1, wave <-> 16-query block qb ("query on the lane": lane (g, n), slot r of key block
//   jb stands for query 16 qb + n and key 16 jb + 4g + r):
//       S^T = K Q^T for all key blocks, + bias + mask, row max, exp, row sum
//       delta_i = sum_j P_ij dP_ij with dP^T = V dO^T produced block by block
//       M_i = max_i + log2(sum_i) and delta_i go to LDS for pass 2
//       dQ rows of the block: dS^T is already the operand of dQ^T = K^T dS^T (dP recomputed
//       block by block; K^T through the transposing LDS read)
//   pass 2, wave <-> 16-key block jb ("key on the lane": lane (g, n), slot r of query block qb
//   stands for query 16 qb + 4g + r and key 16 jb + n):
//       S = Q K^T and dP = dO V^T block by block, P = exp2(score - M_i), dS = P (dP - delta_i):
//       the accumulator layout is exactly the operand layout of dV^T = dO^T P and dK^T = Q^T dS
//       with the queries on the k-slots, so P and dS go straight back into the matrix cores.
//
// Nothing is transposed and no L x L tile is ever stored; the price is a second S / dP / exp.
// P and dS enter the matrix cores as hi + lo bf16 pairs (16 significant bits), as in the
// kernels for small windows.
//
// Additive term: in pass 2 a lane needs B[i][j] for 4 queries and one key, 16 lanes cover 16
// consecutive keys: dword loads, 64 contiguous bytes per 16 lanes.  In pass 1 a lane needs 4
// consecutive keys of one query row and neighbouring lanes sit in different rows, which the
// memory pipeline serves a lane at a time; there the wave copies 16 rows x 64 columns at a time
// with row-contiguous 16-byte loads into a private LDS patch and picks its values from there.
#include "fwa_device.h"
#include "fwa_internal.h"

namespace fwa {
namespace {

struct LargeGeom {
    uint32_t heads, G;
    uint32_t xcd_q, xcd_r;
};

constexpr int large_waves(int nb) { return (nb + 1) / 2; }

__device__ __forceinline__ bf16x8 pair_operand(bf16x4 a, bf16x4 b) {
    const uint2 ua = __builtin_bit_cast(uint2, a), ub = __builtin_bit_cast(uint2, b);
    return as_bf16x8(u32x4{ua.x, ua.y, ub.x, ub.y});
}

template <int NB, bool BM>
__global__ void __launch_bounds__(64 * large_waves(NB)) bwd_bf16_large_kernel(BwdArgs p, LargeGeom gm) {
    constexpr int W = large_waves(NB);
    constexpr int NB2 = (NB + 1) / 2;
    constexpr int ROWS = 16 * NB;
    constexpr int PASSES = (ROWS + 16 * W - 1) / (16 * W);  // the workgroup moves 16 W slab rows per pass
    constexpr uint32_t STRIDE = 5;                           // slab row: 64 bytes of data + 16 of padding
    constexpr uint32_t SROW = STRIDE * 8;                    // the same in bf16 elements
    constexpr uint32_t SG = 68;                              // patch row: 64 floats + 4 of padding
    extern __shared__ __attribute__((aligned(16))) uint4 lds[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int n = lane & 15, g = lane >> 4;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const uint32_t lb = xcd_logical_block(blockIdx.x, gm.xcd_q, gm.xcd_r);  // heads of a window: one XCD
    const uint32_t h = lb % gm.heads, bw = lb / gm.heads;
    const int L = p.L;
    const uint32_t row_bytes = (uint32_t)p.C * 2u;
    const float sl2 = p.scale * kLog2e;
    const f32x4 zero = {0.f, 0.f, 0.f, 0.f};

    // LDS: slabs [K][V][Q][dO], each [ROWS][STRIDE] uint4; M[ROWS], delta[ROWS]; one patch per wave
    uint4* const lk = lds;
    uint4* const lv = lds + ROWS * STRIDE;
    uint4* const lq = lds + 2 * ROWS * STRIDE;
    uint4* const lg = lds + 3 * ROWS * STRIDE;
    float* const stM = reinterpret_cast<float*>(lds + 4 * ROWS * STRIDE);
    float* const stD = stM + ROWS;
    float* const patch = stD + ROWS + wave * (16 * SG);

    const uint32_t ll = (uint32_t)L * L * 4u;
    const __amdgpu_buffer_rsrc_t rb =
        (BM && p.bias) ? make_rsrc(p.bias + (size_t)h * L * L, ll) : make_rsrc(nullptr, 0);

    const uint32_t srow = (uint32_t)tid >> 2, scol = (uint32_t)tid & 3u;  // slab movement: (row, 16 B column)
    const uint32_t tile_bytes = (uint32_t)(L - 1) * row_bytes + 2u * kHeadDim;
    const uint32_t trs = (4u * g + (n >> 2)) * SROW + 4u * (n & 3);  // transposing-read base inside a slab
    const uint32_t opd = (uint32_t)n * STRIDE + g;                   // row operand of block b: slab[opd + 16 b STRIDE]
    const uint32_t off_half = (uint32_t)n * row_bytes + 8u * g;      // channels 4g..4g+3 of row n (+32 B: 16+4g..)
    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

    for (uint32_t w = bw; w < (uint32_t)p.N; w += gm.G) {
        const size_t tile = ((size_t)w * L * p.C + (size_t)h * kHeadDim) * 2u;
        {
            const __amdgpu_buffer_rsrc_t rk = make_rsrc((const char*)p.k + tile, tile_bytes);
            const __amdgpu_buffer_rsrc_t rv = make_rsrc((const char*)p.v + tile, tile_bytes);
            const __amdgpu_buffer_rsrc_t rq = make_rsrc((const char*)p.q + tile, tile_bytes);
            const __amdgpu_buffer_rsrc_t rg = make_rsrc((const char*)p.d_o + tile, tile_bytes);
            u32x4 pk[PASSES], pv[PASSES], pq[PASSES], pg[PASSES];
#pragma unroll
            for (int t = 0; t < PASSES; ++t) {
                const uint32_t off = (16 * W * t + srow) * row_bytes + scol * 16u;  // rows beyond L arrive as zeros
                pk[t] = __builtin_amdgcn_raw_buffer_load_b128(rk, off, 0, 0);
                pv[t] = __builtin_amdgcn_raw_buffer_load_b128(rv, off, 0, 0);
                pq[t] = __builtin_amdgcn_raw_buffer_load_b128(rq, off, 0, 0);
                pg[t] = __builtin_amdgcn_raw_buffer_load_b128(rg, off, 0, 0);
            }
#pragma unroll
            for (int t = 0; t < PASSES; ++t) {
                const uint32_t row = 16 * W * t + srow;
                if (row < (uint32_t)ROWS) {
                    lk[row * STRIDE + scol] = __builtin_bit_cast(uint4, pk[t]);
                    lv[row * STRIDE + scol] = __builtin_bit_cast(uint4, pv[t]);
                    lq[row * STRIDE + scol] = __builtin_bit_cast(uint4, pq[t]);
                    lg[row * STRIDE + scol] = __builtin_bit_cast(uint4, pg[t]);
                }
            }
        }
        __syncthreads();
        const __amdgpu_buffer_rsrc_t rm =
            (BM && p.mask) ? make_rsrc(p.mask + (size_t)(w % (uint32_t)p.nW) * L * L, ll) : make_rsrc(nullptr, 0);

        // ---------------- pass 1: query blocks wave, wave + W ----------------
        for (int qb = (int)wave; qb < NB; qb += W) {
            const bf16x8 qop = __builtin_bit_cast(bf16x8, lq[opd + 16 * qb * STRIDE]);
            const bf16x8 gop = __builtin_bit_cast(bf16x8, lg[opd + 16 * qb * STRIDE]);
            f32x4 s[NB];
#pragma unroll
            for (int jb = 0; jb < NB; ++jb)
                s[jb] = mfma_bf16(__builtin_bit_cast(bf16x8, lk[opd + 16 * jb * STRIDE]), qop, zero);
            if (BM) {
                // rows 16 qb .. 16 qb + 15 of (bias + mask), 64 columns at a time: lane -> (row 4t + lane / 16,
                // columns 4 (lane % 16) ..), 256 contiguous bytes per 16 lanes; rows beyond L lie outside the
                // descriptors and read as zero, columns beyond L are overwritten with -inf below
                const uint32_t prow = (uint32_t)lane >> 4, pcol = 4u * ((uint32_t)lane & 15u);
#pragma unroll
                for (int ch = 0; ch < (NB + 3) / 4; ++ch) {
                    f32x4 t4[4];
#pragma unroll
                    for (int t = 0; t < 4; ++t) {
                        const uint32_t off = ((uint32_t)(16 * qb + 4 * t + prow) * L + 64 * ch + pcol) * 4u;
                        t4[t] = (load_f32x4(rb, off) + load_f32x4(rm, off)) * kLog2e;
                    }
#pragma unroll
                    for (int t = 0; t < 4; ++t) *reinterpret_cast<f32x4*>(patch + (4 * t + prow) * SG + pcol) = t4[t];
#pragma unroll
                    for (int b = 0; b < 4; ++b) {
                        const int jb = 4 * ch + b;
                        if (jb < NB) {
                            const f32x4 a = *reinterpret_cast<const f32x4*>(patch + n * SG + 16 * b + 4 * g);
#pragma unroll
                            for (int r = 0; r < 4; ++r) s[jb][r] = fmaf(s[jb][r], sl2, a[r]);
                        }
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            } else {
#pragma unroll
                for (int jb = 0; jb < NB; ++jb) s[jb] *= sl2;
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
            for (int jb = 0; jb < NB; ++jb) {
                const f32x4 dp = mfma_bf16(__builtin_bit_cast(bf16x8, lv[opd + 16 * jb * STRIDE]), gop, zero);
#pragma unroll
                for (int r = 0; r < 4; ++r) delta = fmaf(s[jb][r], dp[r], delta);
            }
            delta = sum_over_g(delta) * inv;
            if (g == 0) {
                stM[16 * qb + n] = m + __builtin_amdgcn_logf(sum);  // p_ij = exp2(score_ij - M_i)
                stD[16 * qb + n] = delta;
            }
            // dQ^T = K^T dS^T over pairs of key blocks
            f32x4 q0 = zero, q1 = zero;  // dQ[16 qb + n][4g + r], dQ[16 qb + n][16 + 4g + r]
            const uint16_t* lk16 = reinterpret_cast<const uint16_t*>(lk) + trs;
#pragma unroll
            for (int kp = 0; kp < NB2; ++kp) {
                const bool two = 2 * kp + 1 < NB;
                bf16x4 hi[2], lo[2];
                hi[1] = lo[1] = as_bf16x4(uint2{0u, 0u});
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    if (u == 1 && !two) break;
                    const int jb = 2 * kp + u;
                    const f32x4 dp = mfma_bf16(__builtin_bit_cast(bf16x8, lv[opd + 16 * jb * STRIDE]), gop, zero);
                    f32x4 ds;
#pragma unroll
                    for (int r = 0; r < 4; ++r) ds[r] = s[jb][r] * inv * (dp[r] - delta);
                    split_hi_lo(ds, hi[u], lo[u]);
                }
                const bf16x8 dh = pair_operand(hi[0], hi[1]), dl = pair_operand(lo[0], lo[1]);
                const bf16x8 k0 = operand_tr(lk16 + (32 * kp) * SROW, 16 * SROW, two);
                const bf16x8 k1 = operand_tr(lk16 + (32 * kp) * SROW + 16, 16 * SROW, two);
                q0 = mfma_bf16(k0, dh, q0);
                q1 = mfma_bf16(k1, dh, q1);
                q0 = mfma_bf16(k0, dl, q0);
                q1 = mfma_bf16(k1, dl, q1);
                __builtin_amdgcn_sched_barrier(0);
            }
            const u32x2 lo2 = {pack_bf16(q0[0] * p.scale, q0[1] * p.scale), pack_bf16(q0[2] * p.scale, q0[3] * p.scale)};
            const u32x2 hi2 = {pack_bf16(q1[0] * p.scale, q1[1] * p.scale), pack_bf16(q1[2] * p.scale, q1[3] * p.scale)};
            const __amdgpu_buffer_rsrc_t rdq = make_rsrc((char*)p.dq + tile, tile_bytes);
            __builtin_amdgcn_raw_buffer_store_b64(lo2, rdq, off_half + 16 * qb * row_bytes, 0, 0);
            __builtin_amdgcn_raw_buffer_store_b64(hi2, rdq, off_half + 32 + 16 * qb * row_bytes, 0, 0);
        }
        __syncthreads();

        // ---------------- pass 2: key blocks wave, wave + W ----------------
        for (int jb = (int)wave; jb < NB; jb += W) {
            const bf16x8 kop = __builtin_bit_cast(bf16x8, lk[opd + 16 * jb * STRIDE]);
            const bf16x8 vop = __builtin_bit_cast(bf16x8, lv[opd + 16 * jb * STRIDE]);
            const uint32_t jcol = 16u * jb + n;
            const bool valid = jcol < (uint32_t)L;
            f32x4 v0 = zero, v1 = zero, k0 = zero, k1 = zero;  // dV, dK [16 jb + n][4g + r] and [..][16 + 4g + r]
            const uint16_t* lg16 = reinterpret_cast<const uint16_t*>(lg) + trs;
            const uint16_t* lq16 = reinterpret_cast<const uint16_t*>(lq) + trs;
#pragma unroll
            for (int qp = 0; qp < NB2; ++qp) {
                const bool two = 2 * qp + 1 < NB;
                bf16x4 ph[2], pl[2], sh[2], sl[2];
                ph[1] = pl[1] = sh[1] = sl[1] = as_bf16x4(uint2{0u, 0u});
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    if (u == 1 && !two) break;
                    const int qb = 2 * qp + u;
                    f32x4 add = zero;
                    if (BM) {
                        // rows beyond L lie outside the descriptors; a key beyond L gets p = 0 below
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            const uint32_t off = ((uint32_t)(16 * qb + 4 * g + r) * L + jcol) * 4u;
                            add[r] = (load_f32(rb, off) + load_f32(rm, off)) * kLog2e;
                        }
                    }
                    const f32x4 sc = mfma_bf16(__builtin_bit_cast(bf16x8, lq[opd + 16 * qb * STRIDE]), kop, zero);
                    const f32x4 dp = mfma_bf16(__builtin_bit_cast(bf16x8, lg[opd + 16 * qb * STRIDE]), vop, zero);
                    const f32x4 M4 = *reinterpret_cast<const f32x4*>(stM + 16 * qb + 4 * g);
                    const f32x4 D4 = *reinterpret_cast<const f32x4*>(stD + 16 * qb + 4 * g);
                    f32x4 pr, ds;
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const float x = BM ? fmaf(sc[r], sl2, add[r]) - M4[r] : fmaf(sc[r], sl2, -M4[r]);
                        pr[r] = valid ? __builtin_amdgcn_exp2f(x) : 0.f;
                        ds[r] = pr[r] * (dp[r] - D4[r]);
                    }
                    split_hi_lo(pr, ph[u], pl[u]);
                    split_hi_lo(ds, sh[u], sl[u]);
                }
                const bf16x8 PH = pair_operand(ph[0], ph[1]), PL = pair_operand(pl[0], pl[1]);
                const bf16x8 SH = pair_operand(sh[0], sh[1]), SL = pair_operand(sl[0], sl[1]);
                // dO^T and Q^T of the 32 queries (channel on the lane)
                const bf16x8 g0 = operand_tr(lg16 + (32 * qp) * SROW, 16 * SROW, two);
                const bf16x8 g1 = operand_tr(lg16 + (32 * qp) * SROW + 16, 16 * SROW, two);
                const bf16x8 x0 = operand_tr(lq16 + (32 * qp) * SROW, 16 * SROW, two);
                const bf16x8 x1 = operand_tr(lq16 + (32 * qp) * SROW + 16, 16 * SROW, two);
                v0 = mfma_bf16(g0, PH, v0);
                v1 = mfma_bf16(g1, PH, v1);
                k0 = mfma_bf16(x0, SH, k0);
                k1 = mfma_bf16(x1, SH, k1);
                v0 = mfma_bf16(g0, PL, v0);
                v1 = mfma_bf16(g1, PL, v1);
                k0 = mfma_bf16(x0, SL, k0);
                k1 = mfma_bf16(x1, SL, k1);
                __builtin_amdgcn_sched_barrier(0);  // keep the next pair's loads from being hoisted over this one
            }
            const u32x2 va = {pack_bf16(v0[0], v0[1]), pack_bf16(v0[2], v0[3])};
            const u32x2 vb = {pack_bf16(v1[0], v1[1]), pack_bf16(v1[2], v1[3])};
            const u32x2 ka = {pack_bf16(k0[0] * p.scale, k0[1] * p.scale), pack_bf16(k0[2] * p.scale, k0[3] * p.scale)};
            const u32x2 kb = {pack_bf16(k1[0] * p.scale, k1[1] * p.scale), pack_bf16(k1[2] * p.scale, k1[3] * p.scale)};
            const __amdgpu_buffer_rsrc_t rdv = make_rsrc((char*)p.dv + tile, tile_bytes);
            const __amdgpu_buffer_rsrc_t rdk = make_rsrc((char*)p.dk + tile, tile_bytes);
            __builtin_amdgcn_raw_buffer_store_b64(va, rdv, off_half + 16 * jb * row_bytes, 0, 0);
            __builtin_amdgcn_raw_buffer_store_b64(vb, rdv, off_half + 32 + 16 * jb * row_bytes, 0, 0);
            __builtin_amdgcn_raw_buffer_store_b64(ka, rdk, off_half + 16 * jb * row_bytes, 0, 0);
            __builtin_amdgcn_raw_buffer_store_b64(kb, rdk, off_half + 32 + 16 * jb * row_bytes, 0, 0);
        }
        __syncthreads();  // the slabs are rewritten for the next window
    }
}

template <int NB, bool BM>
hipError_t launch_large_one(const BwdArgs& a, hipStream_t st) {
    constexpr int W = large_waves(NB);
    const void* fn = reinterpret_cast<const void*>(&bwd_bf16_large_kernel<NB, BM>);
    const unsigned block = 64u * W;
    const size_t lds = (size_t)4 * 16 * NB * 5 * 16 + (size_t)2 * 16 * NB * 4 + (BM ? (size_t)W * 16 * 68 * 4 : 0);
    // Workgroups one CU holds (LDS and registers decide), asked once per kernel.
    static int per_cu = 0;
    if (per_cu == 0) {
        if (lds > 64 * 1024) {
            const hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
        }
        int nblk = 0;
        const hipError_t e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&nblk, fn, (int)block, lds);
        if (e != hipSuccess) return e;
        per_cu = nblk < 1 ? 1 : nblk;
    }
    LargeGeom gm;
    gm.heads = (uint32_t)a.heads;
    long long G = 256LL * per_cu / a.heads;  // one resident workgroup per slot and head
    if (G < 1) G = 1;
    if (G > a.N) G = a.N;
    gm.G = (uint32_t)G;
    const unsigned grid = gm.G * gm.heads;
    gm.xcd_q = grid / 8u;
    gm.xcd_r = grid % 8u;
    hipLaunchKernelGGL((bwd_bf16_large_kernel<NB, BM>), dim3(grid), dim3(block), lds, st, a, gm);
    return hipGetLastError();
}

template <int NB>
hipError_t launch_large_nb(const BwdArgs& a, hipStream_t st) {
    return (a.bias || a.mask) ? launch_large_one<NB, true>(a, st) : launch_large_one<NB, false>(a, st);
}

}  // namespace

hipError_t launch_backward_bf16_large(const BwdArgs& a, hipStream_t s) {
    if (a.dbias != nullptr) return hipErrorNotSupported;
    switch ((a.L + 15) / 16) {
        case 5: return launch_large_nb<5>(a, s);
        case 6: return launch_large_nb<6>(a, s);
        case 7: return launch_large_nb<7>(a, s);
        case 8: return launch_large_nb<8>(a, s);
        case 9: return launch_large_nb<9>(a, s);
        case 10: return launch_large_nb<10>(a, s);
        case 11: return launch_large_nb<11>(a, s);
        case 12: return launch_large_nb<12>(a, s);
        case 13: return launch_large_nb<13>(a, s);
        case 14: return launch_large_nb<14>(a, s);
        case 15: return launch_large_nb<15>(a, s);
        case 16: return launch_large_nb<16>(a, s);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace fwa
