// Backward (paper Algorithm 2) for 64 < L <= 256: the score matrix of a tile no longer fits
// the registers of a few waves, so it is produced twice, block by block, in the two
// orientations the two kinds of output need, and never leaves the registers.
//
// A workgroup of W = 4 (NB <= 10) or 8 waves (NB = ceil(L / 16) blocks of 16 rows; a multiple of
// the 4 SIMDs, so that two 4-wave workgroups or one 8-wave workgroup load a CU evenly) owns one head,
// parks the K, V, Q, dO slabs of the current window in LDS and walks the windows
// bw, bw + G, ...  Per window:
//
//   pass 1, wave <-> 16-query blocks qb = wave, wave + W, ... ("query on the lane": lane (g, n), slot r of key block
//   jb stands for query 16 qb + n and key 16 jb + 4g + r):
//       S^T = K Q^T for all key blocks, + bias + mask, row max, exp, row sum
//       delta_i = sum_j P_ij dP_ij with dP^T = V dO^T produced block by block
//       M_i = max_i + log2(sum_i) and delta_i go to LDS for pass 2
//       dQ rows of the block: dS^T is already the operand of dQ^T = K^T dS^T (dP recomputed
//       block by block; K^T through the transposing LDS read)
//   pass 2, wave <-> 16-key blocks jb = wave, wave + W, ... ("key on the lane": lane (g, n), slot r of query block qb
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
#include "fwa_softmax.h"

#include <type_traits>

namespace fwa {
namespace {

struct LargeGeom {
    uint32_t heads, G;
    uint32_t xcd_q, xcd_r;
};

constexpr int large_waves(int nb) { return nb <= 10 ? 4 : 8; }
// Slab rows of the kernel below in 16-byte units: 64 bytes of data and no padding.  Row-operand and transposing
// reads run at the same rate as with 16 bytes of padding (measured), and the smaller workgroup lets a CU hold a third
// one where registers allow (pass 1 alone at L = 100: 294 -> 261 us with dBias).
constexpr uint32_t kLargeStride = 4;
__device__ __forceinline__ bf16x8 pair_operand(bf16x4 a, bf16x4 b) {
    const uint2 ua = __builtin_bit_cast(uint2, a), ub = __builtin_bit_cast(uint2, b);
    return as_bf16x8(u32x4{ua.x, ua.y, ub.x, ub.y});
}

// HB: no bias (0) or an fp32 bias (1; a bf16 bias arrives as an fp32 copy made once per call); HM: no mask (0), a dense mask (1), or region
// labels from which the mask values are formed in registers (2).  What is absent costs neither
// loads nor registers.
// P2 = false: pass 1 only (dQ, and the row statistics to the workspace); dK, dV and dBias are then
// left to bwd_bf16_large_keys_kernel.
template <int NB, int HB, int HM, bool P2>
__global__ void __launch_bounds__(64 * large_waves(NB)) bwd_bf16_large_kernel(BwdArgs p, LargeGeom gm) {
    constexpr bool BM = HB != 0 || HM != 0;
    constexpr int W = large_waves(NB);
    constexpr int NB2 = (NB + 1) / 2;
    constexpr int ROWS = 16 * NB;
    constexpr int PASSES = (ROWS + 16 * W - 1) / (16 * W);  // the workgroup moves 16 W slab rows per pass
    constexpr uint32_t STRIDE = kLargeStride;                // slab row in 16-byte units
    constexpr uint32_t SROW = STRIDE * 8;                    // the same in bf16 elements
    constexpr uint32_t SG = 68;                              // patch row: 64 floats + 4 of padding
    extern __shared__ __attribute__((aligned(16))) uint4 lds[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int n = lane & 15, g = lane >> 4;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const uint32_t lb = xcd_logical_block(blockIdx.x, gm.xcd_q, gm.xcd_r);  // heads of a window: one XCD
    const uint32_t h = lb % gm.heads, bw = lb / gm.heads;
    const int L = p.L;
    // token rows are p.ldq (q, k, v), p.ldg (d_o), p.ldd (dq, dk, dv) elements apart; window w starts at row w L
    const uint32_t row_bytes = (uint32_t)p.ldq * 2u, row_g = (uint32_t)p.ldg * 2u, row_d = (uint32_t)p.ldd * 2u;
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
    const float* const bias32 = static_cast<const float*>(p.bias);
    const __amdgpu_buffer_rsrc_t rb =
        HB == 1 ? make_rsrc(bias32 + (size_t)h * L * L, ll) : make_rsrc(nullptr, 0);

    const uint32_t srow = (uint32_t)tid >> 2, scol = (uint32_t)tid & 3u;  // slab movement: (row, 16 B column)
    const uint32_t tile_bytes = (uint32_t)(L - 1) * row_bytes + 2u * kHeadDim;
    const uint32_t trs = (4u * g + (n >> 2)) * SROW + 4u * (n & 3);  // transposing-read base inside a slab
    const uint32_t opd = (uint32_t)n * STRIDE + g;                   // row operand of block b: slab[opd + 16 b STRIDE]
    const uint32_t tile_bytes_g = (uint32_t)(L - 1) * row_g + 2u * kHeadDim;
    const uint32_t tile_bytes_d = (uint32_t)(L - 1) * row_d + 2u * kHeadDim;
    typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
    // 16 output rows of this wave (64 bytes each: channels 0..15 in `lo`, 16..31 in `hi`, accumulator
    // order) leave through the wave's patch area, free whenever a block's results are ready: written
    // there, read back 16 bytes per lane, one store of 64-byte row pieces instead of two of 32.
    auto store_rows = [&](const u32x2_t lo, const u32x2_t hi, const __amdgpu_buffer_rsrc_t dst, int blk) {
        char* const cell = reinterpret_cast<char*>(patch);
        *reinterpret_cast<u32x2_t*>(cell + n * 80 + g * 8) = lo;
        *reinterpret_cast<u32x2_t*>(cell + n * 80 + 32 + g * 8) = hi;
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        const uint32_t r = (uint32_t)(lane >> 2), c = (uint32_t)(lane & 3);
        const u32x4 rows = *reinterpret_cast<const u32x4*>(cell + r * 80 + c * 16);
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_raw_buffer_store_b128(rows, dst, (uint32_t)(16 * blk + r) * row_d + 16u * c, 0, 0);
    };
    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

    // The slabs of the next window are requested into registers by every wave right before its last stores of the
    // current one -- the big temporaries of the passes are dead by then --, so that their way through memory
    // overlaps with those stores and with the wait for the slowest wave; they are parked between the two barriers
    // that separate the windows.
    u32x4 pk[PASSES], pv[PASSES], pq[PASSES], pg[PASSES];
    auto request = [&](uint32_t w) {
        const size_t tile = ((size_t)w * L * p.ldq + (size_t)h * kHeadDim) * 2u;
        const size_t tile_g = ((size_t)w * L * p.ldg + (size_t)h * kHeadDim) * 2u;
        const __amdgpu_buffer_rsrc_t rk = make_rsrc((const char*)p.k + tile, tile_bytes);
        const __amdgpu_buffer_rsrc_t rv = make_rsrc((const char*)p.v + tile, tile_bytes);
        const __amdgpu_buffer_rsrc_t rq = make_rsrc((const char*)p.q + tile, tile_bytes);
        const __amdgpu_buffer_rsrc_t rg = make_rsrc((const char*)p.d_o + tile_g, tile_bytes_g);
#pragma unroll
        for (int t = 0; t < PASSES; ++t) {
            const uint32_t off = (16 * W * t + srow) * row_bytes + scol * 16u;  // rows beyond L arrive as zeros
            pk[t] = __builtin_amdgcn_raw_buffer_load_b128(rk, off, 0, 0);
            pv[t] = __builtin_amdgcn_raw_buffer_load_b128(rv, off, 0, 0);
            pq[t] = __builtin_amdgcn_raw_buffer_load_b128(rq, off, 0, 0);
            pg[t] = __builtin_amdgcn_raw_buffer_load_b128(rg, (16 * W * t + srow) * row_g + scol * 16u, 0, 0);
        }
    };
    auto park = [&]() {
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
    };
    if (bw < (uint32_t)p.N) {
        request(bw);
        park();
    }

    for (uint32_t w = bw; w < (uint32_t)p.N; w += gm.G) {
        const size_t tile_d = ((size_t)w * L * p.ldd + (size_t)h * kHeadDim) * 2u;
        const bool has_next = w + gm.G < (uint32_t)p.N;
        __syncthreads();  // the slabs are in place
        // dead until the request at the end of this window: said so, or the compiler carries the old values
        // through both passes on behalf of the path on which no request happens
#pragma unroll
        for (int t = 0; t < PASSES; ++t) pk[t] = pv[t] = pq[t] = pg[t] = u32x4{0u, 0u, 0u, 0u};
        // the labels of the window's tokens when the mask comes as labels
        const __amdgpu_buffer_rsrc_t rl =
            HM == 2 ? make_rsrc(p.labels + (size_t)(w % (uint32_t)p.nW) * L, (uint32_t)L * 4u) : make_rsrc(nullptr, 0);

        // ---------------- pass 1: query blocks wave, wave + W ----------------
        for (int qb = (int)wave; qb < NB; qb += W) {
            const bf16x8 qop = __builtin_bit_cast(bf16x8, lq[opd + 16 * qb * STRIDE]);
            const bf16x8 gop = __builtin_bit_cast(bf16x8, lg[opd + 16 * qb * STRIDE]);
            // rows 16 qb .. 16 qb + 15 of (bias + mask), 64 columns at a time: lane -> (row 4t + lane / 16,
            // columns 4 (lane % 16) ..), 256 contiguous bytes per 16 lanes; rows beyond L lie outside the
            // descriptors and read as zero, columns beyond L are overwritten with -inf below.  The first
            // patch is requested before the products are formed, each further one a patch ahead.
            const uint32_t prow = (uint32_t)lane >> 4, pcol = 4u * ((uint32_t)lane & 15u);
            constexpr int CH = (NB + 3) / 4;
            f32x4 tb[2][4], tm[2][4];
            i32x4 tk[2];  // with labels: those of a patch's 4 columns ...
            int tq[4];    // ... and of the lane's 4 patch rows
            const uint32_t qrow = (uint32_t)(16 * qb) * L * 4u;  // < ll: the block starts inside the tile
            const __amdgpu_buffer_rsrc_t rbq = HB == 1 ? make_rsrc(bias32 + (size_t)h * L * L + (size_t)16 * qb * L, ll - qrow) : rb;
            const __amdgpu_buffer_rsrc_t rmq =
                HM == 1 ? make_rsrc(p.mask + (size_t)(w % (uint32_t)p.nW) * L * L + (size_t)16 * qb * L, ll - qrow) : rb;
            if (HM == 2) {
#pragma unroll
                for (int t = 0; t < 4; ++t) tq[t] = load_i32(rl, (uint32_t)(16 * qb + 4 * t + prow) * 4u);
            }
            auto request_patch = [&](int ch, int slot) {
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const uint32_t off = ((uint32_t)(4 * t + prow) * L + pcol) * 4u + 256u * ch;
                    if (HB == 1) tb[slot][t] = load_f32x4(rbq, off);
                    if (HM == 1) tm[slot][t] = load_f32x4(rmq, off);
                }
                if (HM == 2) tk[slot] = load_i32x4(rl, (pcol + 64u * ch) * 4u);
            };
            if (BM) request_patch(0, 0);
            f32x4 s[NB];
#pragma unroll
            for (int jb = 0; jb < NB; ++jb)
                s[jb] = mfma_bf16(__builtin_bit_cast(bf16x8, lk[opd + 16 * jb * STRIDE]), qop, zero);
            if (BM) {
#pragma unroll
                for (int ch = 0; ch < CH; ++ch) {
                    const int cur = ch & 1;
                    if (ch + 1 < CH) request_patch(ch + 1, cur ^ 1);
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int t = 0; t < 4; ++t) {
                        const f32x4 mk = HM == 2 ? mask_of_labels(tq[t], tk[cur], p.mask_value) : tm[cur][t];
                        const f32x4 bq = tb[cur][t];
                        *reinterpret_cast<f32x4*>(patch + (4 * t + prow) * SG + pcol) =
                            (HB && HM ? bq + mk : (HB ? bq : mk)) * kLog2e;
                    }
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
            // s keeps exp(score - max), not normalised: P = s * inv enters delta here and dQ at the very
            // end (one factor per output element instead of one per score)
            float delta = 0.f;
#pragma unroll
            for (int jb = 0; jb < NB; ++jb) {
                const f32x4 dp = mfma_bf16(__builtin_bit_cast(bf16x8, lv[opd + 16 * jb * STRIDE]), gop, zero);
#pragma unroll
                for (int r = 0; r < 4; ++r) delta = fmaf(s[jb][r], dp[r], delta);
            }
            delta = sum_over_g(delta) * inv;
            if (g == 0) {
                const float Mi = m + __builtin_amdgcn_logf(sum);  // p_ij = exp2(score_ij - M_i)
                stM[16 * qb + n] = Mi;
                stD[16 * qb + n] = delta;
                if (p.stats) {  // kept for the dBias kernel, which redoes pass 2 only
                    float* gs = p.stats + ((size_t)w * p.heads + h) * (2 * ROWS) + 16 * qb + n;
                    gs[0] = Mi;
                    gs[ROWS] = delta;
                }
            }
            // dQ^T = K^T dS^T over pairs of key blocks; the operands of the next pair are fetched ahead
            f32x4 q0 = zero, q1 = zero;  // dQ[16 qb + n][4g + r], dQ[16 qb + n][16 + 4g + r]
            const uint16_t* lk16 = reinterpret_cast<const uint16_t*>(lk) + trs;
            bf16x8 ov[2][2], tk0[2], tk1[2];
            auto fetch1 = [&](int kp, int slot) {
                const bool two = 2 * kp + 1 < NB;
                ov[slot][0] = __builtin_bit_cast(bf16x8, lv[opd + 16 * (2 * kp) * STRIDE]);
                if (two) ov[slot][1] = __builtin_bit_cast(bf16x8, lv[opd + 16 * (2 * kp + 1) * STRIDE]);
                tk0[slot] = operand_tr(lk16 + (32 * kp) * SROW, 16 * SROW, two);
                tk1[slot] = operand_tr(lk16 + (32 * kp) * SROW + 16, 16 * SROW, two);
            };
            fetch1(0, 0);
#pragma unroll
            for (int kp = 0; kp < NB2; ++kp) {
                const bool two = 2 * kp + 1 < NB;
                const int cur = kp & 1;
                if (kp + 1 < NB2) fetch1(kp + 1, cur ^ 1);
                __builtin_amdgcn_sched_barrier(0);
                bf16x4 hi[2], lo[2];
                hi[1] = lo[1] = as_bf16x4(uint2{0u, 0u});
                f32x4 dp[2];
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    if (u == 1 && !two) break;
                    dp[u] = mfma_bf16(ov[cur][u], gop, zero);
                }
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    if (u == 1 && !two) break;
                    const int jb = 2 * kp + u;
                    f32x4 ds;
#pragma unroll
                    for (int r = 0; r < 4; ++r) ds[r] = s[jb][r] * (dp[u][r] - delta);
                    split_hi_lo(ds, hi[u], lo[u]);
                }
                const bf16x8 dh = pair_operand(hi[0], hi[1]), dl = pair_operand(lo[0], lo[1]);
                q0 = mfma_bf16(tk0[cur], dh, q0);
                q1 = mfma_bf16(tk1[cur], dh, q1);
                q0 = mfma_bf16(tk0[cur], dl, q0);
                q1 = mfma_bf16(tk1[cur], dl, q1);
                __builtin_amdgcn_sched_barrier(0);
            }
            const float qs = p.scale * inv;  // the lane's query row: dQ_i = scale / sum_i * (the products above)
            const u32x2 lo2 = {pack_bf16(q0[0] * qs, q0[1] * qs), pack_bf16(q0[2] * qs, q0[3] * qs)};
            const u32x2 hi2 = {pack_bf16(q1[0] * qs, q1[1] * qs), pack_bf16(q1[2] * qs, q1[3] * qs)};
            if (!P2 && has_next && qb + W >= NB) request(w + gm.G);  // the wave's last block of this window
            store_rows(lo2, hi2, make_rsrc((char*)p.dq + tile_d, tile_bytes_d), qb);
        }
        __syncthreads();

        // ---------------- pass 2: key blocks wave, wave + W, ..., two at a time ----------------
        // A wave that owns two key blocks works on both at once: every operand it fetches for a query
        // block (Q and dO rows, their transposes, the statistics) then serves two key blocks, which
        // halves the LDS traffic of this pass, and the two blocks are independent chains of work.
        auto pass2 = [&](auto nk_tag, const int jb0) {
            constexpr int NK = decltype(nk_tag)::value;  // key blocks jb0 (and jb0 + W)
            bf16x8 kop[NK], vop[NK];
            f32x4 v0[NK], v1[NK], k0[NK], k1[NK];  // dV, dK [16 jb + n][4g + r] and [..][16 + 4g + r]
            int lkey[NK];
#pragma unroll
            for (int t = 0; t < NK; ++t) {
                const int jb = jb0 + t * W;
                kop[t] = __builtin_bit_cast(bf16x8, lk[opd + 16 * jb * STRIDE]);
                vop[t] = __builtin_bit_cast(bf16x8, lv[opd + 16 * jb * STRIDE]);
                v0[t] = v1[t] = k0[t] = k1[t] = zero;
                lkey[t] = HM == 2 ? load_i32(rl, (uint32_t)(16 * jb + n) * 4u) : 0;
            }
            // A key beyond L (a lane of the last key block) is not masked out: what it computes -- from
            // zero rows of K and V, possibly an overflow -- stays in its own column of every product,
            // i.e. in rows of dV and dK beyond L, which the stores drop.
            const uint16_t* lg16 = reinterpret_cast<const uint16_t*>(lg) + trs;
            const uint16_t* lq16 = reinterpret_cast<const uint16_t*>(lq) + trs;
            uint32_t aoff[4];  // additive term of query 4g + r and key 16 jb0 + n; key block t: + 64 W t bytes
#pragma unroll
            for (int r = 0; r < 4; ++r) aoff[r] = ((uint32_t)(4 * g + r) * L + 16u * jb0 + n) * 4u;
            // Row operands, statistics (LDS) and additive terms (L2) are fetched one query block ahead of
            // their use, the transposed operands one pair of query blocks ahead; the scheduling barriers
            // keep the compiler from hoisting more than that.
            bf16x8 oq[2], og[2], tg0[2], tg1[2], tx0[2], tx1[2];
            f32x4 oM[2], oD[2], ab[2][NK], am[2][NK];
            i32x4 al[2];
            auto fetch_q = [&](int qb, int slot) {
                oq[slot] = __builtin_bit_cast(bf16x8, lq[opd + 16 * qb * STRIDE]);
                og[slot] = __builtin_bit_cast(bf16x8, lg[opd + 16 * qb * STRIDE]);
                oM[slot] = *reinterpret_cast<const f32x4*>(stM + 16 * qb + 4 * g);
                oD[slot] = *reinterpret_cast<const f32x4*>(stD + 16 * qb + 4 * g);
                if (BM) {
                    // rows beyond L lie outside the descriptors (which start at the first row of the query
                    // block, so that the 4 lane offsets serve every block)
                    const uint32_t qrow = (uint32_t)(16 * qb) * L;
                    const __amdgpu_buffer_rsrc_t rbq = HB == 1 ? make_rsrc(bias32 + (size_t)h * L * L + qrow, ll - 4u * qrow) : rb;
                    const __amdgpu_buffer_rsrc_t rmq =
                        HM == 1 ? make_rsrc(p.mask + (size_t)(w % (uint32_t)p.nW) * L * L + qrow, ll - 4u * qrow) : rb;
#pragma unroll
                    for (int t = 0; t < NK; ++t)
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            if (HB == 1) ab[slot][t][r] = load_f32(rbq, aoff[r] + 64u * W * t);
                            if (HM == 1) am[slot][t][r] = load_f32(rmq, aoff[r] + 64u * W * t);
                        }
                    // with labels: those of the 4 query rows, compared with the key's where the term is used
                    if (HM == 2) al[slot] = load_i32x4(rl, (uint32_t)(16 * qb + 4 * g) * 4u);
                }
            };
            auto fetch_t = [&](int qp, int slot) {  // dO^T and Q^T of the 32 queries (channel on the lane)
                const bool two = 2 * qp + 1 < NB;
                tg0[slot] = operand_tr(lg16 + (32 * qp) * SROW, 16 * SROW, two);
                tg1[slot] = operand_tr(lg16 + (32 * qp) * SROW + 16, 16 * SROW, two);
                tx0[slot] = operand_tr(lq16 + (32 * qp) * SROW, 16 * SROW, two);
                tx1[slot] = operand_tr(lq16 + (32 * qp) * SROW + 16, 16 * SROW, two);
            };
            fetch_q(0, 0);
            fetch_t(0, 0);
#pragma unroll
            for (int qp = 0; qp < NB2; ++qp) {
                const bool two = 2 * qp + 1 < NB;
                const int tcur = qp & 1;
                if (qp + 1 < NB2) fetch_t(qp + 1, tcur ^ 1);
                bf16x4 ph[NK][2], pl[NK][2], sh[NK][2], sl[NK][2];
#pragma unroll
                for (int t = 0; t < NK; ++t) ph[t][1] = pl[t][1] = sh[t][1] = sl[t][1] = as_bf16x4(uint2{0u, 0u});
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    if (u == 1 && !two) break;
                    const int qb = 2 * qp + u, cur = qb & 1;
                    if (qb + 1 < NB) fetch_q(qb + 1, cur ^ 1);
                    __builtin_amdgcn_sched_barrier(0);
                    f32x4 sc[NK], dp[NK];
#pragma unroll
                    for (int t = 0; t < NK; ++t) {
                        sc[t] = mfma_bf16(oq[cur], kop[t], zero);  // sc[r] = <q_i, k_j>, i = 16 qb + 4g + r, j = 16 jb + n
                        dp[t] = mfma_bf16(og[cur], vop[t], zero);
                    }
#pragma unroll
                    for (int t = 0; t < NK; ++t) {
                        f32x4 pr, ds;
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            float x;
                            if (BM) {
                                const float mk = HM == 2 ? (al[cur][r] == lkey[t] ? 0.f : p.mask_value) : am[cur][t][r];
                                const float bv = ab[cur][t][r];
                                const float add = HB && HM ? bv + mk : (HB ? bv : mk);
                                x = fmaf(sc[t][r], sl2, fmaf(add, kLog2e, -oM[cur][r]));
                            } else {
                                x = fmaf(sc[t][r], sl2, -oM[cur][r]);
                            }
                            pr[r] = __builtin_amdgcn_exp2f(x);
                            ds[r] = pr[r] * (dp[t][r] - oD[cur][r]);
                        }
                        split_hi_lo(pr, ph[t][u], pl[t][u]);
                        split_hi_lo(ds, sh[t][u], sl[t][u]);
                    }
                }
#pragma unroll
                for (int t = 0; t < NK; ++t) {
                    const bf16x8 PH = pair_operand(ph[t][0], ph[t][1]), PL = pair_operand(pl[t][0], pl[t][1]);
                    const bf16x8 SH = pair_operand(sh[t][0], sh[t][1]), SL = pair_operand(sl[t][0], sl[t][1]);
                    v0[t] = mfma_bf16(tg0[tcur], PH, v0[t]);
                    v1[t] = mfma_bf16(tg1[tcur], PH, v1[t]);
                    k0[t] = mfma_bf16(tx0[tcur], SH, k0[t]);
                    k1[t] = mfma_bf16(tx1[tcur], SH, k1[t]);
                    v0[t] = mfma_bf16(tg0[tcur], PL, v0[t]);
                    v1[t] = mfma_bf16(tg1[tcur], PL, v1[t]);
                    k0[t] = mfma_bf16(tx0[tcur], SL, k0[t]);
                    k1[t] = mfma_bf16(tx1[tcur], SL, k1[t]);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            // The wave's last key blocks of this window (with 8 waves it comes through here once per window;
            // with 4, up to twice, and asks after the loop below instead).
            if (W == 8 && has_next) request(w + gm.G);
#pragma unroll
            for (int t = 0; t < NK; ++t) {
                const int jb = jb0 + t * W;
                const u32x2 va = {pack_bf16(v0[t][0], v0[t][1]), pack_bf16(v0[t][2], v0[t][3])};
                const u32x2 vb = {pack_bf16(v1[t][0], v1[t][1]), pack_bf16(v1[t][2], v1[t][3])};
                const u32x2 ka = {pack_bf16(k0[t][0] * p.scale, k0[t][1] * p.scale), pack_bf16(k0[t][2] * p.scale, k0[t][3] * p.scale)};
                const u32x2 kb = {pack_bf16(k1[t][0] * p.scale, k1[t][1] * p.scale), pack_bf16(k1[t][2] * p.scale, k1[t][3] * p.scale)};
                store_rows(va, vb, make_rsrc((char*)p.dv + tile_d, tile_bytes_d), jb);
                store_rows(ka, kb, make_rsrc((char*)p.dk + tile_d, tile_bytes_d), jb);
            }
        };
        for (int jb0 = (int)wave; P2 && jb0 < NB; jb0 += 2 * W) {
            if (jb0 + W < NB)
                pass2(std::integral_constant<int, 2>{}, jb0);
            else
                pass2(std::integral_constant<int, 1>{}, jb0);
        }
        if (P2 && W == 4 && has_next) request(w + gm.G);
        if (P2) __syncthreads();  // every wave has left the slabs (without pass 2: the barrier after pass 1)
        if (has_next) park();
    }
}

// dK, dV and dBias for 64 < L <= 256 when dBias is wanted.  The dBias accumulator is L x L fp32 per
// head (256 KB at L = 256): half of a CU's register file, which the two passes of the kernel above
// need themselves.  So a call with dBias runs that kernel with pass 1 only (dQ; the row statistics
// M_i, delta_i go to the workspace, 8 bytes per query) and this one for pass 2: a wave owns ONE key
// block of one head for its whole life -- the key blocks of a head are spread over one workgroup
// (up to 8 blocks) or two (9 to 16) -- produces S and dP block by block in the "key on the lane"
// orientation, P = exp2(score - M_i), dS = P (dP - delta_i), feeds both back into the matrix cores
// for its dV and dK rows exactly as pass 2 above, and adds dS into dBias[all queries][its keys],
// held in registers (at most 64) across the windows bw, bw + G, ...  The sums are written out once,
// in register order, as one of G partial sums per head; the reduce kernel adds the slots in a fixed
// order.  Only Q and dO (all rows) go through LDS; the wave takes the K and V rows of its key block
// straight from global memory.
// The key blocks of a head are spread over workgroups of at most 4 waves (one wave per SIMD), of which a CU
// holds two: while one loads or waits at a barrier the other computes.
constexpr int keys_parts(int nb) { return (nb + 3) / 4; }
constexpr int keys_waves(int nb) { return (nb + keys_parts(nb) - 1) / keys_parts(nb); }

template <int NB, int HB, int HM>
__global__ void __launch_bounds__(64 * keys_waves(NB), 2) bwd_bf16_large_keys_kernel(BwdArgs p, LargeGeom gm) {
    constexpr bool BM = HB != 0 || HM != 0;
    constexpr int PARTS = keys_parts(NB);
    constexpr int W = keys_waves(NB);
    constexpr int NB2 = (NB + 1) / 2;
    constexpr int ROWS = 16 * NB;
    constexpr int PASSES = (ROWS + 16 * W - 1) / (16 * W);
    constexpr uint32_t STRIDE = 5;         // slab row: 64 bytes of data + 16 of padding
    constexpr uint32_t SROW = STRIDE * 8;  // the same in bf16 elements
    extern __shared__ __attribute__((aligned(16))) uint4 lds[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int n = lane & 15, g = lane >> 4;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // the parts of a head and the heads of a window are neighbours in the logical order: one XCD
    const uint32_t lb = xcd_logical_block(blockIdx.x, gm.xcd_q, gm.xcd_r);
    const uint32_t part = lb % PARTS, h = (lb / PARTS) % gm.heads, bw = lb / (PARTS * gm.heads);
    const int jb = (int)(part * W + wave);  // this wave's key block
    const bool active = jb < NB;            // wave-uniform
    const int L = p.L;
    const uint32_t row_bytes = (uint32_t)p.ldq * 2u, row_g = (uint32_t)p.ldg * 2u, row_d = (uint32_t)p.ldd * 2u;
    const float sl2 = p.scale * kLog2e;
    const f32x4 zero = {0.f, 0.f, 0.f, 0.f};

    // LDS: slabs [Q][dO], each [ROWS][STRIDE] uint4; M[ROWS], delta[ROWS]; 16 rows x 80 bytes per wave for its output rows
    constexpr uint32_t SET = 2 * ROWS * STRIDE + ROWS / 2;  // in uint4
    char* const cell = reinterpret_cast<char*>(lds + SET) + wave * (16 * 80);

    const uint32_t ll = (uint32_t)L * L * 4u;
    const float* const bias32 = static_cast<const float*>(p.bias);
    const uint32_t srow = (uint32_t)tid >> 2, scol = (uint32_t)tid & 3u;
    const uint32_t tile_bytes = (uint32_t)(L - 1) * row_bytes + 2u * kHeadDim;
    const uint32_t tile_bytes_g = (uint32_t)(L - 1) * row_g + 2u * kHeadDim;
    const uint32_t tile_bytes_d = (uint32_t)(L - 1) * row_d + 2u * kHeadDim;
    const uint32_t trs = (4u * g + (n >> 2)) * SROW + 4u * (n & 3);
    const uint32_t opd = (uint32_t)n * STRIDE + g;
    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
    auto store_rows = [&](const u32x2 lo, const u32x2 hi, const __amdgpu_buffer_rsrc_t dst) {
        *reinterpret_cast<u32x2*>(cell + n * 80 + g * 8) = lo;
        *reinterpret_cast<u32x2*>(cell + n * 80 + 32 + g * 8) = hi;
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        const uint32_t r = (uint32_t)(lane >> 2), c = (uint32_t)(lane & 3);
        const u32x4 rows = *reinterpret_cast<const u32x4*>(cell + r * 80 + c * 16);
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_raw_buffer_store_b128(rows, dst, (uint32_t)(16 * jb + r) * row_d + 16u * c, 0, 0);
    };

    f32x4 dbacc[NB];  // dS summed over the windows: queries 16 qb + 4g + r, key 16 jb + n
#pragma unroll
    for (int qb = 0; qb < NB; ++qb) dbacc[qb] = zero;
    uint32_t aoff[4];  // additive term of query 4g + r (of a query block) and this lane's key
#pragma unroll
    for (int r = 0; r < 4; ++r) aoff[r] = ((uint32_t)(4 * g + r) * L + 16u * jb + n) * 4u;

    // The Q and dO slabs, the statistics and the wave's own K and V rows of the next window are requested into
    // registers at the end of an iteration, in front of its stores, and go from there into LDS between the two
    // barriers that separate the windows.
    constexpr int PASSES_ = PASSES;
    constexpr int SPASSES = (ROWS / 2 + 64 * W - 1) / (64 * W);
    u32x4 pq[PASSES_], pg[PASSES_], st4[SPASSES], pk, pv;
    auto request = [&](uint32_t w) {
        const size_t tile = ((size_t)w * L * p.ldq + (size_t)h * kHeadDim) * 2u;
        const size_t tile_g = ((size_t)w * L * p.ldg + (size_t)h * kHeadDim) * 2u;
        const __amdgpu_buffer_rsrc_t rk = make_rsrc((const char*)p.k + tile, tile_bytes);
        const __amdgpu_buffer_rsrc_t rv = make_rsrc((const char*)p.v + tile, tile_bytes);
        const __amdgpu_buffer_rsrc_t rq = make_rsrc((const char*)p.q + tile, tile_bytes);
        const __amdgpu_buffer_rsrc_t rg = make_rsrc((const char*)p.d_o + tile_g, tile_bytes_g);
        const __amdgpu_buffer_rsrc_t rs =
            make_rsrc(p.stats + ((size_t)w * p.heads + h) * (2 * ROWS), (uint32_t)(2 * ROWS * 4));
#pragma unroll
        for (int t = 0; t < PASSES; ++t) {  // rows beyond L arrive as zeros
            pq[t] = __builtin_amdgcn_raw_buffer_load_b128(rq, (16 * W * t + srow) * row_bytes + scol * 16u, 0, 0);
            pg[t] = __builtin_amdgcn_raw_buffer_load_b128(rg, (16 * W * t + srow) * row_g + scol * 16u, 0, 0);
        }
        // 2 ROWS floats of statistics: 16 bytes per thread
#pragma unroll
        for (int t = 0; t < SPASSES; ++t) st4[t] = __builtin_amdgcn_raw_buffer_load_b128(rs, (uint32_t)(tid + 64 * W * t) * 16u, 0, 0);
        // the wave's own K and V rows as operands: row 16 jb + n, channels 8g .. 8g + 7
        pk = __builtin_amdgcn_raw_buffer_load_b128(rk, (uint32_t)(16 * jb + n) * row_bytes + 16u * g, 0, 0);
        pv = __builtin_amdgcn_raw_buffer_load_b128(rv, (uint32_t)(16 * jb + n) * row_bytes + 16u * g, 0, 0);
    };
    auto park = [&]() {
        uint4* const sq = lds;
        uint4* const sg = sq + ROWS * STRIDE;
#pragma unroll
        for (int t = 0; t < PASSES; ++t) {
            const uint32_t row = 16 * W * t + srow;
            if (row < (uint32_t)ROWS) {
                sq[row * STRIDE + scol] = __builtin_bit_cast(uint4, pq[t]);
                sg[row * STRIDE + scol] = __builtin_bit_cast(uint4, pg[t]);
            }
        }
#pragma unroll
        for (int t = 0; t < SPASSES; ++t)
            if (tid + 64 * W * t < ROWS / 2) sq[2 * ROWS * STRIDE + tid + 64 * W * t] = __builtin_bit_cast(uint4, st4[t]);
    };
    if (bw < (uint32_t)p.N) {
        request(bw);
        park();
    }
    __syncthreads();
    const uint4* const lq = lds;
    const uint4* const lg = lq + ROWS * STRIDE;
    const float* const stM = reinterpret_cast<const float*>(lq + 2 * ROWS * STRIDE);
    const float* const stD = stM + ROWS;
    const uint16_t* const lg16 = reinterpret_cast<const uint16_t*>(lg) + trs;
    const uint16_t* const lq16 = reinterpret_cast<const uint16_t*>(lq) + trs;

    for (uint32_t w = bw; w < (uint32_t)p.N; w += gm.G) {
        const size_t tile_d = ((size_t)w * L * p.ldd + (size_t)h * kHeadDim) * 2u;
        const __amdgpu_buffer_rsrc_t rl =
            HM == 2 ? make_rsrc(p.labels + (size_t)(w % (uint32_t)p.nW) * L, (uint32_t)L * 4u) : make_rsrc(nullptr, 0);
        const bf16x8 kop = as_bf16x8(pk), vop = as_bf16x8(pv);
        const bool has_next = w + gm.G < (uint32_t)p.N;
        u32x2 va = {0u, 0u}, vb = {0u, 0u}, ka = {0u, 0u}, kb = {0u, 0u};  // the wave's 16 rows of dV and dK, packed

        if (active) {
            const int lkey = HM == 2 ? load_i32(rl, (uint32_t)(16 * jb + n) * 4u) : 0;
            f32x4 v0 = zero, v1 = zero, k0 = zero, k1 = zero;  // dV, dK [16 jb + n][4g + r] and [..][16 + 4g + r]
            // operands of a query block one block ahead of their use, transposed operands one pair ahead
            bf16x8 oq[2], og[2], tg0[2], tg1[2], tx0[2], tx1[2];
            f32x4 oM[2], oD[2], ab[2], am[2];
            i32x4 al[2];
            auto fetch_q = [&](int qb, int slot) {
                oq[slot] = __builtin_bit_cast(bf16x8, lq[opd + 16 * qb * STRIDE]);
                og[slot] = __builtin_bit_cast(bf16x8, lg[opd + 16 * qb * STRIDE]);
                oM[slot] = *reinterpret_cast<const f32x4*>(stM + 16 * qb + 4 * g);
                oD[slot] = *reinterpret_cast<const f32x4*>(stD + 16 * qb + 4 * g);
                if (BM) {
                    // descriptors start at the first row of the query block, so that the 4 lane offsets
                    // serve every block; rows beyond L lie outside them
                    const uint32_t qrow = (uint32_t)(16 * qb) * L;
                    const __amdgpu_buffer_rsrc_t rbq =
                        HB == 1 ? make_rsrc(bias32 + (size_t)h * L * L + qrow, ll - 4u * qrow) : make_rsrc(nullptr, 0);
                    const __amdgpu_buffer_rsrc_t rmq =
                        HM == 1 ? make_rsrc(p.mask + (size_t)(w % (uint32_t)p.nW) * L * L + qrow, ll - 4u * qrow)
                                : make_rsrc(nullptr, 0);
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        if (HB == 1) ab[slot][r] = load_f32(rbq, aoff[r]);
                        if (HM == 1) am[slot][r] = load_f32(rmq, aoff[r]);
                    }
                    if (HM == 2) al[slot] = load_i32x4(rl, (uint32_t)(16 * qb + 4 * g) * 4u);
                }
            };
            auto fetch_t = [&](int qp, int slot) {  // dO^T and Q^T of the 32 queries (channel on the lane)
                const bool two = 2 * qp + 1 < NB;
                tg0[slot] = operand_tr(lg16 + (32 * qp) * SROW, 16 * SROW, two);
                tg1[slot] = operand_tr(lg16 + (32 * qp) * SROW + 16, 16 * SROW, two);
                tx0[slot] = operand_tr(lq16 + (32 * qp) * SROW, 16 * SROW, two);
                tx1[slot] = operand_tr(lq16 + (32 * qp) * SROW + 16, 16 * SROW, two);
            };
            fetch_q(0, 0);
            fetch_t(0, 0);
#pragma unroll
            for (int qp = 0; qp < NB2; ++qp) {
                const bool two = 2 * qp + 1 < NB;
                const int tcur = qp & 1;
                if (qp + 1 < NB2) fetch_t(qp + 1, tcur ^ 1);
                bf16x4 ph[2], pl[2], sh[2], sl[2];
                ph[1] = pl[1] = sh[1] = sl[1] = as_bf16x4(uint2{0u, 0u});
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    if (u == 1 && !two) break;
                    const int qb = 2 * qp + u, cur = qb & 1;
                    if (qb + 1 < NB) fetch_q(qb + 1, cur ^ 1);
                    __builtin_amdgcn_sched_barrier(0);
                    const f32x4 sc = mfma_bf16(oq[cur], kop, zero);  // <q_i, k_j>, i = 16 qb + 4g + r, j = 16 jb + n
                    const f32x4 dp = mfma_bf16(og[cur], vop, zero);
                    f32x4 pr, ds;
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        float x;
                        if (BM) {
                            const float mk = HM == 2 ? (al[cur][r] == lkey ? 0.f : p.mask_value) : am[cur][r];
                            const float bv = ab[cur][r];
                            const float add = HB && HM ? bv + mk : (HB ? bv : mk);
                            x = fmaf(sc[r], sl2, fmaf(add, kLog2e, -oM[cur][r]));
                        } else {
                            x = fmaf(sc[r], sl2, -oM[cur][r]);
                        }
                        // a key beyond L is not masked out: its column of every product lands in rows of dV, dK
                        // and columns of dBias beyond L, which the stores and the reduce kernel drop
                        pr[r] = __builtin_amdgcn_exp2f(x);
                        ds[r] = pr[r] * (dp[r] - oD[cur][r]);
                    }
                    dbacc[qb] += ds;
                    split_hi_lo(pr, ph[u], pl[u]);
                    split_hi_lo(ds, sh[u], sl[u]);
                }
                const bf16x8 PH = pair_operand(ph[0], ph[1]), PL = pair_operand(pl[0], pl[1]);
                const bf16x8 SH = pair_operand(sh[0], sh[1]), SL = pair_operand(sl[0], sl[1]);
                v0 = mfma_bf16(tg0[tcur], PH, v0);
                v1 = mfma_bf16(tg1[tcur], PH, v1);
                k0 = mfma_bf16(tx0[tcur], SH, k0);
                k1 = mfma_bf16(tx1[tcur], SH, k1);
                v0 = mfma_bf16(tg0[tcur], PL, v0);
                v1 = mfma_bf16(tg1[tcur], PL, v1);
                k0 = mfma_bf16(tx0[tcur], SL, k0);
                k1 = mfma_bf16(tx1[tcur], SL, k1);
                __builtin_amdgcn_sched_barrier(0);
            }
            va = u32x2{pack_bf16(v0[0], v0[1]), pack_bf16(v0[2], v0[3])};
            vb = u32x2{pack_bf16(v1[0], v1[1]), pack_bf16(v1[2], v1[3])};
            ka = u32x2{pack_bf16(k0[0] * p.scale, k0[1] * p.scale), pack_bf16(k0[2] * p.scale, k0[3] * p.scale)};
            kb = u32x2{pack_bf16(k1[0] * p.scale, k1[1] * p.scale), pack_bf16(k1[2] * p.scale, k1[3] * p.scale)};
        }
        // The next window is requested here, behind the last loads of this one's additive term and in front of
        // its stores: memory operations of a wave complete in the order issued, so a request at the top of the
        // window would hold up every small load behind it.
        if (has_next) request(w + gm.G);
        if (active) {
            store_rows(va, vb, make_rsrc((char*)p.dv + tile_d, tile_bytes_d));
            store_rows(ka, kb, make_rsrc((char*)p.dk + tile_d, tile_bytes_d));
        }
        __syncthreads();  // every wave is done with the slabs
        if (has_next) park();
        __syncthreads();
    }

    // partial sums in register order: [slot][head][jb][qb][lane] float4, element r of lane (g, n) being
    // dS summed over windows for query 16 qb + 4g + r and key 16 jb + n
    if (active) {
        f32x4* dst = reinterpret_cast<f32x4*>(p.partial) + ((size_t)bw * p.heads + h) * (NB * NB * 64) + lane;
#pragma unroll
        for (int qb = 0; qb < NB; ++qb) dst[(jb * NB + qb) * 64] = dbacc[qb];
    }
}

// Workgroups of `fn` one CU holds (LDS and registers decide), asked once per kernel; threads racing
// through the first call ask twice and store the same figure.
hipError_t workgroups_per_cu(const void* fn, unsigned block, size_t lds, std::atomic<int>& once, int& per_cu) {
    const hipError_t e = allow_lds(fn, lds);
    if (e != hipSuccess) return e;
    per_cu = once.load(std::memory_order_relaxed);
    if (per_cu == 0) {
        int nblk = 0;
        const hipError_t q = hipOccupancyMaxActiveBlocksPerMultiprocessor(&nblk, fn, (int)block, lds);
        if (q != hipSuccess) return q;
        per_cu = nblk < 1 ? 1 : nblk;
        once.store(per_cu, std::memory_order_relaxed);
    }
    return hipSuccess;
}

// dK, dV and the dBias partial sums; `slots` receives the number of partial sums per head
template <int NB, int HB, int HM>
hipError_t launch_large_keys(const BwdArgs& a, hipStream_t st, int& slots) {
    constexpr int W = keys_waves(NB), HALVES = keys_parts(NB);
    const void* fn = reinterpret_cast<const void*>(&bwd_bf16_large_keys_kernel<NB, HB, HM>);
    const unsigned block = 64u * W;
    const size_t lds = (size_t)2 * 16 * NB * 5 * 16 + (size_t)2 * 16 * NB * 4 + (size_t)W * 16 * 80;  // slabs, statistics, the waves' output cells
    static std::atomic<int> once{0};
    int per_cu = 1;
    const hipError_t e = workgroups_per_cu(fn, block, lds, once, per_cu);
    if (e != hipSuccess) return e;
    LargeGeom gm;
    gm.heads = (uint32_t)a.heads;
    long long G = (long long)cu_count() * per_cu / ((long long)a.heads * HALVES);  // resident workgroups only
    if (G > a.slots) G = a.slots;  // the workspace holds a.slots partial sums per head
    if (G > a.N) G = a.N;
    if (G < 1) G = 1;
    gm.G = (uint32_t)G;
    slots = (int)G;
    const unsigned grid = gm.G * gm.heads * HALVES;
    gm.xcd_q = grid / 8u;
    gm.xcd_r = grid % 8u;
    hipLaunchKernelGGL((bwd_bf16_large_keys_kernel<NB, HB, HM>), dim3(grid), dim3(block), lds, st, a, gm);
    return hipGetLastError();
}

template <int NB, int HB, int HM, bool P2>
hipError_t launch_large_one(const BwdArgs& a, hipStream_t st) {
    constexpr int W = large_waves(NB);
    const void* fn = reinterpret_cast<const void*>(&bwd_bf16_large_kernel<NB, HB, HM, P2>);
    const unsigned block = 64u * W;
    const size_t lds = (size_t)4 * 16 * NB * kLargeStride * 16 + (size_t)2 * 16 * NB * 4 + (size_t)W * 16 * 68 * 4;  // slabs, statistics, one patch per wave
    static std::atomic<int> once{0};
    int per_cu = 1;
    const hipError_t e = workgroups_per_cu(fn, block, lds, once, per_cu);
    if (e != hipSuccess) return e;
    LargeGeom gm;
    gm.heads = (uint32_t)a.heads;
    long long G = (long long)cu_count() * per_cu / a.heads;  // one resident workgroup per slot and head
    if (G < 1) G = 1;
    if (G > a.N) G = a.N;
    gm.G = (uint32_t)G;
    const unsigned grid = gm.G * gm.heads;
    gm.xcd_q = grid / 8u;
    gm.xcd_r = grid % 8u;
    hipLaunchKernelGGL((bwd_bf16_large_kernel<NB, HB, HM, P2>), dim3(grid), dim3(block), lds, st, a, gm);
    return hipGetLastError();
}

// Without dBias one kernel does both passes.  With it: pass 1 (dQ, statistics), then the keys kernel
// (dK, dV, dBias partial sums), then the reduction of the partial sums.
template <int NB, int HB, int HM>
hipError_t launch_large_both(const BwdArgs& a, hipStream_t st) {
    if (a.dbias == nullptr) return launch_large_one<NB, HB, HM, true>(a, st);
    hipError_t e = launch_large_one<NB, HB, HM, false>(a, st);
    if (e != hipSuccess) return e;
    int slots = a.slots;
    e = launch_large_keys<NB, HB, HM>(a, st, slots);
    if (e != hipSuccess) return e;
    BwdArgs r = a;
    r.slots = slots;
    return launch_dbias_reduce(r, st, true);
}

template <int NB>
hipError_t launch_large_nb(const BwdArgs& a, hipStream_t st) {
    if (a.bias && a.bias_bf16) return hipErrorInvalidValue;  // the caller hands over an fp32 copy
    if (a.bias) {
        if (a.labels) return launch_large_both<NB, 1, 2>(a, st);
        return a.mask ? launch_large_both<NB, 1, 1>(a, st) : launch_large_both<NB, 1, 0>(a, st);
    }
    if (a.labels) return launch_large_both<NB, 0, 2>(a, st);
    return a.mask ? launch_large_both<NB, 0, 1>(a, st) : launch_large_both<NB, 0, 0>(a, st);
}

}  // namespace

// Slots of dBias partial sums for large windows: one resident workgroup of the dBias kernel per CU
// when its slabs fill most of the LDS (more than 10 blocks of 16 rows), two otherwise
int backward_large_slots(long long N, int heads, int L) {
    long long G = (L > 160 ? 1 : 2) * cu_count() / heads;
    if (G < 1) G = 1;
    return (int)(G > N ? N : G);
}

hipError_t launch_backward_bf16_large(const BwdArgs& a, hipStream_t s) {
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
