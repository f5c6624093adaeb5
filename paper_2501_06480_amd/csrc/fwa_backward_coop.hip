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
//       P and dS rows of its block, as hi + lo bf16, written row-major into LDS tiles
//   phase B, wave jb (16 keys):
//       dV, dK rows of its block = contraction over all queries of P resp. dS with dO^T resp.
//       Q^T.  The operands with the queries on the k-slots come out of LDS through the
//       transposing read ds_read_b64_tr_b16: the P/dS tiles with the key on the lane, the
//       dO/Q slabs (and the K slab for dQ in phase A) with the channel on the lane.
//
// The workgroup loads the Q, K, V, dO slabs of its heads (whole 128-byte lines per row) with
// coalesced 16-byte loads into LDS once per window and requests the next window's slabs before
// computing.  A workgroup keeps its heads and walks the windows bw, bw + G, ...; G is a
// multiple of nW, so (bias[h] + mask[bw % nW]) * log2e is loaded once, into registers.
#include "fwa_device.h"
#include "fwa_internal.h"
#include "fwa_softmax.h"

namespace fwa {
namespace {

constexpr int kCoopWavesPerTile = 4;
constexpr int kCoopMaxHeads = 3;  // heads per workgroup: 12 waves, 3 per SIMD, <= 170 VGPRs each

struct CoopGeom {
    FastDiv groups;         // workgroups per window position
    FastDiv lanes_per_row;  // 4 * heads_per_block
    uint32_t heads_per_block;
    uint32_t G;             // window positions walked in parallel (= dBias slots)
    uint32_t xcd_remap, xcd_q, xcd_r;
};

// KT < 4 promises that only the first KT of a lane's 4 columns in the last key block can be real
// (L <= 16 (NB - 1) + KT, e.g. KT = 1 for L = 49): the others are zero without any arithmetic.
// PW ("per window"): the mask comes as labels whose period G is no multiple of.  The registers then
// hold bias * log2e alone; the labels of a window travel with its slabs into LDS and phase A forms
// the mask per score (AddendRegsLabels).
template <int NB, bool BM, bool DB, int KT, bool PW>
__global__ void __launch_bounds__(64 * kCoopWavesPerTile * kCoopMaxHeads) bwd_bf16_coop_kernel(BwdArgs p, CoopGeom gm) {
    constexpr int NB2 = (NB + 1) / 2;
    constexpr int ROWS = 16 * NB;
    extern __shared__ __attribute__((aligned(16))) uint4 lds[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int n = lane & 15, g = lane >> 4;
    const uint32_t wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const uint32_t hl = wv >> 2;            // head inside the workgroup
    const int role = (int)(wv & 3u);        // query block in phase A, key block in phase B
    // workgroups that share 128-byte lines (head groups of one window) are neighbours in the logical
    // order; when a group is not made of whole lines the order is mapped so that they share an XCD
    const uint32_t lb = gm.xcd_remap ? xcd_logical_block(blockIdx.x, gm.xcd_q, gm.xcd_r) : blockIdx.x;
    const uint32_t bw = fastdiv(lb, gm.groups);
    const uint32_t hg = lb - bw * gm.groups.d;
    const uint32_t hpb = gm.heads_per_block;
    const uint32_t h = hg * hpb + hl;
    const int L = p.L;
    // token rows are p.ldq (q, k, v), p.ldg (d_o), p.ldd (dq, dk, dv) elements apart; window w starts at row w L
    const uint32_t row_bytes = (uint32_t)p.ldq * 2u, row_g = (uint32_t)p.ldg * 2u, row_d = (uint32_t)p.ldd * 2u;
    const uint32_t stride = 4u * hpb + 1u;  // slab row stride in 16-byte units
    const float sl2 = p.scale * kLog2e;
    const bool active = role < NB;

    // LDS: slabs [K][V][Q][dO], each [ROWS][stride] uint4; then per head four bf16 tiles.
    uint4* const lk = lds;
    uint4* const lv = lds + ROWS * stride;
    uint4* const lq = lds + 2 * ROWS * stride;
    uint4* const lg = lds + 3 * ROWS * stride;
    // P_hi, P_lo, dS_hi, dS_lo tiles of this head: [ROWS][64] bf16.  A row is 16 units of 4 keys; unit
    // (block b, quarter c) of row i sits at unit (b ^ (i & 3), c ^ ((i >> 2) & 3)): the 16 lanes of a
    // write (16 rows, one unit each) and of a transposing read (4 rows x 4 units) then touch 16
    // different units, i.e. every bank once.
    constexpr uint32_t XS = 64, XT = ROWS * XS;
    uint16_t* const ex = reinterpret_cast<uint16_t*>(lds + 4 * ROWS * stride) + (size_t)hl * (4 * XT);
    // PW: the labels of the window in LDS, behind the tiles of all heads
    int* const llab = reinterpret_cast<int*>(reinterpret_cast<uint16_t*>(lds + 4 * ROWS * stride) + (size_t)hpb * (4 * XT));
    const uint32_t srow = stride * 8u;  // slab row stride in bf16 elements
    // transposing-read base of this lane inside a slab (channel on the lane) and inside a tile
    const uint32_t trs = (4u * g + (n >> 2)) * srow + 32u * hl + 4u * (n & 3);
    // transposing read of key block jb = role: row 4g + (n >> 2) (+ 16, 32, ...: same low row bits)
    const uint32_t trx = (4u * g + (n >> 2)) * XS + ((((uint32_t)role) ^ (uint32_t)(n >> 2)) << 4) + ((((uint32_t)n & 3u) ^ (uint32_t)g) << 2);
    const uint32_t opd = (uint32_t)n * stride + 4u * hl + g;  // operand of row block b: slab[opd + 16 b stride]

    f32x4 dbacc[NB];
#pragma unroll
    for (int jb = 0; jb < NB; ++jb) dbacc[jb] = f32x4{0.f, 0.f, 0.f, 0.f};

    const f32x4 zero = {0.f, 0.f, 0.f, 0.f};

    // slab movement: thread -> (row, 16-byte column); one pass covers 64 rows
    const uint32_t rip = fastdiv((uint32_t)tid, gm.lanes_per_row);
    const uint32_t col = (uint32_t)tid - rip * gm.lanes_per_row.d;
    const uint32_t slab_bytes = (uint32_t)(L - 1) * row_bytes + hpb * 2u * kHeadDim;
    const uint32_t slab_bytes_g = (uint32_t)(L - 1) * row_g + hpb * 2u * kHeadDim;
    const uint32_t goff = rip * row_bytes + col * 16u;
    const uint32_t goff_g = rip * row_g + col * 16u;
    const uint32_t loff = rip * stride + col;
    u32x4 pk, pv, pq, pg;
    i32x4 plab = {0, 0, 0, 0};  // PW: labels 4 tid .. 4 tid + 3 of the requested window (0 beyond L)
    auto request = [&](uint32_t w) {
        const size_t slab = ((size_t)w * L * p.ldq + (size_t)hg * hpb * kHeadDim) * 2u;
        const size_t slab_g = ((size_t)w * L * p.ldg + (size_t)hg * hpb * kHeadDim) * 2u;
        // rows beyond L lie outside the descriptors and arrive as zeros
        pk = __builtin_amdgcn_raw_buffer_load_b128(make_rsrc((const char*)p.k + slab, slab_bytes), goff, 0, 0);
        pv = __builtin_amdgcn_raw_buffer_load_b128(make_rsrc((const char*)p.v + slab, slab_bytes), goff, 0, 0);
        pq = __builtin_amdgcn_raw_buffer_load_b128(make_rsrc((const char*)p.q + slab, slab_bytes), goff, 0, 0);
        pg = __builtin_amdgcn_raw_buffer_load_b128(make_rsrc((const char*)p.d_o + slab_g, slab_bytes_g), goff_g, 0, 0);
        if (PW && wv == 0) plab = load_i32x4(make_rsrc(p.labels + (size_t)(w % (uint32_t)p.nW) * L, (uint32_t)L * 4u), (uint32_t)tid * 16u);
    };
    auto park = [&]() {
        if (rip < (uint32_t)ROWS) {
            lk[loff] = __builtin_bit_cast(uint4, pk);
            lv[loff] = __builtin_bit_cast(uint4, pv);
            lq[loff] = __builtin_bit_cast(uint4, pq);
            lg[loff] = __builtin_bit_cast(uint4, pg);
        }
        if (PW && tid < ROWS / 4) reinterpret_cast<i32x4*>(llab)[tid] = plab;
    };
    if (bw < (uint32_t)p.N) request(bw);  // in flight while the additive term is fetched
    // additive score term of this wave's query rows, in registers (see the file comment)
    f32x4 add[NB];
    if (BM && active) {
        const BiasSrc rb = bias_of_head(p, h);
        const MaskSrc msk = PW ? MaskSrc{make_rsrc(nullptr, 0), 0.f, false} : mask_of_window(p, bw);
        addend_at(rb, msk, (uint32_t)(16 * role + n), 4u * g, (uint32_t)L).fill(add, kLog2e);
    }
    const float mv = p.mask_value * kLog2e;
    if (bw < (uint32_t)p.N) park();

    const uint32_t tile_bytes = (uint32_t)(L - 1) * row_d + 2u * kHeadDim;  // of an output tile
    const uint32_t off_half = (uint32_t)n * row_d + 8u * g;  // channels 4g..4g+3 of row n (+32 B: 16+4g..)

    // The next window's slabs are requested at the top of an iteration and parked in LDS at its
    // end, i.e. always with this iteration's output stores younger than them in the memory queue:
    // the wait in front of the LDS writes then counts those stores out instead of waiting for them
    // (at the top of the loop the compiler has to assume the worst of both ways in).  The request
    // stands behind the barrier, not in front of it: a wave that is held up while it issues its
    // loads (the 48 wave-level loads of a workgroup queue at the CU's one address unit) then holds
    // up nobody else (stage 1: 135 -> 128 us, stage 2: 75 -> 70; spreading the four loads of a
    // thread over the stages of phase A adds nothing to that).
    for (uint32_t w = bw; w < (uint32_t)p.N; w += gm.G) {
        const bool has_next = w + gm.G < (uint32_t)p.N;
        __syncthreads();
        if (has_next) request(w + gm.G);  // in flight while this window is computed

        const size_t tile = ((size_t)w * L * p.ldd + (size_t)h * kHeadDim) * 2u;
        typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
        u32x2 dq_lo = {0u, 0u}, dq_hi = {0u, 0u};
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
            // softmax of the block's rows: s <- exp(score - rowmax), inv = 1 / rowsum
            float inv;
            if (BM && PW) {
                const AddendRegsLabels<NB> addend = {add, llab, llab[16 * qb + n], mv, g};
                inv = softmax_block<NB, true, AddendRegsLabels<NB>, KT>(s, sl2, addend, L, g);
            } else if (BM) {
                const AddendRegs<NB> addend = {add};
                inv = softmax_block<NB, true, AddendRegs<NB>, KT>(s, sl2, addend, L, g);
            } else {
                inv = softmax_block<NB, false, AddendNone, KT>(s, sl2, AddendNone{}, L, g);
            }
            float delta = 0.f;
#pragma unroll
            for (int jb = 0; jb < NB; ++jb)
#pragma unroll
                for (int r = 0; r < (jb == NB - 1 ? KT : 4); ++r) {
                    s[jb][r] *= inv;  // P
                    delta = fmaf(s[jb][r], dp[jb][r], delta);
                }
            delta = sum_over_g(delta);
#pragma unroll
            for (int jb = 0; jb < NB; ++jb) {
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    dp[jb][r] = (jb == NB - 1 && r >= KT) ? 0.f : s[jb][r] * (dp[jb][r] - delta);  // dS
                if (DB) dbacc[jb] += dp[jb];
            }
            // hi + lo bf16 parts of P and dS: rows of this block into the LDS tiles for phase B
            bf16x4 ds_hi[NB], ds_lo[NB];
#pragma unroll
            for (int jb = 0; jb < NB; ++jb) {
                bf16x4 p_hi, p_lo;
                split_hi_lo(s[jb], p_hi, p_lo);
                split_hi_lo(dp[jb], ds_hi[jb], ds_lo[jb]);
                uint16_t* cell = ex + (16 * qb + n) * XS + ((jb ^ (n & 3)) << 4) + ((g ^ ((n >> 2) & 3)) << 2);
                *reinterpret_cast<uint2*>(cell + 0 * XT) = __builtin_bit_cast(uint2, p_hi);
                *reinterpret_cast<uint2*>(cell + 1 * XT) = __builtin_bit_cast(uint2, p_lo);
                *reinterpret_cast<uint2*>(cell + 2 * XT) = __builtin_bit_cast(uint2, ds_hi[jb]);
                *reinterpret_cast<uint2*>(cell + 3 * XT) = __builtin_bit_cast(uint2, ds_lo[jb]);
            }
            // dQ^T = K^T dS^T over pairs of key blocks; K^T (channels 0..15 / 16..31 on the lane)
            // straight from the K slab
            f32x4 q0 = zero, q1 = zero;  // dQ[16 qb + n][4g + r], dQ[16 qb + n][16 + 4g + r]
            const uint16_t* lk16 = reinterpret_cast<const uint16_t*>(lk) + trs;
#pragma unroll
            for (int kp = 0; kp < NB2; ++kp) {
                const bool two = 2 * kp + 1 < NB;
                const int j1 = two ? 2 * kp + 1 : 0;
                const bf16x8 k0 = operand_tr(lk16 + (32 * kp) * srow, 16 * srow, two);
                const bf16x8 k1 = operand_tr(lk16 + (32 * kp) * srow + 16, 16 * srow, two);
                const uint2 h0 = __builtin_bit_cast(uint2, ds_hi[2 * kp]), l0 = __builtin_bit_cast(uint2, ds_lo[2 * kp]);
                uint2 h1 = {0u, 0u}, l1 = {0u, 0u};
                if (two) {
                    h1 = __builtin_bit_cast(uint2, ds_hi[j1]);
                    l1 = __builtin_bit_cast(uint2, ds_lo[j1]);
                }
                const bf16x8 dh = as_bf16x8(u32x4{h0.x, h0.y, h1.x, h1.y}), dl = as_bf16x8(u32x4{l0.x, l0.y, l1.x, l1.y});
                q0 = mfma_bf16(k0, dh, q0);
                q1 = mfma_bf16(k1, dh, q1);
                q0 = mfma_bf16(k0, dl, q0);
                q1 = mfma_bf16(k1, dl, q1);
            }
            dq_lo = u32x2{pack_bf16(q0[0] * p.scale, q0[1] * p.scale), pack_bf16(q0[2] * p.scale, q0[3] * p.scale)};
            dq_hi = u32x2{pack_bf16(q1[0] * p.scale, q1[1] * p.scale), pack_bf16(q1[2] * p.scale, q1[3] * p.scale)};
        }
        __syncthreads();
        // ---------------- phase B: key block `role` ----------------
        if (active) {
            {   // the dQ rows of phase A leave behind the barrier
                const __amdgpu_buffer_rsrc_t rdq = make_rsrc((char*)p.dq + tile, tile_bytes);
                __builtin_amdgcn_raw_buffer_store_b64(dq_lo, rdq, off_half + 16 * role * row_d, 0, 0);
                __builtin_amdgcn_raw_buffer_store_b64(dq_hi, rdq, off_half + 32 + 16 * role * row_d, 0, 0);
            }
            const int jb = role;
            f32x4 v0 = zero, v1 = zero, k0 = zero, k1 = zero;  // dV, dK [16 jb + n][4g + r] and [..][16 + 4g + r]
            const uint16_t* lg16 = reinterpret_cast<const uint16_t*>(lg) + trs;
            const uint16_t* lq16 = reinterpret_cast<const uint16_t*>(lq) + trs;
            const uint16_t* xt = ex + trx;
#pragma unroll
            for (int qp = 0; qp < NB2; ++qp) {
                const bool two = 2 * qp + 1 < NB;
                // dO^T and Q^T of the 32 queries (channel on the lane), P and dS of the same
                // queries (key on the lane)
                const bf16x8 g0 = operand_tr(lg16 + (32 * qp) * srow, 16 * srow, two);
                const bf16x8 g1 = operand_tr(lg16 + (32 * qp) * srow + 16, 16 * srow, two);
                const bf16x8 x0 = operand_tr(lq16 + (32 * qp) * srow, 16 * srow, two);
                const bf16x8 x1 = operand_tr(lq16 + (32 * qp) * srow + 16, 16 * srow, two);
                const bf16x8 ph = operand_tr(xt + 0 * XT + (32 * qp) * XS, 16 * XS, two);
                const bf16x8 pl = operand_tr(xt + 1 * XT + (32 * qp) * XS, 16 * XS, two);
                const bf16x8 sh = operand_tr(xt + 2 * XT + (32 * qp) * XS, 16 * XS, two);
                const bf16x8 sl = operand_tr(xt + 3 * XT + (32 * qp) * XS, 16 * XS, two);
                v0 = mfma_bf16(g0, ph, v0);
                v1 = mfma_bf16(g1, ph, v1);
                k0 = mfma_bf16(x0, sh, k0);
                k1 = mfma_bf16(x1, sh, k1);
                v0 = mfma_bf16(g0, pl, v0);
                v1 = mfma_bf16(g1, pl, v1);
                k0 = mfma_bf16(x0, sl, k0);
                k1 = mfma_bf16(x1, sl, k1);
            }
            typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
            const u32x2 va = {pack_bf16(v0[0], v0[1]), pack_bf16(v0[2], v0[3])};
            const u32x2 vb = {pack_bf16(v1[0], v1[1]), pack_bf16(v1[2], v1[3])};
            const u32x2 ka = {pack_bf16(k0[0] * p.scale, k0[1] * p.scale), pack_bf16(k0[2] * p.scale, k0[3] * p.scale)};
            const u32x2 kb = {pack_bf16(k1[0] * p.scale, k1[1] * p.scale), pack_bf16(k1[2] * p.scale, k1[3] * p.scale)};
            // The rows leave through the K and V slabs, which nothing reads in phase B (only this wave
            // touches its head's 64-byte slice of its 16 rows), and from there as whole rows.
            u32x2* const rowv = reinterpret_cast<u32x2*>(lv + (16 * jb + n) * stride + 4 * hl);
            u32x2* const rowk = reinterpret_cast<u32x2*>(lk + (16 * jb + n) * stride + 4 * hl);
            rowv[g] = va;
            rowv[4 + g] = vb;
            rowk[g] = ka;
            rowk[4 + g] = kb;
        }
        __syncthreads();  // dK, dV rows complete; slabs and exchange area are rewritten by the next window
        if (rip < (uint32_t)ROWS) {  // 16 bytes per lane, whole rows; rows beyond L are dropped by the range check
            const size_t slab_d = ((size_t)w * L * p.ldd + (size_t)hg * hpb * kHeadDim) * 2u;
            const uint32_t slab_bytes_d = (uint32_t)(L - 1) * row_d + hpb * 2u * kHeadDim;
            const uint32_t goff_d = rip * row_d + col * 16u;
            __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, lk[loff]), make_rsrc((char*)p.dk + slab_d, slab_bytes_d), goff_d, 0, 0);
            __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, lv[loff]), make_rsrc((char*)p.dv + slab_d, slab_bytes_d), goff_d, 0, 0);
        }
        if (has_next) park();  // each thread overwrites the slab cells it has just read out
    }

    if (DB && active) {
        // partial sums in register order: [slot][head][qb][jb][lane] float4 -- contiguous 16-byte stores
        f32x4* dst = reinterpret_cast<f32x4*>(p.partial) + ((size_t)bw * p.heads + h) * (NB * NB * 64) + lane;
#pragma unroll
        for (int jb = 0; jb < NB; ++jb) dst[(role * NB + jb) * 64] = dbacc[jb];
    }
}

template <int NB, bool BM, bool DB, int KT, bool PW>
hipError_t launch_coop_pw(const BwdArgs& a, const CoopGeom& gm, unsigned grid, unsigned block, size_t lds,
                          hipStream_t st) {
    if (PW) lds += (size_t)16 * NB * 4;  // the window's labels
    {
        const hipError_t e = allow_lds(reinterpret_cast<const void*>(&bwd_bf16_coop_kernel<NB, BM, DB, KT, PW>), lds);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL((bwd_bf16_coop_kernel<NB, BM, DB, KT, PW>), dim3(grid), dim3(block), lds, st, a, gm);
    return hipGetLastError();
}

template <int NB, bool BM, bool DB, int KT>
hipError_t launch_coop_kt(const BwdArgs& a, const CoopGeom& gm, unsigned grid, unsigned block, size_t lds,
                          hipStream_t st) {
    if constexpr (BM) {
        if (a.per_window) return launch_coop_pw<NB, true, DB, KT, true>(a, gm, grid, block, lds, st);
    }
    return launch_coop_pw<NB, BM, DB, KT, false>(a, gm, grid, block, lds, st);
}

template <int NB, bool BM, bool DB>
hipError_t launch_coop_one(const BwdArgs& a, const CoopGeom& gm, unsigned grid, unsigned block, size_t lds,
                           hipStream_t st) {
    // a single column in the last key block (L = 16 (NB - 1) + 1: the 7 x 7 window): the trimmed variant
    if (a.L == 16 * (NB - 1) + 1 && NB > 1) return launch_coop_kt<NB, BM, DB, 1>(a, gm, grid, block, lds, st);
    return launch_coop_kt<NB, BM, DB, 4>(a, gm, grid, block, lds, st);
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
    const size_t lds = (size_t)4 * 16 * NB * (4 * hpb + 1) * 16 + (size_t)hpb * 4 * (16 * NB) * 64 * 2;
    gm.xcd_remap = (hpb % 2 == 1 && groups > 1) ? 1u : 0u;
    gm.xcd_q = grid / 8u;
    gm.xcd_r = grid % 8u;
    const bool bm = a.bias || has_mask(a), db = a.dbias != nullptr;
    if (bm)
        return db ? launch_coop_one<NB, true, true>(a, gm, grid, block, lds, st)
                  : launch_coop_one<NB, true, false>(a, gm, grid, block, lds, st);
    return db ? launch_coop_one<NB, false, true>(a, gm, grid, block, lds, st)
              : launch_coop_one<NB, false, false>(a, gm, grid, block, lds, st);
}

}  // namespace

// Heads per workgroup of the cooperative kernel: all of them when the row has at most 3 (the
// slab is then whole rows: full 128-byte lines in and out).  Beyond that, groups of 2 (whole
// lines) or 3 heads with one workgroup per CU, or single heads with three 4-wave workgroups per
// CU that run their phases independently but fetch and store 64-byte halves of lines.  Measured,
// backward with dBias: 4, 8, 16, 32 heads in pairs are 16-18 % faster than singly (Swin-B stages
// 1-4); 6 and 12 heads in threes 14 % and 8 % faster at 8192 and 2048 windows (Swin-L stages 1, 2)
// but 2-5 % slower at 512 and 128 windows (Swin-T stages 3, 4), where a workgroup meets too few
// windows to make up for its longer set-up: threes from 16 windows per workgroup on.  With 48
// heads (Swin-L stage 4, 128 windows) threes are 8 % faster already at 8 windows per workgroup
// (24 heads at 256 windows: no difference either way).
int coop_heads_per_block(int heads, long long N) {
    if (heads <= kCoopMaxHeads) return heads;
    if (heads % 3 == 0)   // windows per workgroup = N / (compute units / (heads / 3))
        return (N * heads >= 16LL * 3 * cu_count() || (heads >= 48 && N * heads >= 8LL * 3 * cu_count())) ? 3 : 1;
    return heads % 2 == 0 ? 2 : 1;
}

// Window positions walked in parallel: about one workgroup per CU (LDS allows no more), a
// multiple of nW so that every workgroup keeps one mask tile; 0 = the kernel does not apply.
int coop_slots(long long N, int heads, int nW) {
    const int hpb = coop_heads_per_block(heads, N);
    if (hpb == 0 || nW < 1) return 0;
    const int groups = heads / hpb;
    const int per_cu = hpb == 3 ? 1 : (hpb == 2 ? 1 : 3);
    long long G = ((long long)cu_count() * per_cu / groups) / nW * nW;
    if (G > N) G = N / nW * nW;
    if (G < nW || G <= 0) return 0;
    return (int)G;
}

hipError_t launch_backward_bf16_coop(const BwdArgs& a, hipStream_t s) {
    const int hpb = coop_heads_per_block(a.heads, a.N);
    switch ((a.L + 15) / 16) {
        case 1: return launch_coop_nb<1>(a, hpb, s);
        case 2: return launch_coop_nb<2>(a, hpb, s);
        case 3: return launch_coop_nb<3>(a, hpb, s);
        case 4: return launch_coop_nb<4>(a, hpb, s);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace fwa
