// Forward kernel for L <= 64 with LDS-staged, fully coalesced global traffic.
//
// Same arithmetic and register layouts as fwd_bf16_kernel (one wave per
// (window, head) tile, S^T in the accumulators, softmax across the 4 lanes
// sharing n, O^T = V^T P^T), but the workgroup moves its slab of Q, K, V --
// the rows of one window restricted to the workgroup's heads, a run of
// whole 128-byte lines per row -- with 16-byte loads whose lanes cover
// consecutive addresses, parks it in LDS, and every wave then picks its own
// head's operands out of LDS:
//   K, Q rows : ds_read_b128  (row n, 16 B at 16 g of the head's 64 B slice)
//   V columns : ds_read_b64_tr_b16, the transposing read: lane t of a row of 16
//               lanes receives X[i0 + e][j0 + t], e = 0..3, i.e. the k-slots of
//               the A operand of O^T with the channel on the lane.
// The output goes back through LDS the same way and leaves as whole rows.
// Reading 64-byte head slices straight from HBM (the other kernel) costs about
// 8 % of bandwidth against this pattern.
#include "fwa_device.h"
#include "fwa_internal.h"
#include "fwa_softmax.h"

namespace fwa {
namespace {

struct StagedGeom {
    FastDiv groups;            // workgroups per window
    FastDiv lanes_per_row;     // 4 * heads_per_block lanes move one slab row
    uint32_t heads_per_block;
};

// QS = waves per head: 1 (a wave walks all query blocks of its head), 2 or 4 (a wave takes every
// QS-th query block: less work per wave, for calls with too few tiles to fill the chip otherwise).
template <int NB, bool BM, int QS>
__global__ void __launch_bounds__(64 * kWavesPerBlock * QS) fwd_bf16_staged_kernel(FwdArgs p, StagedGeom gm) {
    constexpr int NB2 = (NB + 1) / 2;
    constexpr int ROWS = 16 * NB;
    constexpr int PASSES = (NB + QS - 1) / QS;  // the workgroup moves 16 QS slab rows per pass
    extern __shared__ __attribute__((aligned(16))) uint4 lds[];  // [3][ROWS][stride]: K, V, Q (then O)
    const int tid = threadIdx.x, lane = tid & 63;
    const int n = lane & 15, g = lane >> 4;
    const uint32_t wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const uint32_t hl = wv / QS;  // head inside the workgroup
    const int qs = (int)(wv % QS);
    const uint32_t w = fastdiv(blockIdx.x, gm.groups);
    const uint32_t hg = blockIdx.x - w * gm.groups.d;
    const uint32_t hpb = gm.heads_per_block;
    const uint32_t h = hg * hpb + hl;
    const int L = p.L;
    // token rows are p.ldq (q, k, v) resp. p.ldo (o) elements apart; window w starts at row w L
    const uint32_t row_bytes = (uint32_t)p.ldq * 2u, row_out = (uint32_t)p.ldo * 2u;
    const uint32_t stride = 4u * hpb + 1u;  // LDS row stride in 16-byte units (one unit of padding)

    // ---- stage the slab: thread -> (row of a 16-row pass, 16-byte column)
    const uint32_t rip = fastdiv((uint32_t)tid, gm.lanes_per_row);
    const uint32_t col = (uint32_t)tid - rip * gm.lanes_per_row.d;
    const size_t slab = ((size_t)w * L * p.ldq + (size_t)hg * hpb * kHeadDim) * 2u;
    const uint32_t slab_bytes = (uint32_t)(L - 1) * row_bytes + hpb * 2u * kHeadDim;
    const __amdgpu_buffer_rsrc_t rq = make_rsrc((const char*)p.q + slab, slab_bytes);
    const __amdgpu_buffer_rsrc_t rk = make_rsrc((const char*)p.k + slab, slab_bytes);
    const __amdgpu_buffer_rsrc_t rv = make_rsrc((const char*)p.v + slab, slab_bytes);
    const __amdgpu_buffer_rsrc_t ro = make_rsrc((char*)p.o + ((size_t)w * L * p.ldo + (size_t)hg * hpb * kHeadDim) * 2u,
                                                (uint32_t)(L - 1) * row_out + hpb * 2u * kHeadDim);
    const uint32_t goff = rip * row_bytes + col * 16u;  // plus 16 t rows
    const uint32_t goff_o = rip * row_out + col * 16u;
    const uint32_t loff = rip * stride + col;           // plus 16 t rows, in uint4 units
    u32x4 sk[PASSES], sv[PASSES], sq[PASSES];
#pragma unroll
    for (int t = 0; t < PASSES; ++t) {
        // rows beyond L lie outside the descriptor and arrive as zeros
        sk[t] = __builtin_amdgcn_raw_buffer_load_b128(rk, goff + 16 * QS * t * row_bytes, 0, 0);
        sq[t] = __builtin_amdgcn_raw_buffer_load_b128(rq, goff + 16 * QS * t * row_bytes, 0, 0);
        sv[t] = __builtin_amdgcn_raw_buffer_load_b128(rv, goff + 16 * QS * t * row_bytes, 0, 0);
    }
    // The additive term of this wave's query blocks, requested right behind the slab so that its
    // trip to L2 overlaps the slab's trip to HBM instead of following the score products.
    constexpr int NQ = (NB + QS - 1) / QS;  // query blocks of this wave: qs, qs + QS, ...
    f32x4 add[NQ][NB];
    if (BM) {
        const uint32_t hh = h < (uint32_t)p.heads ? h : 0u;
        const BiasSrc rb = bias_of_head(p, hh);
        const MaskSrc msk = mask_of_window(p, w);
        AddendGlobal rows[NQ];  // blocks beyond the last one: rows outside the tile, zeros
#pragma unroll
        for (int t = 0; t < NQ; ++t) rows[t] = addend_at(rb, msk, (uint32_t)(16 * (qs + QS * t) + n), 4u * g, (uint32_t)L);
        fill_rows<NQ, NB>(add, rows, kLog2e);
    }
    uint4* const lk = lds;
    uint4* const lv = lds + ROWS * stride;
    uint4* const lq = lds + 2 * ROWS * stride;
#pragma unroll
    for (int t = 0; t < PASSES; ++t) {
        if (QS == 1 || 16 * QS * t + rip < (uint32_t)ROWS) {
            lk[loff + 16 * QS * t * stride] = __builtin_bit_cast(uint4, sk[t]);
            lq[loff + 16 * QS * t * stride] = __builtin_bit_cast(uint4, sq[t]);
            lv[loff + 16 * QS * t * stride] = __builtin_bit_cast(uint4, sv[t]);
        }
    }
    __syncthreads();

    // ---- operands of this wave's head
    bf16x8 kop[NB], qop[NQ];
#pragma unroll
    for (int b = 0; b < NB; ++b) kop[b] = __builtin_bit_cast(bf16x8, lk[(16 * b + n) * stride + 4 * hl + g]);
#pragma unroll
    for (int b = 0; b < NQ; ++b)  // a block beyond the last one reads inside the slab area and is never used
        qop[b] = __builtin_bit_cast(bf16x8, lq[((16 * (qs + QS * b)) % ROWS + n) * stride + 4 * hl + g]);
    // V: A operands of O^T per pair of key blocks, channels 0..15 and 16..31.
    // lane r of a row points at V[i0 + (r >> 2)][j0 + 4 (r & 3)], i0 = first key of the 4 the lane row owns
    bf16x8 vop[NB2][2];
    {
        const uint16_t* lvh = reinterpret_cast<const uint16_t*>(lv) + 32 * hl;
        const uint32_t el = (4 * g + (n >> 2)) * (stride * 8u) + 4 * (n & 3);
#pragma unroll
        for (int kp = 0; kp < NB2; ++kp)
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                const uint2 a = lds_read_tr(lvh + el + (32 * kp) * (stride * 8u) + 16 * c);
                uint2 b = {0u, 0u};
                if (2 * kp + 1 < NB) b = lds_read_tr(lvh + el + (32 * kp + 16) * (stride * 8u) + 16 * c);
                const u32x4 v = {a.x, a.y, b.x, b.y};
                vop[kp][c] = as_bf16x8(v);
            }
    }

    const float sl2 = p.scale * kLog2e;

#pragma unroll
    for (int it = 0; it < NQ; ++it) {
        const int qb = qs + QS * it;
        if (16 * qb >= L) break;  // uniform
        f32x4 s[NB];
#pragma unroll
        for (int jb = 0; jb < NB; ++jb) {
            const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
            s[jb] = mfma_bf16(kop[jb], qop[it], zero);  // S[16 qb + n][16 jb + 4g + r]
        }
        const AddendRegs<NB> addend = {add[it]};
        const float inv = softmax_block<NB, BM>(s, sl2, addend, L, g);

        f32x4 o0 = {0.f, 0.f, 0.f, 0.f}, o1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kp = 0; kp < NB2; ++kp) {
            const bf16x8 pop = prob_operand<NB>(s, kp);
            o0 = mfma_bf16(vop[kp][0], pop, o0);  // o0[r] = O[16 qb + n][4g + r]
            o1 = mfma_bf16(vop[kp][1], pop, o1);  // o1[r] = O[16 qb + n][16 + 4g + r]
        }
        // park the row in the Q tile (only this wave reads or writes its head's 64 B slice)
        uint2 lo, hi;
        lo.x = pack_bf16(o0[0] * inv, o0[1] * inv);
        lo.y = pack_bf16(o0[2] * inv, o0[3] * inv);
        hi.x = pack_bf16(o1[0] * inv, o1[1] * inv);
        hi.y = pack_bf16(o1[2] * inv, o1[3] * inv);
        uint2* row = reinterpret_cast<uint2*>(lq + (16 * qb + n) * stride + 4 * hl);
        row[g] = lo;
        row[4 + g] = hi;
    }
    __syncthreads();
    // ---- whole rows back to global memory; rows beyond L are dropped by the range check
#pragma unroll
    for (int t = 0; t < PASSES; ++t) {
        if (QS == 1 || 16 * QS * t + rip < (uint32_t)ROWS) {
            const u32x4 v = __builtin_bit_cast(u32x4, lq[loff + 16 * QS * t * stride]);
            __builtin_amdgcn_raw_buffer_store_b128(v, ro, goff_o + 16 * QS * t * row_out, 0, 0);
        }
    }
}

// ---------------------------------------------------------------------------
// Persistent variant of the staged kernel for calls with a bias and/or mask.
//
// Re-reading the bias tile (L x L fp32 per head, as large as the head's Q/K/V/O traffic) for
// every window costs as much time as the window's own data even though it comes from L2.  Here a
// workgroup keeps its heads and walks the windows bw, bw + G, bw + 2G, ...; G is a multiple of
// nW, so all of them share the mask tile bw % nW.  Each wave therefore loads
// (bias[h] + mask[bw % nW]) * log2e ONCE, straight into the registers of the score layout, and
// the per-window work is that of the bias-free kernel plus one fused multiply-add per score.
// The slab of the next window is requested before the current one is computed.
// PW: the mask comes as labels whose period does not divide G; the bias alone stays in registers,
// the labels of a window travel with its slab and the mask is formed per score (see
// AddendRegsLabels).
template <int NB, bool PW>
__global__ void __launch_bounds__(64 * kWavesPerBlock) fwd_bf16_persistent_kernel(FwdArgs p, StagedGeom gm, uint32_t G) {
    constexpr int NB2 = (NB + 1) / 2;
    constexpr int ROWS = 16 * NB;
    extern __shared__ __attribute__((aligned(16))) uint4 lds[];  // [3][ROWS][stride]: K, V, Q (then O); then (PW) [ROWS] labels
    const int tid = threadIdx.x, lane = tid & 63;
    const int n = lane & 15, g = lane >> 4;
    const uint32_t hl = __builtin_amdgcn_readfirstlane(tid >> 6);
    const uint32_t bw = fastdiv(blockIdx.x, gm.groups);
    const uint32_t hg = blockIdx.x - bw * gm.groups.d;
    const uint32_t hpb = gm.heads_per_block;
    const uint32_t h = hg * hpb + hl;
    const int L = p.L;
    const uint32_t row_bytes = (uint32_t)p.ldq * 2u, row_out = (uint32_t)p.ldo * 2u;
    const uint32_t stride = 4u * hpb + 1u;
    const float sl2 = p.scale * kLog2e;

    const uint32_t rip = fastdiv((uint32_t)tid, gm.lanes_per_row);
    const uint32_t col = (uint32_t)tid - rip * gm.lanes_per_row.d;
    const uint32_t slab_bytes = (uint32_t)(L - 1) * row_bytes + hpb * 2u * kHeadDim;
    const uint32_t goff = rip * row_bytes + col * 16u;
    const uint32_t goff_o = rip * row_out + col * 16u;
    const uint32_t loff = rip * stride + col;
    uint4* const lk = lds;
    uint4* const lv = lds + ROWS * stride;
    uint4* const lq = lds + 2 * ROWS * stride;
    int* const llab = reinterpret_cast<int*>(lds + 3 * ROWS * stride);
    const uint16_t* const lvh = reinterpret_cast<const uint16_t*>(lv) + 32 * hl +
                                (4 * g + (n >> 2)) * (stride * 8u) + 4 * (n & 3);

    u32x4 sk[NB], sv[NB], sq[NB];
    i32x4 slab_labels = {0, 0, 0, 0};  // PW: labels 4 tid .. 4 tid + 3 of the requested window (0 beyond L)
    auto request = [&](uint32_t w) {
        const size_t slab = ((size_t)w * L * p.ldq + (size_t)hg * hpb * kHeadDim) * 2u;
        const __amdgpu_buffer_rsrc_t rq = make_rsrc((const char*)p.q + slab, slab_bytes);
        const __amdgpu_buffer_rsrc_t rk = make_rsrc((const char*)p.k + slab, slab_bytes);
        const __amdgpu_buffer_rsrc_t rv = make_rsrc((const char*)p.v + slab, slab_bytes);
#pragma unroll
        for (int t = 0; t < NB; ++t) {
            sk[t] = __builtin_amdgcn_raw_buffer_load_b128(rk, goff + 16 * t * row_bytes, 0, 0);
            sq[t] = __builtin_amdgcn_raw_buffer_load_b128(rq, goff + 16 * t * row_bytes, 0, 0);
            sv[t] = __builtin_amdgcn_raw_buffer_load_b128(rv, goff + 16 * t * row_bytes, 0, 0);
        }
        if (PW && hl == 0)  // one wave fetches them
            slab_labels = load_i32x4(make_rsrc(p.labels + (size_t)(w % (uint32_t)p.nW) * L, (uint32_t)L * 4u), (uint32_t)tid * 16u);
    };
    auto park = [&]() {
#pragma unroll
        for (int t = 0; t < NB; ++t) {
            lk[loff + 16 * t * stride] = __builtin_bit_cast(uint4, sk[t]);
            lq[loff + 16 * t * stride] = __builtin_bit_cast(uint4, sq[t]);
            lv[loff + 16 * t * stride] = __builtin_bit_cast(uint4, sv[t]);
        }
        if (PW && tid < ROWS / 4) reinterpret_cast<i32x4*>(llab)[tid] = slab_labels;
    };
    if (bw < (uint32_t)p.N) request(bw);  // in flight while the additive term is fetched
    // the additive term of this wave's head and this workgroup's mask tile, in score layout
    f32x4 add[NB][NB];
    {
        const BiasSrc rb = bias_of_head(p, h);
        const MaskSrc msk = PW ? MaskSrc{make_rsrc(nullptr, 0), 0.f, false} : mask_of_window(p, bw);
        fill_rows<NB, NB>(add, rb, msk, (uint32_t)n, 4u * g, (uint32_t)L, kLog2e);
    }
    const float mv = p.mask_value * kLog2e;

    if (bw < (uint32_t)p.N) park();

    // The next slab is parked at the END of an iteration: there the loads it waits for are always
    // older than this iteration's output stores, so the wait counts the stores out.  At the top of
    // the loop the compiler must assume the worse of the two ways in and would wait for the stores.
    for (uint32_t w = bw; w < (uint32_t)p.N; w += G) {
        const bool has_next = w + G < (uint32_t)p.N;
        __syncthreads();
        bf16x8 kop[NB], qop[NB];
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            kop[b] = __builtin_bit_cast(bf16x8, lk[(16 * b + n) * stride + 4 * hl + g]);
            qop[b] = __builtin_bit_cast(bf16x8, lq[(16 * b + n) * stride + 4 * hl + g]);
        }
        bf16x8 vop[NB2][2];
#pragma unroll
        for (int kp = 0; kp < NB2; ++kp)
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                const uint2 a = lds_read_tr(lvh + (32 * kp) * (stride * 8u) + 16 * c);
                uint2 b = {0u, 0u};
                if (2 * kp + 1 < NB) b = lds_read_tr(lvh + (32 * kp + 16) * (stride * 8u) + 16 * c);
                const u32x4 v = {a.x, a.y, b.x, b.y};
                vop[kp][c] = as_bf16x8(v);
            }
        int tq[NB];  // PW: labels of this lane's query rows
#pragma unroll
        for (int b = 0; b < NB; ++b) tq[b] = PW ? llab[16 * b + n] : 0;
        if (has_next) request(w + G);  // in flight while this window is computed

#pragma unroll
        for (int qb = 0; qb < NB; ++qb) {
            f32x4 s[NB];
#pragma unroll
            for (int jb = 0; jb < NB; ++jb) {
                const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
                s[jb] = mfma_bf16(kop[jb], qop[qb], zero);
            }
            float inv;
            if (PW) {
                const AddendRegsLabels<NB> addend = {add[qb], llab, tq[qb], mv, g};
                inv = softmax_block<NB, true>(s, sl2, addend, L, g);
            } else {
                const AddendRegs<NB> addend = {add[qb]};
                inv = softmax_block<NB, true>(s, sl2, addend, L, g);
            }
            f32x4 o0 = {0.f, 0.f, 0.f, 0.f}, o1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kp = 0; kp < NB2; ++kp) {
                const bf16x8 pop = prob_operand<NB>(s, kp);
                o0 = mfma_bf16(vop[kp][0], pop, o0);
                o1 = mfma_bf16(vop[kp][1], pop, o1);
            }
            uint2 lo, hi;
            lo.x = pack_bf16(o0[0] * inv, o0[1] * inv);
            lo.y = pack_bf16(o0[2] * inv, o0[3] * inv);
            hi.x = pack_bf16(o1[0] * inv, o1[1] * inv);
            hi.y = pack_bf16(o1[2] * inv, o1[3] * inv);
            uint2* row = reinterpret_cast<uint2*>(lq + (16 * qb + n) * stride + 4 * hl);
            row[g] = lo;
            row[4 + g] = hi;
        }
        __syncthreads();
        {
            const size_t slab = ((size_t)w * L * p.ldo + (size_t)hg * hpb * kHeadDim) * 2u;
            const __amdgpu_buffer_rsrc_t ro = make_rsrc((char*)p.o + slab, (uint32_t)(L - 1) * row_out + hpb * 2u * kHeadDim);
#pragma unroll
            for (int t = 0; t < NB; ++t) {
                const u32x4 v = __builtin_bit_cast(u32x4, lq[loff + 16 * t * stride]);
                __builtin_amdgcn_raw_buffer_store_b128(v, ro, goff_o + 16 * t * row_out, 0, 0);
            }
        }
        __syncthreads();  // every wave has copied its output rows out of the Q tile
        if (has_next) park();
    }
}

// ---------------------------------------------------------------------------
// Row-blocked forward for 64 < L <= 256 (paper Discussion: such windows do not fit its
// on-chip tile; here K and V of the head stay on chip and the queries are walked in blocks
// of 16).  The workgroup parks the K and V slabs of its heads in LDS once; QW waves share
// each head and take every QW-th 16-query block.  Per block a wave reads its K operands
// (ds_read_b128) and V operands (transposing reads) from LDS, keeps the 16 x L score block
// in registers, and loads Q / stores O for its own rows directly.
struct RowBlockGeom {
    FastDiv groups;         // workgroups per window
    FastDiv lanes_per_row;  // 4 * heads_per_block
    uint32_t heads_per_block;
    uint32_t xcd_remap, xcd_q, xcd_r;
};

template <int NB, bool BM, int QW>
__global__ void __launch_bounds__(64 * 2 * QW) fwd_bf16_rowblock_kernel(FwdArgs p, RowBlockGeom gm) {
    constexpr int NB2 = (NB + 1) / 2;
    constexpr int ROWS = 16 * NB;
    constexpr int RPP = 16 * QW;                       // slab rows the workgroup moves per pass
    constexpr int PASSES = (ROWS + RPP - 1) / RPP;
    extern __shared__ __attribute__((aligned(16))) uint4 lds[];  // [2][ROWS][stride]: K, V
    const int tid = threadIdx.x, lane = tid & 63;
    const int n = lane & 15, g = lane >> 4;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const uint32_t hl = wave / QW, qs = wave % QW;
    const uint32_t lb = gm.xcd_remap ? xcd_logical_block(blockIdx.x, gm.xcd_q, gm.xcd_r) : blockIdx.x;
    const uint32_t w = fastdiv(lb, gm.groups);
    const uint32_t hg = lb - w * gm.groups.d;
    const uint32_t hpb = gm.heads_per_block;
    const uint32_t h = hg * hpb + hl;
    const int L = p.L;
    const uint32_t row_bytes = (uint32_t)p.ldq * 2u, row_out = (uint32_t)p.ldo * 2u;
    const uint32_t stride = 4u * hpb + 1u;  // LDS row stride in 16-byte units

    uint4* const lk = lds;
    uint4* const lv = lds + ROWS * stride;
    {
        const uint32_t rip = fastdiv((uint32_t)tid, gm.lanes_per_row);  // 0..RPP-1
        const uint32_t col = (uint32_t)tid - rip * gm.lanes_per_row.d;
        const size_t slab = ((size_t)w * L * p.ldq + (size_t)hg * hpb * kHeadDim) * 2u;
        const uint32_t slab_bytes = (uint32_t)(L - 1) * row_bytes + hpb * 2u * kHeadDim;
        const __amdgpu_buffer_rsrc_t rk = make_rsrc((const char*)p.k + slab, slab_bytes);
        const __amdgpu_buffer_rsrc_t rv = make_rsrc((const char*)p.v + slab, slab_bytes);
        u32x4 sk[PASSES], sv[PASSES];
#pragma unroll
        for (int t = 0; t < PASSES; ++t) {
            const uint32_t off = (RPP * t + rip) * row_bytes + col * 16u;  // rows beyond L arrive as zeros
            sk[t] = __builtin_amdgcn_raw_buffer_load_b128(rk, off, 0, 0);
            sv[t] = __builtin_amdgcn_raw_buffer_load_b128(rv, off, 0, 0);
        }
#pragma unroll
        for (int t = 0; t < PASSES; ++t) {
            const uint32_t row = RPP * t + rip;
            if (row < (uint32_t)ROWS) {
                lk[row * stride + col] = __builtin_bit_cast(uint4, sk[t]);
                lv[row * stride + col] = __builtin_bit_cast(uint4, sv[t]);
            }
        }
    }
    __syncthreads();

    const uint32_t tile_bytes = (uint32_t)(L - 1) * row_bytes + 2u * kHeadDim;
    const size_t tile = ((size_t)w * L * p.ldq + (size_t)h * kHeadDim) * 2u;
    const __amdgpu_buffer_rsrc_t rq = make_rsrc((const char*)p.q + tile, tile_bytes);
    const __amdgpu_buffer_rsrc_t ro = make_rsrc((char*)p.o + ((size_t)w * L * p.ldo + (size_t)h * kHeadDim) * 2u,
                                                (uint32_t)(L - 1) * row_out + 2u * kHeadDim);
    const uint32_t off_row = (uint32_t)n * row_bytes + 16u * g;
    const float sl2 = p.scale * kLog2e;
    BiasSrc rb = no_bias();
    MaskSrc msk = {make_rsrc(nullptr, 0), 0.f, false};
    if (BM) {
        rb = bias_of_head(p, h);
        msk = mask_of_window(p, w);
    }
    const uint4* const lkh = lk + n * stride + 4 * hl + g;  // K[16 jb + n][8g..] at lkh[16 jb * stride]
    const uint16_t* const lvh = reinterpret_cast<const uint16_t*>(lv) + 32 * hl +
                                (4 * g + (n >> 2)) * (stride * 8u) + 4 * (n & 3);

    u32x4 qnext = __builtin_amdgcn_raw_buffer_load_b128(rq, off_row + 16 * qs * row_bytes, 0, 0);
    for (int qb = qs; qb < NB; qb += QW) {
        const bf16x8 qop = as_bf16x8(qnext);
        if (qb + QW < NB) qnext = __builtin_amdgcn_raw_buffer_load_b128(rq, off_row + 16 * (qb + QW) * row_bytes, 0, 0);
        f32x4 s[NB];
#pragma unroll
        for (int jb = 0; jb < NB; ++jb) {
            const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
            const bf16x8 kop = __builtin_bit_cast(bf16x8, lkh[16 * jb * stride]);
            s[jb] = mfma_bf16(kop, qop, zero);  // S[16 qb + n][16 jb + 4g + r]
        }
        const AddendGlobal addend = addend_at(rb, msk, (uint32_t)(16 * qb + n), 4u * g, (uint32_t)L);
        float mul, sum = 0.f;
        const float mb = softmax_scale_max<NB, BM>(s, sl2, addend, L, g, mul);
        f32x4 o0 = {0.f, 0.f, 0.f, 0.f}, o1 = {0.f, 0.f, 0.f, 0.f}, osum = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kp = 0; kp < NB2; ++kp) {
            // the V operands of this pair of key blocks are requested before its exponentials
            u32x4 v[2];
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                const uint2 a = lds_read_tr(lvh + (32 * kp) * (stride * 8u) + 16 * c);
                uint2 b = {0u, 0u};
                if (2 * kp + 1 < NB) b = lds_read_tr(lvh + (32 * kp + 16) * (stride * 8u) + 16 * c);
                v[c] = u32x4{a.x, a.y, b.x, b.y};
            }
            softmax_exp_pair<NB, false>(s, kp, mul, mb, sum);
            const bf16x8 pop = prob_operand<NB>(s, kp);
            o0 = mfma_bf16(as_bf16x8(v[0]), pop, o0);  // o0[r] = O[16 qb + n][4g + r]
            o1 = mfma_bf16(as_bf16x8(v[1]), pop, o1);  // o1[r] = O[16 qb + n][16 + 4g + r]
            osum = mfma_bf16(ones_operand(), pop, osum);  // every component: the row sum of query 16 qb + n
        }
        const float inv = __builtin_amdgcn_rcpf(osum[0]);
        typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
        u32x2 lo, hi;
        lo.x = pack_bf16(o0[0] * inv, o0[1] * inv);
        lo.y = pack_bf16(o0[2] * inv, o0[3] * inv);
        hi.x = pack_bf16(o1[0] * inv, o1[1] * inv);
        hi.y = pack_bf16(o1[2] * inv, o1[3] * inv);
        const uint32_t off_o = (uint32_t)(16 * qb + n) * row_out + 8u * g;
        __builtin_amdgcn_raw_buffer_store_b64(lo, ro, off_o, 0, 0);
        __builtin_amdgcn_raw_buffer_store_b64(hi, ro, off_o + 32, 0, 0);
    }
}

// ---------------------------------------------------------------------------
// Row-blocked forward with bias / mask, persistent.  At these sizes the additive term is
// 4 L^2 bytes per head against 256 L bytes of Q, K, V, O per tile, and a lane's part of it
// (one query row, 4 consecutive keys per key block) is 16 bytes in a row of its own, so
// re-reading it for every window costs more than everything else.  Here a wave keeps one
// 16-query block of one head for its whole life: (bias[h] + mask[w % nW]) * log2e of those
// 16 rows sits in registers (NB float4 per lane), and the workgroup (W waves = W consecutive
// query blocks of the head; the head is split over `parts` workgroups when NB > 12) walks the
// windows bw, bw + G, ... with G a multiple of nW.  K and V of the head go through a double
// buffered LDS slab and are requested two windows ahead (one window's slabs wait in registers
// while the next one's are in flight: 4-5 % over one window ahead at L = 144 and 256); one
// barrier per window.  Workgroups that
// share 128-byte lines (the two heads of a pair, the parts of a head) are neighbours in the
// logical block order, which is mapped so that neighbours run on the same XCD.
struct RowPersistGeom {
    uint32_t groups, parts, G;  // groups = heads / HPB
    uint32_t xcd_q, xcd_r;
};

constexpr int rowpersist_waves(int nb) { return nb <= 12 ? nb : (nb + 1) / 2; }

// HPB heads per workgroup (HPB W waves): slab rows of HPB * 64 bytes, which are whole 128-byte
// lines when HPB is even or the whole token row when HPB is the head count.  Used with HPB > 1
// for L <= 64, where W <= 4.
//
// PW ("per window"): the mask comes as labels and its period does not divide G, so that a workgroup
// meets a different mask tile at every window.  Then only the bias stays in registers; the labels
// of a window travel with its slabs (requested two windows ahead, parked in LDS beside them) and
// the mask is formed per score.
template <int NB, int HPB, bool PW>
__global__ void __launch_bounds__(64 * HPB * rowpersist_waves(NB)) fwd_bf16_rowpersist_kernel(FwdArgs p, RowPersistGeom gm) {
    constexpr int W = rowpersist_waves(NB);
    constexpr int NB2 = (NB + 1) / 2;
    constexpr int ROWS = 16 * NB;
    constexpr int PASSES = (ROWS + 16 * W - 1) / (16 * W);  // the workgroup moves 16 W slab rows per pass
    constexpr uint32_t TPR = 4 * HPB;                        // threads per slab row, 16 bytes each
    constexpr uint32_t STRIDE = TPR + 1;                     // LDS row: HPB * 64 bytes of data + 16 of padding
    extern __shared__ __attribute__((aligned(16))) uint4 lds[];  // [2 buffers][K, V][ROWS][STRIDE], then (PW) [2][ROWS] labels
    const int tid = threadIdx.x, lane = tid & 63;
    const int n = lane & 15, g = lane >> 4;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const uint32_t hl = wave / W, wq = wave % W;  // head inside the workgroup, query block inside the part
    int* const llab = reinterpret_cast<int*>(lds + 2 * (2 * ROWS * STRIDE));
    uint4* const oscratch = lds + 2 * (2 * ROWS * STRIDE) + (2 * ROWS) / 4;  // behind the labels: 1 KB per wave
    const uint32_t lb = xcd_logical_block(blockIdx.x, gm.xcd_q, gm.xcd_r);
    const uint32_t part = lb % gm.parts, bh = lb / gm.parts;
    const uint32_t grp = bh % gm.groups, bw = bh / gm.groups;
    const uint32_t h = grp * HPB + hl;
    const int qb = (int)(part * W + wq);
    const bool active = qb < NB;
    const int L = p.L;
    const uint32_t row_bytes = (uint32_t)p.ldq * 2u, row_out = (uint32_t)p.ldo * 2u;
    const float sl2 = p.scale * kLog2e;

    const uint32_t srow = (uint32_t)tid / TPR, scol = (uint32_t)tid % TPR;  // slab movement: thread -> (row, 16 B column)
    const uint32_t tile_bytes = (uint32_t)(L - 1) * row_bytes + 2u * kHeadDim * HPB;
    const uint32_t off_row = (uint32_t)(16 * qb + n) * row_bytes + 64u * hl + 16u * g;
    // Register sets of slab data: while window w is computed out of LDS, the slabs of w + step
    // sit in one set (requested earlier, parked at the end of this iteration) and those of
    // w + 2 step are requested into the other, so that two windows are in flight per workgroup
    // (with a third set: w + 2 step is in flight already and w + 3 step is requested).
    struct Slab {
        u32x4 k[PASSES], v[PASSES], q;
        i32x4 lab;  // PW: labels 4 tid .. 4 tid + 3 of the window
    };
    // three windows ahead at NB > 12, whose 8 waves per workgroup may use 256 registers per lane (a third set of
    // slab registers; 3-4 % at L = 196 and 256).  At 64 < L <= 192 the set would cost the second workgroup per
    // CU or spill, and with several heads per workgroup (L <= 64) it measured no gain.
    constexpr bool D3 = HPB == 1 && NB > 12;
    constexpr uint32_t AHEAD = D3 ? 3u : 2u;
    Slab sa, sb, sc;
    sa.q = sb.q = sc.q = u32x4{0u, 0u, 0u, 0u};
    sa.lab = sb.lab = sc.lab = i32x4{0, 0, 0, 0};
    auto request = [&](Slab& d, uint32_t w) {
        const size_t tile = ((size_t)w * L * p.ldq + (size_t)grp * HPB * kHeadDim) * 2u;
        const __amdgpu_buffer_rsrc_t rk = make_rsrc((const char*)p.k + tile, tile_bytes);
        const __amdgpu_buffer_rsrc_t rv = make_rsrc((const char*)p.v + tile, tile_bytes);
#pragma unroll
        for (int t = 0; t < PASSES; ++t) {
            const uint32_t off = (16 * W * t + srow) * row_bytes + scol * 16u;  // rows beyond L arrive as zeros
            d.k[t] = __builtin_amdgcn_raw_buffer_load_b128(rk, off, 0, 0);
            d.v[t] = __builtin_amdgcn_raw_buffer_load_b128(rv, off, 0, 0);
        }
        if (active)
            d.q = __builtin_amdgcn_raw_buffer_load_b128(make_rsrc((const char*)p.q + tile, tile_bytes), off_row, 0, 0);
        if (PW && wave == 0)  // one wave fetches them; tokens beyond L lie outside the descriptor: label 0
            d.lab = load_i32x4(make_rsrc(p.labels + (size_t)(w % (uint32_t)p.nW) * L, (uint32_t)L * 4u), (uint32_t)tid * 16u);
    };
    auto park = [&](const Slab& d, uint32_t b) {
        uint4* const dk = lds + b * (2 * ROWS * STRIDE);
        uint4* const dv = dk + ROWS * STRIDE;
#pragma unroll
        for (int t = 0; t < PASSES; ++t) {
            const uint32_t row = 16 * W * t + srow;
            if (row < (uint32_t)ROWS) {
                dk[row * STRIDE + scol] = __builtin_bit_cast(uint4, d.k[t]);
                dv[row * STRIDE + scol] = __builtin_bit_cast(uint4, d.v[t]);
            }
        }
        if (PW && tid < ROWS / 4) reinterpret_cast<i32x4*>(llab + b * ROWS)[tid] = d.lab;
    };
    // The windows of this workgroup: w0, w0 + step, ... below `end`
    uint32_t w0 = bw, step = gm.G, end = (uint32_t)p.N;
    if (w0 < end) request(sa, w0);  // in flight while the additive term is fetched
    if (w0 + step < end) request(sb, w0 + step);
    if (D3 && w0 + 2 * step < end) request(sc, w0 + 2 * step);
    f32x4 add[NB];
    {
        const BiasSrc rb = bias_of_head(p, h);
        // rows beyond L (and the whole block of an idle wave) fall outside the descriptors: zeros
        const MaskSrc msk = PW ? MaskSrc{make_rsrc(nullptr, 0), 0.f, false} : mask_of_window(p, w0);
        addend_at(rb, msk, active ? (uint32_t)(16 * qb + n) : (uint32_t)L, 4u * g, (uint32_t)L).fill(add, kLog2e);
    }
    const float mv = p.mask_value * kLog2e;
    if (w0 < end) park(sa, 0);

    // One window: K, V of window w are in LDS buffer `buf`, its Q rows in cur.q; nxt holds window
    // w + step.  Request w + 2 step into cur, one barrier, compute, store, then park nxt in the
    // other buffer.  That buffer was last read in the previous iteration, which every wave has left
    // before any wave passes this iteration's barrier; and parking after the stores means the wait
    // in front of it counts the stores and the younger loads out instead of waiting for them.
    auto window = [&](uint32_t w, Slab& cur, const Slab& nxt, uint32_t buf) {
        const bool has_next = w + step < end;
        uint4* const lk = lds + buf * (2 * ROWS * STRIDE);
        uint4* const lv = lk + ROWS * STRIDE;
        const bf16x8 qop = as_bf16x8(cur.q);
        __syncthreads();
        if (w + AHEAD * step < end) request(cur, w + AHEAD * step);
        if (active) {
            const uint4* const lkh = lk + n * STRIDE + 4 * hl + g;  // K[16 jb + n][8g..] of head hl at lkh[16 jb * STRIDE]
            const uint16_t* const lvh =
                reinterpret_cast<const uint16_t*>(lv) + 32 * hl + (4 * g + (n >> 2)) * (STRIDE * 8u) + 4 * (n & 3);
            f32x4 s[NB];
#pragma unroll
            for (int jb = 0; jb < NB; ++jb) {
                const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
                s[jb] = mfma_bf16(__builtin_bit_cast(bf16x8, lkh[16 * jb * STRIDE]), qop, zero);  // S[16 qb + n][16 jb + 4g + r]
            }
            float mul, sum = 0.f, mb;
            if (PW) {
                const int* const lab = llab + buf * ROWS;
                const AddendRegsLabels<NB> addend = {add, lab, lab[16 * qb + n], mv, g};
                mb = softmax_scale_max<NB, true>(s, sl2, addend, L, g, mul);
            } else {
                const AddendRegs<NB> addend = {add};
                mb = softmax_scale_max<NB, true>(s, sl2, addend, L, g, mul);
            }
            f32x4 o0 = {0.f, 0.f, 0.f, 0.f}, o1 = {0.f, 0.f, 0.f, 0.f}, osum = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kp = 0; kp < NB2; ++kp) {
                // the V operands of this pair of key blocks are requested before its exponentials
                u32x4 v[2];
#pragma unroll
                for (int c = 0; c < 2; ++c) {
                    const uint2 a = lds_read_tr(lvh + (32 * kp) * (STRIDE * 8u) + 16 * c);
                    uint2 b = {0u, 0u};
                    if (2 * kp + 1 < NB) b = lds_read_tr(lvh + (32 * kp + 16) * (STRIDE * 8u) + 16 * c);
                    v[c] = u32x4{a.x, a.y, b.x, b.y};
                }
                softmax_exp_pair<NB, false>(s, kp, mul, mb, sum);
                const bf16x8 pop = prob_operand<NB>(s, kp);
                o0 = mfma_bf16(as_bf16x8(v[0]), pop, o0);  // o0[r] = O[16 qb + n][4g + r]
                o1 = mfma_bf16(as_bf16x8(v[1]), pop, o1);  // o1[r] = O[16 qb + n][16 + 4g + r]
                osum = mfma_bf16(ones_operand(), pop, osum);  // every component: the row sum of query 16 qb + n
            }
            const float inv = __builtin_amdgcn_rcpf(osum[0]);
            typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
            u32x2 lo, hi;
            lo.x = pack_bf16(o0[0] * inv, o0[1] * inv);
            lo.y = pack_bf16(o0[2] * inv, o0[3] * inv);
            hi.x = pack_bf16(o1[0] * inv, o1[1] * inv);
            hi.y = pack_bf16(o1[2] * inv, o1[3] * inv);
            const size_t tile = ((size_t)w * L * p.ldo + (size_t)h * kHeadDim) * 2u;
            const __amdgpu_buffer_rsrc_t ro = make_rsrc((char*)p.o + tile, (uint32_t)(L - 1) * row_out + 2u * kHeadDim);
            if constexpr (HPB > 1) {  // three or four heads fill the rows between them: direct stores are faster
                const uint32_t off_o = (uint32_t)(16 * qb + n) * row_out + 8u * g;
                __builtin_amdgcn_raw_buffer_store_b64(lo, ro, off_o, 0, 0);
                __builtin_amdgcn_raw_buffer_store_b64(hi, ro, off_o + 32, 0, 0);
            } else {
            // One head per workgroup: through 1 KB of LDS of this wave's own, written in accumulator order
            // and read back 16 bytes per lane, so that one store covers the wave's 16 rows x 64 bytes
            // instead of two stores of 32-byte pieces (43 -> 41 us at L = 144).
            uint4* const mine = oscratch + 64 * wave;
            u32x2* const rowo = reinterpret_cast<u32x2*>(mine + 4 * n);
            rowo[g] = lo;
            rowo[4 + g] = hi;
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
            const u32x4 rows = __builtin_bit_cast(u32x4, mine[lane]);
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_raw_buffer_store_b128(rows, ro, (uint32_t)(16 * qb + (lane >> 2)) * row_out + 16u * (uint32_t)(lane & 3), 0, 0);
            }
        }
        if (has_next) park(nxt, buf ^ 1u);
    };
    if (D3) {
        uint32_t buf = 0u;
        for (uint32_t w = w0; w < end;) {
            window(w, sa, sb, buf);
            w += step, buf ^= 1u;
            if (w >= end) break;
            window(w, sb, sc, buf);
            w += step, buf ^= 1u;
            if (w >= end) break;
            window(w, sc, sa, buf);
            w += step, buf ^= 1u;
        }
    } else {
        for (uint32_t w = w0; w < end; w += 2 * step) {
            window(w, sa, sb, 0u);
            if (w + step < end) window(w + step, sb, sa, 1u);
        }
    }
}

// LDS of one workgroup of the persistent row-blocked kernel: slabs, labels, and (one head per workgroup) 1 KB per
// wave for the output rows
template <int NB, int HPB>
constexpr size_t rowpersist_lds() {
    return (size_t)2 * 2 * 16 * NB * (4 * HPB + 1) * 16 + (size_t)2 * 16 * NB * 4 +
           (HPB == 1 ? (size_t)rowpersist_waves(NB) * 1024 : 0);
}

// Workgroups of the one-head variant a CU holds at once (registers and LDS decide), asked once per kernel.
template <int NB, bool PW>
int rowpersist_per_cu() {
    static std::atomic<int> once{0};
    int per_cu = once.load(std::memory_order_relaxed);
    if (per_cu == 0) {
        const void* fn = reinterpret_cast<const void*>(&fwd_bf16_rowpersist_kernel<NB, 1, PW>);
        int nblk = 0;
        if (allow_lds(fn, rowpersist_lds<NB, 1>()) != hipSuccess ||
            hipOccupancyMaxActiveBlocksPerMultiprocessor(&nblk, fn, 64 * rowpersist_waves(NB), rowpersist_lds<NB, 1>()) != hipSuccess)
            nblk = 1;
        per_cu = nblk < 1 ? 1 : (nblk > 2 ? 2 : nblk);  // a third one measured no faster
        once.store(per_cu, std::memory_order_relaxed);
    }
    return per_cu;
}

// Window positions walked in parallel by the persistent row-blocked kernel (as many workgroups as
// the chip holds at once, two per CU at most: 3-9 % over one per CU where two fit, L <= 128; a
// multiple of the mask period, at least two windows per workgroup); 0 = use the plain row-blocked kernel.
template <int NB>
long long rowpersist_slots(const FwdArgs& a, bool& pw) {
    const long long parts = NB <= 12 ? 1 : 2;
    const long long nW = mask_period(a);
    long long most = (long long)cu_count() * rowpersist_per_cu<NB, false>() / ((long long)a.heads * parts);
    long long G = most / nW * nW;
    if (G > a.N / 2) G = (a.N / 2) / nW * nW;
    pw = false;
    if (G >= nW && G > 0) return G;
    // no multiple of the mask period fits: with the mask as labels the workgroups walk the windows
    // all the same and form the mask of each window from its labels
    if (a.labels == nullptr) return 0;
    pw = true;
    most = (long long)cu_count() * rowpersist_per_cu<NB, true>() / ((long long)a.heads * parts);
    G = most < a.N / 2 ? most : a.N / 2;
    return G > 0 ? G : 0;
}

template <int NB, int HPB, bool PW>
hipError_t launch_rowpersist_pw(const FwdArgs& a, long long G, hipStream_t st) {
    RowPersistGeom gm;
    gm.groups = (uint32_t)(a.heads / HPB);
    gm.parts = NB <= 12 ? 1u : 2u;
    gm.G = (uint32_t)G;
    const unsigned grid = gm.G * gm.groups * gm.parts, block = 64u * (unsigned)(HPB * rowpersist_waves(NB));
    gm.xcd_q = grid / 8u;
    gm.xcd_r = grid % 8u;
    const size_t lds = rowpersist_lds<NB, HPB>();
    {
        const hipError_t e = allow_lds(reinterpret_cast<const void*>(&fwd_bf16_rowpersist_kernel<NB, HPB, PW>), lds);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL((fwd_bf16_rowpersist_kernel<NB, HPB, PW>), dim3(grid), dim3(block), lds, st, a, gm);
    return hipGetLastError();
}

// pw: the mask comes as labels whose period does not divide G (see the kernel)
template <int NB, int HPB>
hipError_t launch_rowpersist_hpb(const FwdArgs& a, long long G, hipStream_t st, bool pw = false) {
    return pw ? launch_rowpersist_pw<NB, HPB, true>(a, G, st) : launch_rowpersist_pw<NB, HPB, false>(a, G, st);
}

template <int NB, bool BM, int QW>
hipError_t launch_rowblock_qw(const FwdArgs& a, const RowBlockGeom& gm, unsigned grid, int hpb, size_t lds, hipStream_t st) {
    const unsigned block = 64u * (unsigned)(QW * hpb);
    {
        const hipError_t e = allow_lds(reinterpret_cast<const void*>(&fwd_bf16_rowblock_kernel<NB, BM, QW>), lds);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL((fwd_bf16_rowblock_kernel<NB, BM, QW>), dim3(grid), dim3(block), lds, st, a, gm);
    return hipGetLastError();
}

template <int NB>
hipError_t launch_rowblock_nb(const FwdArgs& a, hipStream_t st) {
    RowBlockGeom gm;
    const int hpb = a.heads % 2 == 0 ? 2 : 1;
    const uint32_t groups = (uint32_t)(a.heads / hpb);
    gm.groups = make_fastdiv(groups);
    gm.lanes_per_row = make_fastdiv(4u * (uint32_t)hpb);
    gm.heads_per_block = (uint32_t)hpb;
    const unsigned grid = (unsigned)(a.N * groups);
    gm.xcd_remap = (hpb == 1 && groups > 1) ? 1u : 0u;  // 64 B slabs: keep line-sharing heads on one L2
    gm.xcd_q = grid / 8u;
    gm.xcd_r = grid % 8u;
    const size_t lds = (size_t)2 * 16 * NB * (4 * hpb + 1) * 16;
    const bool bm = a.bias || has_mask(a);
    if (bm) {  // without an additive term the walk over windows gains nothing (measured slower)
        bool pw;
        const long long G = rowpersist_slots<NB>(a, pw);
        if (G > 0) return launch_rowpersist_hpb<NB, 1>(a, G, st, pw);
    }
    // waves per head: 2 with two heads per workgroup (3 or 4 measured 3-20 % slower at L = 144..256), 4
    // with one (an odd head count: 10 % faster than 2; not with an additive term, whose registers
    // need the whole file of a SIMD that holds one wave of the workgroup)
    if (bm) return launch_rowblock_qw<NB, true, 2>(a, gm, grid, hpb, lds, st);
    if (hpb == 1) return launch_rowblock_qw<NB, false, 4>(a, gm, grid, hpb, lds, st);
    return launch_rowblock_qw<NB, false, 2>(a, gm, grid, hpb, lds, st);
}

template <int NB>
hipError_t launch_staged_nb(const FwdArgs& a, int hpb, hipStream_t st) {
    StagedGeom gm;
    const uint32_t groups = (uint32_t)(a.heads / hpb);
    gm.groups = make_fastdiv(groups);
    gm.lanes_per_row = make_fastdiv(4u * (uint32_t)hpb);
    gm.heads_per_block = (uint32_t)hpb;
    const unsigned grid = (unsigned)(a.N * groups), block = 64u * (unsigned)hpb;
    const size_t lds = (size_t)3 * 16 * NB * (4 * hpb + 1) * 16;
    // Fewer window-heads than the chip holds waves (4 per SIMD): one wave per query block instead of
    // one per head, so that the call is not one long round of under-occupied CUs.
    const bool few_tiles = NB > 1 && a.N * a.heads <= 16LL * cu_count();
    // Without bias and mask: four waves per head while they all fit the chip at once (32 waves per CU),
    // else two, since a second round of workgroups costs such a call more than the longer life of a
    // wave (9 % at Swin-T stage 4).  With an additive term two waves per head need 113 VGPRs, which
    // allows no more workgroups per CU than four do, and are 5 % slower.
    const bool two_waves = NB > 2 && a.N * a.heads > 8LL * cu_count();
    if (a.bias || has_mask(a)) {
        // Persistent walk over G window positions: a multiple of nW so that a workgroup always
        // sees the same mask tile, about 4 workgroups per CU (measured best of 2..8), at least 2
        // windows per workgroup, and enough workgroups to cover the chip; else one window each.
        const long long nW = mask_period(a);
        // A small call with an additive term whose workgroups of four waves per head would not all be
        // resident at once (Swin-T stage 4: 24 heads x 128 windows): groups of 3 (or 2) heads in the
        // row-persistent kernel instead, one workgroup per CU walking a few windows with the term in
        // registers (13.1 against 14.2 us there, 16.5 against 17.0 us with 32 heads).
        if (few_tiles && two_waves && a.heads > 4 && (a.heads % 3 == 0 || a.heads % 2 == 0)) {
            const int k = a.heads % 3 == 0 ? 3 : 2;
            const long long grp = a.heads / k;
            long long G1 = (cu_count() / grp) / nW * nW;
            if (G1 > a.N / 2) G1 = (a.N / 2) / nW * nW;
            if (G1 >= nW && G1 > 0 && G1 * grp >= cu_count() / 2)
                return k == 3 ? launch_rowpersist_hpb<NB, 3>(a, G1, st, false) : launch_rowpersist_hpb<NB, 2>(a, G1, st, false);
        }
        // All heads of a window in one workgroup (2..4 heads): one wave per head and query block, one
        // workgroup per CU, two windows in flight per workgroup (measured 3 % faster on Swin-T stage 1
        // than one wave per head, and slower than it with more than one workgroup per CU).  Not for 4
        // heads beyond the small calls: there two 4-wave workgroups per CU of the kernel below are
        // 5-8 % faster than one of 16 waves (82.6 against 86.8 us at 8192 windows, 43.2 against 46.8 at 4096).
        if (groups == 1 && hpb > 1 && (hpb < 4 || few_tiles)) {
            const long long cus = cu_count();
            long long G1 = cus / nW * nW;
            if (G1 > a.N / 2) G1 = (a.N / 2) / nW * nW;
            bool pw = false;
            if (!(G1 >= nW && G1 >= cus / 2) && a.labels != nullptr && a.N >= cus) {
                // no multiple of the mask period fits: per-window masks from the labels
                G1 = a.N / 2 < cus ? a.N / 2 : cus;
                pw = true;
            }
            if (pw || (G1 >= nW && G1 >= cus / 2)) {
                switch (hpb) {
                    case 2: return launch_rowpersist_hpb<NB, 2>(a, G1, st, pw);
                    case 3: return launch_rowpersist_hpb<NB, 3>(a, G1, st, pw);
                    default: return launch_rowpersist_hpb<NB, 4>(a, G1, st, pw);
                }
            }
        }
        // as many workgroups as stay resident: the registers of the kernel allow 8 / 12 / 20 / 32 waves per
        // CU at NB = 4 / 3 / 2 / 1 (a second round of workgroups would double the time of a small call)
        const long long waves_per_cu = NB == 4 ? 8 : (NB == 3 ? 12 : (NB == 2 ? 20 : 32));
        long long per_cu = waves_per_cu / hpb;
        if (per_cu > 4) per_cu = 4;
        const long long most = per_cu * cu_count() / (long long)groups;
        long long G = most / nW * nW;
        if (G > a.N / 2) G = (a.N / 2) / nW * nW;
        if (!few_tiles && G >= nW && G > 0 && G * groups >= cu_count()) {
            hipLaunchKernelGGL((fwd_bf16_persistent_kernel<NB, false>), dim3((unsigned)(G * groups)), dim3(block), lds, st,
                               a, gm, (uint32_t)G);
            return hipGetLastError();
        }
        // no multiple of the mask period fits: with the mask as labels, per-window masks from the labels
        G = most < a.N / 2 ? most : a.N / 2;
        if (!few_tiles && a.labels != nullptr && G * groups >= cu_count()) {
            hipLaunchKernelGGL((fwd_bf16_persistent_kernel<NB, true>), dim3((unsigned)(G * groups)), dim3(block),
                               lds + (size_t)16 * NB * 4, st, a, gm, (uint32_t)G);
            return hipGetLastError();
        }
        if (few_tiles)
            hipLaunchKernelGGL((fwd_bf16_staged_kernel<NB, true, 4>), dim3(grid), dim3(4 * block), lds, st, a, gm);
        else
            hipLaunchKernelGGL((fwd_bf16_staged_kernel<NB, true, 1>), dim3(grid), dim3(block), lds, st, a, gm);
    } else if (few_tiles && two_waves) {
        hipLaunchKernelGGL((fwd_bf16_staged_kernel<NB, false, 2>), dim3(grid), dim3(2 * block), lds, st, a, gm);
    } else if (few_tiles) {
        hipLaunchKernelGGL((fwd_bf16_staged_kernel<NB, false, 4>), dim3(grid), dim3(4 * block), lds, st, a, gm);
    } else {
        hipLaunchKernelGGL((fwd_bf16_staged_kernel<NB, false, 1>), dim3(grid), dim3(block), lds, st, a, gm);
    }
    return hipGetLastError();
}

}  // namespace

// Heads per workgroup for the staged kernel, or 0 when it does not apply: the
// slab of a workgroup must consist of whole 128-byte lines per row (an even
// number of heads) or be the whole row.
int staged_heads_per_block(int L, int heads) {
    if (L > 64) return heads % 2 == 0 ? 2 : 1;
    if (heads <= kWavesPerBlock) return heads;
    if (heads % 4 == 0) return 4;
    if (heads % 2 == 0) return 2;
    return 0;
}

hipError_t launch_forward_bf16_staged(const FwdArgs& a, hipStream_t s) {
    const int hpb = staged_heads_per_block(a.L, a.heads);
    switch ((a.L + 15) / 16) {
        case 1: return launch_staged_nb<1>(a, hpb, s);
        case 2: return launch_staged_nb<2>(a, hpb, s);
        case 3: return launch_staged_nb<3>(a, hpb, s);
        case 4: return launch_staged_nb<4>(a, hpb, s);
        case 5: return launch_rowblock_nb<5>(a, s);
        case 6: return launch_rowblock_nb<6>(a, s);
        case 7: return launch_rowblock_nb<7>(a, s);
        case 8: return launch_rowblock_nb<8>(a, s);
        case 9: return launch_rowblock_nb<9>(a, s);
        case 10: return launch_rowblock_nb<10>(a, s);
        case 11: return launch_rowblock_nb<11>(a, s);
        case 12: return launch_rowblock_nb<12>(a, s);
        case 13: return launch_rowblock_nb<13>(a, s);
        case 14: return launch_rowblock_nb<14>(a, s);
        case 15: return launch_rowblock_nb<15>(a, s);
        case 16: return launch_rowblock_nb<16>(a, s);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace fwa
