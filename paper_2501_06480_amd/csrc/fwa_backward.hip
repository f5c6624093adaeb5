// Backward kernels (paper Algorithm 2): dQ, dK, dV (and dBias) from Q, K, V, dO.
//
// The paper's kernel recomputes P on chip, forms dV and dP chunk by chunk,
// then dS, then re-reads Q and K for dQ and dK.  With a head width of 32 the
// whole (window, head) problem fits in one wave's registers, so Q, K, V, dO
// are read from HBM once (the second pass over Q and K of the paper's loop
// is served on chip) and P, dP, dS never leave the registers.
//
// One wave owns one (window, head) tile and walks windows of its head.  Per
// block of 16 queries ("query on the lane": lane (g, n) holds row
// i = 16 qb + n and columns j = 16 jb + 4g + r, the forward's layout):
//
//   S^T  = K Q^T   -> scores, softmax (row max / sum over the 4 lanes sharing n), P
//   dP^T = V dO^T  -> delta_i = sum_j P_ij dP_ij,  dS = P (dP - delta)
//   dQ^T = K^T dS^T: contraction over keys, dS is already a B operand
//   dBias += dS    (fp32, before any rounding)
//
// dV = P^T dO and dK = dS^T Q contract over the queries and need P and dS with
// the key on the lane instead.  A 16x16 block is moved to that layout by the
// matrix core itself: used as the A operand against an identity B operand it
// comes back as D[4g + r][n] = X[i0 + 4g + r][j0 + n], which is exactly the B
// operand (k-slots = queries) of the products above.  The same trick with a 0/1
// matrix that picks the even (odd) channels turns the row operands of K, Q, dO
// into the A operands K^T, Q^T, dO^T, so every tensor is loaded once, as rows,
// with 16-byte loads.  No LDS tiles, no barriers.
//
// Precision: P and dS enter the matrix cores as bf16.  To keep the results
// within half a bf16 ulp of the exact value they are split into a high and a
// low bf16 part (x = hi + lo to 16 bits) and every product that consumes them
// is issued twice; both parts pass the identity product unchanged.
//
// dBias: each wave adds the dS of its windows into a private LDS array, writes
// it to its slot of the workspace at the end, and a second kernel adds the
// slots in a fixed order, so the result is bit-reproducible.
#include "fwa_device.h"
#include "fwa_internal.h"
#include "fwa_softmax.h"

namespace fwa {
namespace {

struct BwdGeom {
    FastDiv groups;  // workgroups per window position
    uint32_t heads_per_block;
    uint32_t slots;  // workgroups along the window axis; window w is handled by slot w % slots
};

// The row operands of the next window are fetched while the current one is computed: the
// loads write straight into a per-wave LDS stage (one 16-byte slot per lane and 16-row
// block, i.e. already in operand order) and are picked up at the top of the next iteration.
typedef const __attribute__((address_space(1))) void* global_cptr;
typedef __attribute__((address_space(3))) void* lds_vptr;

template <int NB, bool BM, bool DB, bool PF>
__global__ void __launch_bounds__(64 * kWavesPerBlock, 2) bwd_bf16_kernel(BwdArgs p, BwdGeom gm) {
    extern __shared__ __attribute__((aligned(16))) float lds_all[];
    const int lane = threadIdx.x & 63;
    const int n = lane & 15, g = lane >> 4;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t slot = fastdiv(blockIdx.x, gm.groups);
    const uint32_t hg = blockIdx.x - slot * gm.groups.d;
    const uint32_t h = hg * gm.heads_per_block + wave;
    if (h >= (uint32_t)p.heads) return;  // wave-uniform; the kernel has no barriers

    // dBias accumulator of this wave: the 4 values of block (qb, jb) of lane l form one
    // float4 at index (qb*NB + jb)*64 + l, so every lane only ever touches its own
    // addresses (plain read-modify-write, no atomics, no barriers, no bank conflicts).
    constexpr int kAccVecs = DB ? NB * NB * 64 : 0, kStageVecs = PF ? 4 * NB * 64 : 0;
    f32x4* const wave_lds = reinterpret_cast<f32x4*>(lds_all) + (size_t)wave * (kAccVecs + kStageVecs);
    f32x4* const dbacc = wave_lds + lane;
    u32x4* const stage = reinterpret_cast<u32x4*>(wave_lds + kAccVecs);  // [tensor][block][lane]
    if (DB) {
#pragma unroll
        for (int e = 0; e < NB * NB; ++e) dbacc[e * 64] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    const int L = p.L;
    // token rows are p.ldq (q, k, v), p.ldg (d_o), p.ldd (dq, dk, dv) elements apart; window w starts at row w L
    const uint32_t row_bytes = (uint32_t)p.ldq * 2u, row_g = (uint32_t)p.ldg * 2u, row_d = (uint32_t)p.ldd * 2u;
    const uint32_t tile_bytes = (uint32_t)(L - 1) * row_bytes + 2u * kHeadDim;
    const uint32_t tile_bytes_g = (uint32_t)(L - 1) * row_g + 2u * kHeadDim;
    const uint32_t tile_bytes_d = (uint32_t)(L - 1) * row_d + 2u * kHeadDim;
    const uint32_t off_row = (uint32_t)n * row_bytes + 16u * g;  // 16 B of row n (plus a block offset)
    const uint32_t off_row_g = (uint32_t)n * row_g + 16u * g, off_row_d = (uint32_t)n * row_d + 16u * g;
    const float sl2 = p.scale * kLog2e;
    BiasSrc rb = no_bias();
    if (BM) rb = bias_of_head(p, h);

    // identity B operand: slot e of lane (g, n) is 1.0 iff 4g + e == n
    uint2 idu;
    idu.x = (4 * g + 0 == n ? 0x3f80u : 0u) | (4 * g + 1 == n ? 0x3f800000u : 0u);
    idu.y = (4 * g + 2 == n ? 0x3f80u : 0u) | (4 * g + 3 == n ? 0x3f800000u : 0u);
    const bf16x4 ident = as_bf16x4(idu);
    const bf16x8 sel_even = channel_selector(g, n, 0), sel_odd = channel_selector(g, n, 1);
    const f32x4 zero = {0.f, 0.f, 0.f, 0.f};

    // Fetch the rows of window `wn` into the stage.  Rows beyond L are skipped: their slots
    // keep the zeros written once below.
    auto stage_rows = [&](long long wn) {
        const size_t t = ((size_t)wn * L * p.ldq + (size_t)h * kHeadDim) * 2u + off_row;
        const size_t tg = ((size_t)wn * L * p.ldg + (size_t)h * kHeadDim) * 2u + off_row_g;
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            if (16 * b + n < L) {
                const size_t o = t + (size_t)(16 * b) * row_bytes;
                const size_t og = tg + (size_t)(16 * b) * row_g;
                __builtin_amdgcn_global_load_lds((global_cptr)((const char*)p.k + o), (lds_vptr)(stage + (0 * NB + b) * 64), 16, 0, 0);
                __builtin_amdgcn_global_load_lds((global_cptr)((const char*)p.q + o), (lds_vptr)(stage + (1 * NB + b) * 64), 16, 0, 0);
                __builtin_amdgcn_global_load_lds((global_cptr)((const char*)p.v + o), (lds_vptr)(stage + (2 * NB + b) * 64), 16, 0, 0);
                __builtin_amdgcn_global_load_lds((global_cptr)((const char*)p.d_o + og), (lds_vptr)(stage + (3 * NB + b) * 64), 16, 0, 0);
            }
        }
    };
    if (PF) {
        const u32x4 z = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int e = 0; e < 4 * NB; ++e) stage[e * 64 + lane] = z;
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        if (slot < p.N) stage_rows(slot);
    }

    for (long long w = slot; w < p.N; w += gm.slots) {
        const size_t tile = ((size_t)w * L * p.ldq + (size_t)h * kHeadDim) * 2u;
        const size_t tile_g = ((size_t)w * L * p.ldg + (size_t)h * kHeadDim) * 2u;
        const size_t tile_d = ((size_t)w * L * p.ldd + (size_t)h * kHeadDim) * 2u;
        const __amdgpu_buffer_rsrc_t rq = make_rsrc((const char*)p.q + tile, tile_bytes);
        const __amdgpu_buffer_rsrc_t rk = make_rsrc((const char*)p.k + tile, tile_bytes);
        const __amdgpu_buffer_rsrc_t rv = make_rsrc((const char*)p.v + tile, tile_bytes);
        const __amdgpu_buffer_rsrc_t rg = make_rsrc((const char*)p.d_o + tile_g, tile_bytes_g);
        const __amdgpu_buffer_rsrc_t rdq = make_rsrc((char*)p.dq + tile_d, tile_bytes_d);
        const __amdgpu_buffer_rsrc_t rdk = make_rsrc((char*)p.dk + tile_d, tile_bytes_d);
        const __amdgpu_buffer_rsrc_t rdv = make_rsrc((char*)p.dv + tile_d, tile_bytes_d);
        MaskSrc msk = {make_rsrc(nullptr, 0), 0.f, false};
        if (BM) msk = mask_of_window(p, (uint32_t)w);

        // Row operands (contraction over the 32 channels): lane (g, n) = X[16 b + n][8g .. 8g+7]
        bf16x8 krow[NB], vrow[NB], qrow[NB], grow[NB];
        if (PF) {
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the staged loads of this window have landed
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                krow[b] = as_bf16x8(stage[(0 * NB + b) * 64 + lane]);
                qrow[b] = as_bf16x8(stage[(1 * NB + b) * 64 + lane]);
                vrow[b] = as_bf16x8(stage[(2 * NB + b) * 64 + lane]);
                grow[b] = as_bf16x8(stage[(3 * NB + b) * 64 + lane]);
            }
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // stage consumed: it may be refilled
            if (w + gm.slots < p.N) stage_rows(w + gm.slots);
        } else {
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                krow[b] = as_bf16x8(__builtin_amdgcn_raw_buffer_load_b128(rk, off_row + 16 * b * row_bytes, 0, 0));
                qrow[b] = as_bf16x8(__builtin_amdgcn_raw_buffer_load_b128(rq, off_row + 16 * b * row_bytes, 0, 0));
            }
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                vrow[b] = as_bf16x8(__builtin_amdgcn_raw_buffer_load_b128(rv, off_row + 16 * b * row_bytes, 0, 0));
                grow[b] = as_bf16x8(__builtin_amdgcn_raw_buffer_load_b128(rg, off_row_g + 16 * b * row_g, 0, 0));
            }
        }
        // Column operands (contraction over the 16 rows of a block): lane (g, m) =
        // X[16 b + 4g + e][channel 2m resp. 2m+1], e = 0..3.  They are the row operands
        // seen through the matrix core: rows times a 0/1 matrix that picks the even (odd)
        // channels returns exactly these values in the accumulator layout.
        bf16x4 kcol[NB][2];
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            kcol[b][0] = pack_exact(mfma_bf16(krow[b], sel_even, zero));
            kcol[b][1] = pack_exact(mfma_bf16(krow[b], sel_odd, zero));
        }

        f32x4 ve[NB], vo[NB], ke[NB], ko[NB];  // dV, dK of key block jb: [16 jb + n][2 (4g + r) (+1)]
#pragma unroll
        for (int jb = 0; jb < NB; ++jb) ve[jb] = vo[jb] = ke[jb] = ko[jb] = zero;

#pragma unroll
        for (int qb = 0; qb < NB; ++qb) {
            const bf16x4 gcol0 = pack_exact(mfma_bf16(grow[qb], sel_even, zero));
            const bf16x4 gcol1 = pack_exact(mfma_bf16(grow[qb], sel_odd, zero));
            const bf16x4 qcol0 = pack_exact(mfma_bf16(qrow[qb], sel_even, zero));
            const bf16x4 qcol1 = pack_exact(mfma_bf16(qrow[qb], sel_odd, zero));
            f32x4 s[NB], dp[NB];
#pragma unroll
            for (int jb = 0; jb < NB; ++jb) {
                s[jb] = mfma_bf16(krow[jb], qrow[qb], zero);   // S[16 qb + n][16 jb + 4g + r]
                dp[jb] = mfma_bf16(vrow[jb], grow[qb], zero);  // dP at the same positions
            }
            if (BM) {
                // 4 consecutive columns of one row: dword-aligned 16-byte loads, range-checked per dword
                f32x4 add[NB];
                addend_at(rb, msk, (uint32_t)(16 * qb + n), 4u * g, (uint32_t)L).template fill<NB, false>(add, kLog2e);  // fp32 bias only: this kernel has no register to spare
#pragma unroll
                for (int jb = 0; jb < NB; ++jb)
#pragma unroll
                    for (int r = 0; r < 4; ++r) s[jb][r] = fmaf(s[jb][r], sl2, add[jb][r]);
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
            for (int jb = 0; jb < NB; ++jb)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    s[jb][r] *= inv;  // P
                    delta = fmaf(s[jb][r], dp[jb][r], delta);
                }
            delta = sum_over_g(delta);
#pragma unroll
            for (int jb = 0; jb < NB; ++jb)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    dp[jb][r] = s[jb][r] * (dp[jb][r] - delta);  // dS
                }
            if (DB) {
                // keep the read-modify-write of this block together: hoisting the LDS reads of
                // later blocks up here would hold their registers for the whole tile
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int jb = 0; jb < NB; ++jb) dbacc[(qb * NB + jb) * 64] += dp[jb];
                __builtin_amdgcn_sched_barrier(0);
            }

            f32x4 qe = zero, qo = zero;  // dQ[16 qb + n][2 (4g + r) (+1)]
#pragma unroll
            for (int jb = 0; jb < NB; ++jb) {
                bf16x4 p_hi, p_lo, ds_hi, ds_lo;
                split_hi_lo(s[jb], p_hi, p_lo);
                split_hi_lo(dp[jb], ds_hi, ds_lo);
                qe = mfma16(kcol[jb][0], ds_hi, qe);
                qo = mfma16(kcol[jb][1], ds_hi, qo);
                // the block with the key on the lane: t[r] = X[16 qb + 4g + r][16 jb + n]
                const f32x4 t0 = mfma16(p_hi, ident, zero);
                const f32x4 t1 = mfma16(p_lo, ident, zero);
                const f32x4 t2 = mfma16(ds_hi, ident, zero);
                const f32x4 t3 = mfma16(ds_lo, ident, zero);
                qe = mfma16(kcol[jb][0], ds_lo, qe);
                qo = mfma16(kcol[jb][1], ds_lo, qo);
                const bf16x4 tp_hi = pack_exact(t0), tp_lo = pack_exact(t1);
                const bf16x4 ts_hi = pack_exact(t2), ts_lo = pack_exact(t3);
                ve[jb] = mfma16(gcol0, tp_hi, ve[jb]);
                vo[jb] = mfma16(gcol1, tp_hi, vo[jb]);
                ke[jb] = mfma16(qcol0, ts_hi, ke[jb]);
                ko[jb] = mfma16(qcol1, ts_hi, ko[jb]);
                ve[jb] = mfma16(gcol0, tp_lo, ve[jb]);
                vo[jb] = mfma16(gcol1, tp_lo, vo[jb]);
                ke[jb] = mfma16(qcol0, ts_lo, ke[jb]);
                ko[jb] = mfma16(qcol1, ts_lo, ko[jb]);
            }
            u32x4 out;
            out.x = pack_bf16(qe[0] * p.scale, qo[0] * p.scale);
            out.y = pack_bf16(qe[1] * p.scale, qo[1] * p.scale);
            out.z = pack_bf16(qe[2] * p.scale, qo[2] * p.scale);
            out.w = pack_bf16(qe[3] * p.scale, qo[3] * p.scale);
            __builtin_amdgcn_raw_buffer_store_b128(out, rdq, off_row_d + 16 * qb * row_d, 0, 0);
        }
#pragma unroll
        for (int jb = 0; jb < NB; ++jb) {
            u32x4 ov, ok;
            ov.x = pack_bf16(ve[jb][0], vo[jb][0]);
            ov.y = pack_bf16(ve[jb][1], vo[jb][1]);
            ov.z = pack_bf16(ve[jb][2], vo[jb][2]);
            ov.w = pack_bf16(ve[jb][3], vo[jb][3]);
            ok.x = pack_bf16(ke[jb][0] * p.scale, ko[jb][0] * p.scale);
            ok.y = pack_bf16(ke[jb][1] * p.scale, ko[jb][1] * p.scale);
            ok.z = pack_bf16(ke[jb][2] * p.scale, ko[jb][2] * p.scale);
            ok.w = pack_bf16(ke[jb][3] * p.scale, ko[jb][3] * p.scale);
            __builtin_amdgcn_raw_buffer_store_b128(ov, rdv, off_row_d + 16 * jb * row_d, 0, 0);
            __builtin_amdgcn_raw_buffer_store_b128(ok, rdk, off_row_d + 16 * jb * row_d, 0, 0);
        }
    }

    if (DB) {
        // partial sums in register order: [slot][head][qb][jb][lane] float4 -- contiguous 16-byte stores
        f32x4* dst = reinterpret_cast<f32x4*>(p.partial) + ((size_t)slot * p.heads + h) * (NB * NB * 64) + lane;
#pragma unroll
        for (int qb = 0; qb < NB; ++qb)
#pragma unroll
            for (int jb = 0; jb < NB; ++jb) dst[(qb * NB + jb) * 64] = dbacc[(qb * NB + jb) * 64];
    }
}

// dbias[h][i][j] = sum over slots of the partial sums, which the backward kernels leave in
// register order: per slot and head, block (qb, jb) holds 64 float4, the one of lane (g, n)
// carrying elements (i, j) = (16 qb + n, 16 jb + 4 g + r), r = 0..3.  A workgroup of 16 x 16
// threads owns 16 consecutive float4 of that array; thread row y adds slots y, y+16, ... in
// index order (contiguous 256-byte reads), then the 16 row sums are added in row order: a
// fixed summation tree, hence bit-reproducible.
constexpr int kReduceRows = 16;
__global__ void __launch_bounds__(16 * kReduceRows)
dbias_reduce_kernel(const f32x4* __restrict__ partial, float* __restrict__ dbias, int slots, int heads, int L,
                    int key_on_lane) {
    __shared__ f32x4 part[kReduceRows][16];
    const int x = threadIdx.x & 15, y = threadIdx.x >> 4;
    const int nb = (L + 15) / 16;
    const size_t padded = (size_t)heads * nb * nb * 64;  // float4 per slot
    const size_t f = (size_t)blockIdx.x * 16 + x;        // < padded: the grid is padded / 16
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    // 8 loads in flight per thread (one at a time leaves the kernel waiting on L2 latency); the
    // additions keep the index order
    for (int s = y; s < slots; s += 8 * kReduceRows) {
        f32x4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int su = s + u * kReduceRows;
            v[u] = su < slots ? partial[(size_t)su * padded + f] : f32x4{0.f, 0.f, 0.f, 0.f};
        }
#pragma unroll
        for (int u = 0; u < 8; ++u)
            if (s + u * kReduceRows < slots) acc += v[u];
    }
    part[y][x] = acc;
    __syncthreads();
    if (y == 0) {
        f32x4 total = part[0][x];
#pragma unroll
        for (int r = 1; r < kReduceRows; ++r) total += part[r][x];
        const int lane = (int)(f & 63), blk = (int)(f >> 6);
        const int b1 = blk % nb, b0 = (blk / nb) % nb, h = blk / (nb * nb);
        if (!key_on_lane) {
            // blocks [qb][jb]; lane (g, n) holds query 16 qb + n, keys 16 jb + 4g + r
            const int i = 16 * b0 + (lane & 15), j = 16 * b1 + 4 * (lane >> 4);
            if (i < L) {
                float* row = dbias + ((size_t)h * L + i) * L;
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    if (j + r < L) row[j + r] = total[r];
            }
        } else {
            // blocks [jb][qb]; lane (g, n) holds key 16 jb + n, queries 16 qb + 4g + r
            const int j = 16 * b0 + (lane & 15), i = 16 * b1 + 4 * (lane >> 4);
            if (j < L) {
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    if (i + r < L) dbias[((size_t)h * L + i + r) * L + j] = total[r];
            }
        }
    }
}

template <int NB, bool BM, bool DB>
hipError_t launch_one(const BwdArgs& a, const BwdGeom& gm, unsigned grid, unsigned block, hipStream_t st) {
    // Prefetching through the LDS stage pays only when nothing else competes for LDS (the dBias
    // accumulator) or for the in-order load queue (bias/mask loads): measured 195 vs 249 us on the
    // Swin-T stage-1 shape without bias, no gain with bias, a loss with dBias.
    const bool pf = !BM && !DB;
    const size_t per_wave = (DB ? (size_t)NB * NB * 64 * 16 : 0) + (pf ? (size_t)4 * NB * 64 * 16 : 0);
    const size_t lds = (size_t)(block / 64) * per_wave;
    const void* fn = pf ? reinterpret_cast<const void*>(&bwd_bf16_kernel<NB, BM, DB, true>)
                        : reinterpret_cast<const void*>(&bwd_bf16_kernel<NB, BM, DB, false>);
    {
        const hipError_t e = allow_lds(fn, lds);
        if (e != hipSuccess) return e;
    }
    if (pf)
        hipLaunchKernelGGL((bwd_bf16_kernel<NB, BM, DB, true>), dim3(grid), dim3(block), lds, st, a, gm);
    else
        hipLaunchKernelGGL((bwd_bf16_kernel<NB, BM, DB, false>), dim3(grid), dim3(block), lds, st, a, gm);
    return hipGetLastError();
}

template <int NB>
hipError_t launch_bwd_nb(const BwdArgs& a, hipStream_t st) {
    BwdGeom gm;
    int hpb = kWavesPerBlock;
    if (a.heads < hpb) hpb = a.heads;
    const uint32_t groups = (uint32_t)((a.heads + hpb - 1) / hpb);
    gm.groups = make_fastdiv(groups);
    gm.heads_per_block = (uint32_t)hpb;
    gm.slots = (uint32_t)a.slots;
    const unsigned grid = gm.slots * groups, block = 64u * (unsigned)hpb;
    const bool bm = a.bias || has_mask(a), db = a.dbias != nullptr;
    hipError_t e;
    if (bm)
        e = db ? launch_one<NB, true, true>(a, gm, grid, block, st) : launch_one<NB, true, false>(a, gm, grid, block, st);
    else
        e = db ? launch_one<NB, false, true>(a, gm, grid, block, st) : launch_one<NB, false, false>(a, gm, grid, block, st);
    return e;
}

}  // namespace

// Workgroups along the window axis (= dBias slots).  The cooperative kernel is used whenever
// its workgroup shape fits the head count and the mask period; the single-wave kernel
// otherwise, with enough slots to fill the chip (two waves per SIMD).
static int single_slots(long long N, int heads) {
    const int hpb = heads < kWavesPerBlock ? heads : kWavesPerBlock;
    const int groups = (heads + hpb - 1) / hpb;
    long long slots = (cu_count() * 8 / hpb + groups - 1) / groups;  // ~8 waves per CU
    if (slots > N) slots = N;
    if (slots < 1) slots = 1;
    return (int)slots;
}

int backward_slots(long long N, int heads, int nW) {
    const int c = coop_slots(N, heads, nW);
    return c > 0 ? c : single_slots(N, heads);
}

int backward_max_slots(long long N, int heads) {
    const int a = coop_slots(N, heads, 1), b = single_slots(N, heads);  // period 1 gives the largest count
    return a > b ? a : b;
}

hipError_t launch_backward_bf16_single(const BwdArgs& a, hipStream_t s) {
    switch ((a.L + 15) / 16) {
        case 1: return launch_bwd_nb<1>(a, s);
        case 2: return launch_bwd_nb<2>(a, s);
        case 3: return launch_bwd_nb<3>(a, s);
        case 4: return launch_bwd_nb<4>(a, s);
        default: return hipErrorNotSupported;
    }
}

// dbias[h][i][j] = sum over the slots of partial[slot][h][i][j]
hipError_t launch_backward_bf16(const BwdArgs& a, hipStream_t s) {
    if (a.C / a.heads != kHeadDim) return launch_backward_bf16_wide(a, s);
    if (a.L > kMaxBackwardL) return launch_backward_bf16_large(a, s);
    const bool coop = a.per_window || coop_slots(a.N, a.heads, mask_period(a)) > 0;
    const hipError_t e = coop ? launch_backward_bf16_coop(a, s) : launch_backward_bf16_single(a, s);
    if (e != hipSuccess || a.dbias == nullptr) return e;
    return launch_dbias_reduce(a, s);
}

// dbias = sum over a.slots slots of the partial sums a backward kernel left in a.partial
hipError_t launch_dbias_reduce(const BwdArgs& a, hipStream_t s, bool key_on_lane) {
    const int nb = (a.L + 15) / 16;
    hipLaunchKernelGGL(dbias_reduce_kernel, dim3((unsigned)(a.heads * nb * nb * 4)), dim3(16 * kReduceRows), 0, s,
                       reinterpret_cast<const f32x4*>(a.partial), a.dbias, a.slots, a.heads, a.L, key_on_lane ? 1 : 0);
    return hipGetLastError();
}


}  // namespace fwa
