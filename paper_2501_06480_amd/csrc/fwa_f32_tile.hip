// fp32 kernels for windows of up to 64 tokens and head widths 32, 64, 128, 256, forward and
// backward (longer windows of width 32 have a forward kernel of their own in fwa_forward.hip).
// True fp32 arithmetic throughout: v_mfma_f32_16x16x4_f32 products, v_exp_f32, IEEE division.
// These are the shapes and the precision of the paper's kernel benchmark (section 3.1).
//
// One workgroup per (window, head), one wave per block of 16 rows.  The fp32 matrix instruction
// takes one value per lane and k-slot group: lane (g, n) gives A[m = n][k = g] and B[k = g][n] and
// receives D[4g + r][n].  A 16-byte LDS or global read of 4 consecutive channels therefore feeds
// 4 successive instructions (k-slot g of step t standing for channel 16 c + 4g + t), which is how
// row operands are read; operands with the contraction index on the rows of a slab (V^T, K^T,
// dO^T, Q^T) are read element by element out of LDS.
//
// Backward: pass 1 with K, V parked gives P, dS and dQ; dV and dK follow from P resp. dS exchanged
// through an LDS tile and the dO resp. Q slab (see the kernel).  dBias is not produced in fp32.
#include "fwa_device.h"
#include "fwa_internal.h"
#include "fwa_softmax.h"

namespace fwa {
namespace {

// slab row stride in floats: D + 4, an odd number of 16-byte units, so that 16-byte reads of 8
// consecutive rows fall into different banks
template <int D>
struct F32Tile {
    static constexpr int RS = D + 4;
    static constexpr int TPR = D / 4;          // threads that move one row (16 bytes each)
    static constexpr int RPP = 256 / TPR;      // rows per pass of the workgroup (TPR <= 64)
    static constexpr int CH = D / 16;          // 16-channel chunks
};

// Rows [0, ROWS) x D floats of a tile on their way into an LDS slab: requested into registers, then
// parked; rows beyond L arrive as zeros.
template <int D, int ROWS>
struct SlabInFlight {
    using T = F32Tile<D>;
    static constexpr int PASSES = (ROWS + T::RPP - 1) / T::RPP;
    f32x4 v[PASSES];
    __device__ __forceinline__ void request(const __amdgpu_buffer_rsrc_t r, uint32_t row_bytes, int tid) {
        const uint32_t srow = (uint32_t)tid / T::TPR, scol = (uint32_t)tid % T::TPR;
#pragma unroll
        for (int t = 0; t < PASSES; ++t) v[t] = load_f32x4(r, (T::RPP * t + srow) * row_bytes + scol * 16u);
    }
    __device__ __forceinline__ void park(float* slab, int tid) const {
        const uint32_t srow = (uint32_t)tid / T::TPR, scol = (uint32_t)tid % T::TPR;
#pragma unroll
        for (int t = 0; t < PASSES; ++t) {
            const uint32_t row = T::RPP * t + srow;
            if (row < (uint32_t)ROWS) *reinterpret_cast<f32x4*>(slab + row * T::RS + 4 * scol) = v[t];
        }
    }
};

template <int D, int ROWS>
__device__ __forceinline__ void park_slab(float* slab, const __amdgpu_buffer_rsrc_t r, uint32_t row_bytes, int tid) {
    SlabInFlight<D, ROWS> x;
    x.request(r, row_bytes, tid);
    x.park(slab, tid);
}

// acc[jb] += X[16 jb + n][:] . own[:] over all channels: X rows from an LDS slab (A operand),
// `own` the 16 rows of this wave (B operand, in registers)
template <int NB, int D>
__device__ __forceinline__ void rows_times_own(f32x4 (&acc)[NB], const float* slab, const f32x4 (&own)[D / 16], int n, int g) {
    using T = F32Tile<D>;
#pragma unroll
    for (int c = 0; c < T::CH; ++c)
#pragma unroll
        for (int jb = 0; jb < NB; ++jb) {
            const f32x4 x = *reinterpret_cast<const f32x4*>(slab + (16 * jb + n) * T::RS + 16 * c + 4 * g);
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const float a = x[t], b = own[c][t];
                acc[jb] = mfma_f32(a, b, acc[jb]);
            }
        }
}

// the 16 rows 16 blk + n of a tile as operands: channels 16 c + 4g .. + 3 per chunk
template <int D>
__device__ __forceinline__ void load_own_rows(f32x4 (&own)[D / 16], const __amdgpu_buffer_rsrc_t r, uint32_t row_bytes,
                                              int blk, int n, int g) {
    const uint32_t off = (uint32_t)(16 * blk + n) * row_bytes + 16u * g;
#pragma unroll
    for (int c = 0; c < D / 16; ++c) own[c] = load_f32x4(r, off + 64 * c);
}

// scores of a block of 16 query rows -> probabilities; returns nothing, leaves P in s and the
// statistics in m (row max of the scaled scores, natural units) and sum
template <int NB, bool BM>
__device__ __forceinline__ void softmax_f32(f32x4 (&s)[NB], float scale, const AddendGlobal& addend, int L, int g,
                                            float& m, float& sum) {
    m = -INFINITY;
    f32x4 add[NB];
    if (BM) addend.fill(add, 1.0f);
#pragma unroll
    for (int jb = 0; jb < NB; ++jb) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            float x = BM ? s[jb][r] * scale + add[jb][r] : s[jb][r] * scale;
            if (jb == NB - 1 && 16 * jb + 4 * g + r >= L) x = -INFINITY;
            s[jb][r] = x;
            m = fmaxf(m, x);
        }
    }
    m = max_over_g(m);
    sum = 0.f;
#pragma unroll
    for (int jb = 0; jb < NB; ++jb)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const float e = __builtin_amdgcn_exp2f((s[jb][r] - m) * kLog2e);
            s[jb][r] = e;
            sum += e;
        }
    sum = sum_over_g(sum);
}

// ------------------------------------------------------------------ forward
template <int NB, int D, bool BM>
__global__ void __launch_bounds__(256) fwd_f32_tile_kernel(FwdArgs p) {
    using T = F32Tile<D>;
    constexpr int ROWS = 16 * NB;
    extern __shared__ __attribute__((aligned(16))) float ldsf[];  // one slab [ROWS][RS]: K, then V
    const int tid = threadIdx.x, lane = tid & 63;
    const int n = lane & 15, g = lane >> 4;
    const int qb = __builtin_amdgcn_readfirstlane(tid >> 6);
    const uint32_t w = blockIdx.x / (uint32_t)p.heads, h = blockIdx.x % (uint32_t)p.heads;
    const int L = p.L;
    const uint32_t row_bytes = (uint32_t)p.ldq * 4u, row_out = (uint32_t)p.ldo * 4u;
    const size_t tile = ((size_t)w * L * p.ldq + (size_t)h * D) * 4u;
    const uint32_t tile_bytes = (uint32_t)(L - 1) * row_bytes + 4u * D;
    const bool active = qb < NB;  // the other waves only move slab rows

    // K and V take turns in one slab: V waits in registers while the scores are made from K.  Half
    // the LDS of two slabs means twice the workgroups per CU, so that one of them computes while
    // another one loads (at width 256 a two-slab workgroup had the CU to itself).
    f32x4 qv[T::CH];
    SlabInFlight<D, ROWS> kin, vin;
    kin.request(make_rsrc((const char*)p.k + tile, tile_bytes), row_bytes, tid);
    load_own_rows<D>(qv, make_rsrc((const char*)p.q + tile, tile_bytes), row_bytes, qb, n, g);
    kin.park(ldsf, tid);
    vin.request(make_rsrc((const char*)p.v + tile, tile_bytes), row_bytes, tid);
    __syncthreads();

    f32x4 s[NB];
    float m = 0.f, sum = 1.f;
    if (active) {
#pragma unroll
        for (int jb = 0; jb < NB; ++jb) s[jb] = f32x4{0.f, 0.f, 0.f, 0.f};
        rows_times_own<NB, D>(s, ldsf, qv, n, g);  // S[16 qb + n][16 jb + 4g + r]
    }
    __syncthreads();  // every wave has read its K rows
    vin.park(ldsf, tid);
    if (active) {
        BiasSrc rb = no_bias();
        MaskSrc msk = {make_rsrc(nullptr, 0), 0.f, false};
        if (BM) {
            rb = bias_of_head(p, h);
            msk = mask_of_window(p, w);
        }
        softmax_f32<NB, BM>(s, p.scale, addend_at(rb, msk, (uint32_t)(16 * qb + n), 4u * g, (uint32_t)L), L, g, m, sum);
    }
    __syncthreads();  // V is in place
    if (!active) return;  // no barrier follows

    // O^T = V^T P^T, 16 channels at a time: k-slot g of step (jb, r) stands for key 16 jb + 4g + r
    const __amdgpu_buffer_rsrc_t ro =
        make_rsrc((char*)p.o + ((size_t)w * L * p.ldo + (size_t)h * D) * 4u, (uint32_t)(L - 1) * row_out + 4u * D);
    const uint32_t off_o = (uint32_t)(16 * qb + n) * row_out + 16u * g;
#pragma unroll
    for (int cb = 0; cb < T::CH; ++cb) {
        f32x4 o = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int jb = 0; jb < NB; ++jb)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float pv = s[jb][r];
                o = mfma_f32(ldsf[(16 * jb + 4 * g + r) * T::RS + 16 * cb + n], pv, o);  // o[r'] = O[16 qb + n][16 cb + 4g + r']
            }
        store_f32x4(o / sum, ro, off_o + 64 * cb);
    }
}

// ----------------------------------------------------------------- backward
// Pass 1 ("query on the lane", K and V parked in the two slabs): S, softmax, dP, delta, dS, dQ.
// P and dS are not made a second time for dV and dK: the fp32 matrix instruction takes single
// values, so any orientation can be read out of a row-major tile.  dV and dK are made one after the
// other, each from one slab and one tile, and the tile lives where a dead slab was (a tile row, 68
// floats, is not longer than a slab row except at width 32, where the slab area is sized by the
// tile): dO -> slab B and P -> tile in slab A, dV; then Q -> slab B and dS -> tile in slab A, dK.
// The waves write those slabs and tiles from the registers of pass 1, so every input is read from
// global memory once, and the matrix cores do 10 L^2 D flops per tile (making S and dP again in
// the second orientation, as the large-window bf16 kernel must, costs 14 and was 15-30 % slower).
constexpr int kTileStrideF32 = 68;  // floats per tile row: rows 4 apart fall 16 banks apart
template <int NB, int D, bool BM>
__global__ void __launch_bounds__(256) bwd_f32_tile_kernel(BwdArgs p) {
    using T = F32Tile<D>;
    constexpr int ROWS = 16 * NB;
    constexpr int TS = kTileStrideF32;
    static_assert(TS <= T::RS || D == 32, "a tile must fit into a slab");
    extern __shared__ __attribute__((aligned(16))) float ldsf[];  // two slabs [ROWS][max(RS, TS)]
    constexpr int SLAB = ROWS * (T::RS > TS ? T::RS : TS);
    const int tid = threadIdx.x, lane = tid & 63;
    const int n = lane & 15, g = lane >> 4;
    const int role = __builtin_amdgcn_readfirstlane(tid >> 6);  // query block in pass 1, key block afterwards
    const bool active = role < NB;
    const uint32_t w = blockIdx.x / (uint32_t)p.heads, h = blockIdx.x % (uint32_t)p.heads;
    const int L = p.L;
    const uint32_t row_bytes = (uint32_t)p.ldq * 4u, row_g = (uint32_t)p.ldg * 4u, row_d = (uint32_t)p.ldd * 4u;
    const size_t tile = ((size_t)w * L * p.ldq + (size_t)h * D) * 4u;
    const size_t tile_g = ((size_t)w * L * p.ldg + (size_t)h * D) * 4u;
    const size_t tile_d = ((size_t)w * L * p.ldd + (size_t)h * D) * 4u;
    const uint32_t tile_bytes = (uint32_t)(L - 1) * row_bytes + 4u * D;
    const uint32_t tile_bytes_g = (uint32_t)(L - 1) * row_g + 4u * D;
    const uint32_t tile_bytes_d = (uint32_t)(L - 1) * row_d + 4u * D;
    const __amdgpu_buffer_rsrc_t rq = make_rsrc((const char*)p.q + tile, tile_bytes);
    const __amdgpu_buffer_rsrc_t rk = make_rsrc((const char*)p.k + tile, tile_bytes);
    const __amdgpu_buffer_rsrc_t rv = make_rsrc((const char*)p.v + tile, tile_bytes);
    const __amdgpu_buffer_rsrc_t rg = make_rsrc((const char*)p.d_o + tile_g, tile_bytes_g);
    float* const sa = ldsf;         // K, then the P tile, then the dS tile
    float* const sb = ldsf + SLAB;  // V, then dO, then Q
    const f32x4 zero = {0.f, 0.f, 0.f, 0.f};

    f32x4 qv[T::CH], gv[T::CH];  // own Q and dO rows (rows beyond L arrive as zeros)
    load_own_rows<D>(qv, rq, row_bytes, role, n, g);
    load_own_rows<D>(gv, rg, row_g, role, n, g);
    park_slab<D, ROWS>(sa, rk, row_bytes, tid);
    park_slab<D, ROWS>(sb, rv, row_bytes, tid);
    __syncthreads();

    // ---------------- pass 1: query block `role` ----------------
    f32x4 s[NB], dp[NB];
    if (active) {
        const int qb = role;
        BiasSrc rb = no_bias();
        MaskSrc msk = {make_rsrc(nullptr, 0), 0.f, false};
        if (BM) {
            rb = bias_of_head(p, h);
            msk = mask_of_window(p, w);
        }
#pragma unroll
        for (int jb = 0; jb < NB; ++jb) s[jb] = dp[jb] = zero;
        rows_times_own<NB, D>(s, sa, qv, n, g);   // <k_j, q_i>: query i = 16 qb + n, key j = 16 jb + 4g + r
        rows_times_own<NB, D>(dp, sb, gv, n, g);  // <v_j, do_i>
        float m, sum;
        softmax_f32<NB, BM>(s, p.scale, addend_at(rb, msk, (uint32_t)(16 * qb + n), 4u * g, (uint32_t)L), L, g, m, sum);
        float delta = 0.f;
#pragma unroll
        for (int jb = 0; jb < NB; ++jb)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                s[jb][r] = s[jb][r] / sum;  // P
                delta = fmaf(s[jb][r], dp[jb][r], delta);
            }
        delta = sum_over_g(delta);
#pragma unroll
        for (int jb = 0; jb < NB; ++jb)
#pragma unroll
            for (int r = 0; r < 4; ++r) dp[jb][r] = s[jb][r] * (dp[jb][r] - delta);  // dS
        // dQ^T = K^T dS^T, 16 channels at a time: k-slot g of step (jb, r) stands for key 16 jb + 4g + r
        const __amdgpu_buffer_rsrc_t rdq = make_rsrc((char*)p.dq + tile_d, tile_bytes_d);
        const uint32_t off_q = (uint32_t)(16 * qb + n) * row_d + 16u * g;
#pragma unroll
        for (int cb = 0; cb < T::CH; ++cb) {
            f32x4 acc = zero;
#pragma unroll
            for (int jb = 0; jb < NB; ++jb)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const float ds = dp[jb][r];
                    acc = mfma_f32(sa[(16 * jb + 4 * g + r) * T::RS + 16 * cb + n], ds, acc);
                }
            store_f32x4(acc * p.scale, rdq, off_q + 64 * cb);  // acc[r'] = dQ[16 qb + n][16 cb + 4g + r']
        }
    }
    const uint32_t off_k = (uint32_t)(16 * role + n) * row_d + 16u * g;
    // out[16 role + n][:] = sum over queries of tile[query][16 role + n] * slab B[query][:], times `mul`
    auto contract_and_store = [&](const __amdgpu_buffer_rsrc_t dst, float mul) {
        f32x4 acc[T::CH];
#pragma unroll
        for (int cb = 0; cb < T::CH; ++cb) acc[cb] = zero;
#pragma unroll
        for (int qb = 0; qb < NB; ++qb) {
            f32x4 t;  // the tile with the query on the slot: t[r] = tile[16 qb + 4g + r][16 role + n]
#pragma unroll
            for (int r = 0; r < 4; ++r) t[r] = sa[(16 * qb + 4 * g + r) * TS + 16 * role + n];
#pragma unroll
            for (int cb = 0; cb < T::CH; ++cb)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const float tv = t[r];
                    acc[cb] = mfma_f32(sb[(16 * qb + 4 * g + r) * T::RS + 16 * cb + n], tv, acc[cb]);
                }
        }
#pragma unroll
        for (int cb = 0; cb < T::CH; ++cb) store_f32x4(acc[cb] * mul, dst, off_k + 64 * cb);
    };
    auto place = [&](const f32x4 (&rows)[T::CH], const f32x4 (&tile_rows)[NB]) {
#pragma unroll
        for (int c = 0; c < T::CH; ++c) *reinterpret_cast<f32x4*>(sb + (16 * role + n) * T::RS + 16 * c + 4 * g) = rows[c];
#pragma unroll
        for (int jb = 0; jb < NB; ++jb) *reinterpret_cast<f32x4*>(sa + (16 * role + n) * TS + 16 * jb + 4 * g) = tile_rows[jb];
    };
    __syncthreads();  // K, V no longer needed
    if (active) place(gv, s);  // dO rows and P rows of this wave's query block
    __syncthreads();
    if (active) contract_and_store(make_rsrc((char*)p.dv + tile_d, tile_bytes_d), 1.0f);  // dV^T = dO^T P
    __syncthreads();  // dO and P no longer needed
    if (active) place(qv, dp);  // Q rows and dS rows
    __syncthreads();
    if (active) contract_and_store(make_rsrc((char*)p.dk + tile_d, tile_bytes_d), p.scale);  // dK^T = Q^T dS
}

template <int NB, int D>
size_t f32_slab_bytes() {
    return (size_t)2 * 16 * NB * (D + 4) * 4;
}

template <int NB, int D>
hipError_t launch_fwd_nb(const FwdArgs& a, hipStream_t st) {
    const unsigned grid = (unsigned)(a.N * a.heads);
    const size_t lds = f32_slab_bytes<NB, D>() / 2;  // K and V take turns in one slab
    const bool bm = a.bias || has_mask(a);
    const void* fn = bm ? reinterpret_cast<const void*>(&fwd_f32_tile_kernel<NB, D, true>)
                        : reinterpret_cast<const void*>(&fwd_f32_tile_kernel<NB, D, false>);
    {
        const hipError_t e = allow_lds(fn, lds);
        if (e != hipSuccess) return e;
    }
    if (bm)
        hipLaunchKernelGGL((fwd_f32_tile_kernel<NB, D, true>), dim3(grid), dim3(256), lds, st, a);
    else
        hipLaunchKernelGGL((fwd_f32_tile_kernel<NB, D, false>), dim3(grid), dim3(256), lds, st, a);
    return hipGetLastError();
}

template <int NB, int D>
hipError_t launch_bwd_nb(const BwdArgs& a, hipStream_t st) {
    const unsigned grid = (unsigned)(a.N * a.heads);
    const bool bm = a.bias || has_mask(a);
    constexpr size_t rs = (D + 4) > kTileStrideF32 ? (D + 4) : kTileStrideF32;  // a slab also holds a tile
    const size_t lds = (size_t)2 * 16 * NB * rs * 4;
    const void* fn = bm ? reinterpret_cast<const void*>(&bwd_f32_tile_kernel<NB, D, true>)
                        : reinterpret_cast<const void*>(&bwd_f32_tile_kernel<NB, D, false>);
    {
        const hipError_t e = allow_lds(fn, lds);
        if (e != hipSuccess) return e;
    }
    if (bm)
        hipLaunchKernelGGL((bwd_f32_tile_kernel<NB, D, true>), dim3(grid), dim3(256), lds, st, a);
    else
        hipLaunchKernelGGL((bwd_f32_tile_kernel<NB, D, false>), dim3(grid), dim3(256), lds, st, a);
    return hipGetLastError();
}

#define FWA_F32_NB_SWITCH(FN, D, a, s)            \
    switch (((a).L + 15) / 16) {                  \
        case 1: return FN<1, D>(a, s);            \
        case 2: return FN<2, D>(a, s);            \
        case 3: return FN<3, D>(a, s);            \
        case 4: return FN<4, D>(a, s);            \
        default: return hipErrorInvalidValue;     \
    }

template <int D>
hipError_t fwd_d(const FwdArgs& a, hipStream_t s) { FWA_F32_NB_SWITCH(launch_fwd_nb, D, a, s) }
template <int D>
hipError_t bwd_d(const BwdArgs& a, hipStream_t s) { FWA_F32_NB_SWITCH(launch_bwd_nb, D, a, s) }

}  // namespace

hipError_t launch_forward_f32_tile(const FwdArgs& a, hipStream_t s) {
    switch (a.C / a.heads) {
        case 32: return fwd_d<32>(a, s);
        case 64: return fwd_d<64>(a, s);
        case 128: return fwd_d<128>(a, s);
        case 256: return fwd_d<256>(a, s);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_backward_f32(const BwdArgs& a, hipStream_t s) {
    if (a.dbias != nullptr || a.L > kMaxWideL) return hipErrorNotSupported;
    switch (a.C / a.heads) {
        case 32: return bwd_d<32>(a, s);
        case 64: return bwd_d<64>(a, s);
        case 128: return bwd_d<128>(a, s);
        case 256: return bwd_d<256>(a, s);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace fwa
