// Backward (paper Algorithm 2) for head widths 64, 128 and 256 at L <= 64: the shapes of the
// paper's forward-backward kernel benchmark (section 3.1).
//
// One workgroup per (window, head), one wave per 16-row block, two phases as in the kernel for
// width 32, with every product over the feature dimension run chunk by chunk (eq. 5-6: D / 32
// k-steps for S and dP) and every D-wide output produced in D / 16 blocks of 16 channels that
// are stored as soon as they are complete, so that no wave ever holds a D-wide accumulator.
//
//   LDS, first half of the tile's life : K, V slabs (row operands of S^T = K Q^T and dP^T = V dO^T,
//                                        K^T for dQ through the transposing read)
//   phase A, wave <-> query block      : own Q, dO rows straight from global memory as operands;
//                                        softmax, delta, dS; dQ; P and dS as hi + lo bf16 into
//                                        swizzled LDS tiles
//   LDS, second half                   : the Q, dO slabs take the place of K, V, written by the
//                                        waves from the operand registers of phase A
//   phase B, wave <-> key block        : dV^T = dO^T P, dK^T = Q^T dS with P, dS (key on the lane)
//                                        and dO^T, Q^T (channel on the lane) through the
//                                        transposing read
//
// Every input is read from global memory once.
//
// A workgroup walks the windows bw, bw + G, ... of its head (G = N, one window each, for widths 64
// and 128 without dBias; one workgroup per CU at width 256); the K, V slabs of the next window are
// requested during phase B of the current one.  dBias rows of a wave's query block are summed in registers across its windows and
// leave as per-workgroup partial sums in register order, like those of the kernel for width 32;
// the same reduce kernel adds the slots.
#include "fwa_device.h"
#include "fwa_internal.h"
#include "fwa_softmax.h"

namespace fwa {
namespace {

// F16: the data are IEEE half instead of bf16.  P and dS then enter the matrix cores as single half
// operands (11 significant bits, against 16 for the hi + lo bf16 pairs: products stay within 3e-4
// relative, far inside the 1e-2 bound), so the lo tiles, their LDS traffic and the second product of
// each pair are absent.  |dS| must stay inside the half range (65504), as everything in half data must.
template <int NB, int D, bool BM, bool DB, bool F16>
__global__ void __launch_bounds__(256) bwd_bf16_wide_kernel(BwdArgs p, uint32_t G) {
    constexpr int NB2 = (NB + 1) / 2;
    constexpr int ROWS = 16 * NB;
    constexpr int CH = D / 32;               // chunks of the products over the feature dimension
    constexpr int CB = D / 16;               // 16-channel blocks of dQ, dK, dV
    constexpr uint32_t STRIDE = D / 8 + 1;   // slab row in 16-byte units: D * 2 bytes of data + 16 of padding
    constexpr uint32_t SROW = STRIDE * 8;    // the same in bf16 elements
    constexpr int TPR = D / 8;               // threads that move one slab row
    constexpr int RPP = 256 / TPR;           // rows per pass of the workgroup
    constexpr int PASSES = (ROWS + RPP - 1) / RPP;
    constexpr uint32_t XS = 64, XT = ROWS * XS;  // P / dS tiles: [ROWS][64] bf16, units swizzled (see below)
    constexpr int NT = F16 ? 2 : 4;              // tiles: P, dS (half) or P_hi, P_lo, dS_hi, dS_lo (bf16)
    extern __shared__ __attribute__((aligned(16))) uint4 lds[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int n = lane & 15, g = lane >> 4;
    const int role = __builtin_amdgcn_readfirstlane(tid >> 6);  // query block in phase A, key block in phase B
    const bool active = role < NB;
    const uint32_t bw = blockIdx.x / (uint32_t)p.heads, h = blockIdx.x % (uint32_t)p.heads;
    const int L = p.L;
    // token rows are p.ldq (q, k, v), p.ldg (d_o), p.ldd (dq, dk, dv) elements apart; window w starts at row w L
    const uint32_t row_bytes = (uint32_t)p.ldq * 2u, row_g = (uint32_t)p.ldg * 2u, row_d = (uint32_t)p.ldd * 2u;
    const uint32_t tile_bytes = (uint32_t)(L - 1) * row_bytes + 2u * D;  // rows beyond L read as zero
    const uint32_t tile_bytes_g = (uint32_t)(L - 1) * row_g + 2u * D;
    const uint32_t tile_bytes_d = (uint32_t)(L - 1) * row_d + 2u * D;
    const float sl2 = p.scale * kLog2e;
    const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

    uint4* const sa = lds;                  // K, then Q
    uint4* const sb = lds + ROWS * STRIDE;  // V, then dO
    // Tiles P_hi, P_lo, dS_hi, dS_lo.  A row is 16 units of 4 keys; unit (block b, quarter c) of
    // row i sits at unit (b ^ (i & 3), c ^ ((i >> 2) & 3)): the 16 lanes of a write (16 rows, one
    // unit each) and of a transposing read (4 rows x 4 units) then touch every bank once.
    uint16_t* const ex = reinterpret_cast<uint16_t*>(lds + 2 * ROWS * STRIDE);
    const uint32_t srow = (uint32_t)tid / TPR, scol = (uint32_t)tid % TPR;  // slab movement: (row, 16 B column)
    const uint32_t opd = (uint32_t)n * STRIDE + g;                   // row operand: slab[opd + 16 b STRIDE + 4 c]
    const uint32_t trs = (4u * g + (n >> 2)) * SROW + 4u * (n & 3);  // transposing-read base inside a slab
    // The output rows of a wave leave through 16 x 144 bytes of LDS of its own, four 16-channel blocks
    // (a 128-byte line per row) at a time: written in accumulator order, read back 16 bytes per lane,
    // two stores of 8 whole lines each instead of four stores of 32-byte pieces (12 % at width 128,
    // 8-11 % at width 64 although the 9 KB cost it one of its three workgroups per CU).
    char* const mine = reinterpret_cast<char*>(ex + NT * XT) + role * (16 * 144);
    auto gather = [&](const u32x2 v, int cb) { *reinterpret_cast<u32x2*>(mine + n * 144 + (cb & 3) * 32 + g * 8) = v; };
    auto flush = [&](const __amdgpu_buffer_rsrc_t dst, int blk, int cb) {
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const uint32_t r = (uint32_t)(8 * i + (lane >> 3)), c = (uint32_t)(lane & 7);
            const u32x4 rows = *reinterpret_cast<const u32x4*>(mine + r * 144 + c * 16);
            __builtin_amdgcn_raw_buffer_store_b128(rows, dst, (uint32_t)(16 * blk + r) * row_d + 128u * (uint32_t)(cb >> 2) + 16u * c, 0, 0);
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
    };
    f32x4 dbacc[NB];
#pragma unroll
    for (int jb = 0; jb < NB; ++jb) dbacc[jb] = zero;

    // The K and V slabs are requested one window ahead, during phase B of the window before, and
    // wait in registers until the slab area is free.
    u32x4 sk[PASSES], sv[PASSES];
    auto request = [&](uint32_t w) {
        const size_t tile = ((size_t)w * L * p.ldq + (size_t)h * D) * 2u;
        const __amdgpu_buffer_rsrc_t rk = make_rsrc((const char*)p.k + tile, tile_bytes);
        const __amdgpu_buffer_rsrc_t rv = make_rsrc((const char*)p.v + tile, tile_bytes);
#pragma unroll
        for (int t = 0; t < PASSES; ++t) {
            const uint32_t o = (RPP * t + srow) * row_bytes + scol * 16u;
            sk[t] = __builtin_amdgcn_raw_buffer_load_b128(rk, o, 0, 0);
            sv[t] = __builtin_amdgcn_raw_buffer_load_b128(rv, o, 0, 0);
        }
    };
    if (bw < (uint32_t)p.N) request(bw);

    for (uint32_t w = bw; w < (uint32_t)p.N; w += G) {
    const bool has_next = w + G < (uint32_t)p.N;
    const size_t tile = ((size_t)w * L * p.ldq + (size_t)h * D) * 2u;
    const size_t tile_g = ((size_t)w * L * p.ldg + (size_t)h * D) * 2u;
    const size_t tile_d = ((size_t)w * L * p.ldd + (size_t)h * D) * 2u;
    const __amdgpu_buffer_rsrc_t rq = make_rsrc((const char*)p.q + tile, tile_bytes);
    const __amdgpu_buffer_rsrc_t rg = make_rsrc((const char*)p.d_o + tile_g, tile_bytes_g);
    // own Q and dO rows as operands: lane (g, n) takes channels 32 c + 8g .. + 7 of row 16 role + n
    bf16x8 qop[CH], gop[CH];
    {
        const uint32_t off = (uint32_t)(16 * role + n) * row_bytes + 16u * g;
        const uint32_t off_g = (uint32_t)(16 * role + n) * row_g + 16u * g;
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            qop[c] = as_bf16x8(__builtin_amdgcn_raw_buffer_load_b128(rq, off + 64 * c, 0, 0));
            gop[c] = as_bf16x8(__builtin_amdgcn_raw_buffer_load_b128(rg, off_g + 64 * c, 0, 0));
        }
    }
#pragma unroll
    for (int t = 0; t < PASSES; ++t) {
        const uint32_t row = RPP * t + srow;
        if (row < (uint32_t)ROWS) {
            sa[row * STRIDE + scol] = __builtin_bit_cast(uint4, sk[t]);
            sb[row * STRIDE + scol] = __builtin_bit_cast(uint4, sv[t]);
        }
    }
    __syncthreads();

    // ---------------- phase A: query block `role` ----------------
    if (active) {
        const int qb = role;
        f32x4 s[NB], dp[NB];
#pragma unroll
        for (int jb = 0; jb < NB; ++jb) s[jb] = dp[jb] = zero;
#pragma unroll
        for (int c = 0; c < CH; ++c)
#pragma unroll
            for (int jb = 0; jb < NB; ++jb) {
                s[jb] = mfma_e<F16>(__builtin_bit_cast(bf16x8, sa[opd + 16 * jb * STRIDE + 4 * c]), qop[c], s[jb]);
                dp[jb] = mfma_e<F16>(__builtin_bit_cast(bf16x8, sb[opd + 16 * jb * STRIDE + 4 * c]), gop[c], dp[jb]);
            }
        // softmax of the block's rows: s <- exp(score - rowmax), inv = 1 / rowsum
        float inv;
        if (BM) {
            const BiasSrc rb = bias_of_head(p, h);
            const AddendGlobal addend = addend_at(rb, mask_of_window(p, w), (uint32_t)(16 * qb + n), 4u * g, (uint32_t)L);
            inv = softmax_block<NB, true>(s, sl2, addend, L, g);
        } else {
            inv = softmax_block<NB, false>(s, sl2, AddendNone{}, L, g);
        }
        float delta = 0.f;
#pragma unroll
        for (int jb = 0; jb < NB; ++jb)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                s[jb][r] *= inv;  // P
                delta = fmaf(s[jb][r], dp[jb][r], delta);
            }
        delta = sum_over_g(delta);
        bf16x4 ds_hi[NB], ds_lo[NB];
#pragma unroll
        for (int jb = 0; jb < NB; ++jb) {
#pragma unroll
            for (int r = 0; r < 4; ++r) dp[jb][r] = s[jb][r] * (dp[jb][r] - delta);  // dS
            if (DB) dbacc[jb] += dp[jb];
            uint16_t* cell = ex + (16 * qb + n) * XS + ((jb ^ (n & 3)) << 4) + ((g ^ ((n >> 2) & 3)) << 2);
            if constexpr (F16) {
                const uint2 ph = {pack_e<true>(s[jb][0], s[jb][1]), pack_e<true>(s[jb][2], s[jb][3])};
                const uint2 dh = {pack_e<true>(dp[jb][0], dp[jb][1]), pack_e<true>(dp[jb][2], dp[jb][3])};
                ds_hi[jb] = as_bf16x4(dh);
                ds_lo[jb] = as_bf16x4(uint2{0u, 0u});
                *reinterpret_cast<uint2*>(cell + 0 * XT) = ph;
                *reinterpret_cast<uint2*>(cell + 1 * XT) = dh;
            } else {
                bf16x4 p_hi, p_lo;
                split_hi_lo(s[jb], p_hi, p_lo);
                split_hi_lo(dp[jb], ds_hi[jb], ds_lo[jb]);
                *reinterpret_cast<uint2*>(cell + 0 * XT) = __builtin_bit_cast(uint2, p_hi);
                *reinterpret_cast<uint2*>(cell + 1 * XT) = __builtin_bit_cast(uint2, p_lo);
                *reinterpret_cast<uint2*>(cell + 2 * XT) = __builtin_bit_cast(uint2, ds_hi[jb]);
                *reinterpret_cast<uint2*>(cell + 3 * XT) = __builtin_bit_cast(uint2, ds_lo[jb]);
            }
        }
        // dS of pairs of key blocks as operands (keys on the k-slots)
        bf16x8 dh[NB2], dl[NB2];
#pragma unroll
        for (int kp = 0; kp < NB2; ++kp) {
            const bool two = 2 * kp + 1 < NB;
            const uint2 h0 = __builtin_bit_cast(uint2, ds_hi[2 * kp]), l0 = __builtin_bit_cast(uint2, ds_lo[2 * kp]);
            uint2 h1 = {0u, 0u}, l1 = {0u, 0u};
            if (two) {
                h1 = __builtin_bit_cast(uint2, ds_hi[two ? 2 * kp + 1 : 0]);
                l1 = __builtin_bit_cast(uint2, ds_lo[two ? 2 * kp + 1 : 0]);
            }
            dh[kp] = as_bf16x8(u32x4{h0.x, h0.y, h1.x, h1.y});
            dl[kp] = as_bf16x8(u32x4{l0.x, l0.y, l1.x, l1.y});
        }
        // dQ^T = K^T dS^T, 16 channels at a time: acc[r] = dQ[16 qb + n][16 cb + 4g + r]
        const uint16_t* lk16 = reinterpret_cast<const uint16_t*>(sa) + trs;
        const __amdgpu_buffer_rsrc_t rdq = make_rsrc((char*)p.dq + tile_d, tile_bytes_d);
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) {
            f32x4 acc = zero;
#pragma unroll
            for (int kp = 0; kp < NB2; ++kp) {
                const bf16x8 kt = operand_tr(lk16 + (32 * kp) * SROW + 16 * cb, 16 * SROW, 2 * kp + 1 < NB);
                acc = mfma_e<F16>(kt, dh[kp], acc);
                if constexpr (!F16) acc = mfma_bf16(kt, dl[kp], acc);
            }
            const u32x2 v = {pack_e<F16>(acc[0] * p.scale, acc[1] * p.scale), pack_e<F16>(acc[2] * p.scale, acc[3] * p.scale)};
            gather(v, cb);
            if ((cb & 3) == 3) flush(rdq, qb, cb);
        }
    }
    __syncthreads();  // K, V no longer needed; tiles complete
    // The Q and dO slabs of phase B take their place: the four waves hold all rows between them,
    // as the operands of phase A, and put them down themselves (no second read of Q and dO).
    if (active) {
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            sa[opd + 16 * role * STRIDE + 4 * c] = __builtin_bit_cast(uint4, qop[c]);
            sb[opd + 16 * role * STRIDE + 4 * c] = __builtin_bit_cast(uint4, gop[c]);
        }
    }
    __syncthreads();
    if (has_next) request(w + G);  // in flight during phase B

    // ---------------- phase B: key block `role` ----------------
    if (active) {
        const int jb = role;
        // P and dS of all queries for this key block (key on the lane, queries on the k-slots)
        const uint16_t* xt = ex + (4u * g + (n >> 2)) * XS + ((((uint32_t)jb) ^ (uint32_t)(n >> 2)) << 4) +
                             ((((uint32_t)n & 3u) ^ (uint32_t)g) << 2);
        bf16x8 ph[NB2], pl[NB2], sh[NB2], sl[NB2];
#pragma unroll
        for (int qp = 0; qp < NB2; ++qp) {
            const bool two = 2 * qp + 1 < NB;
            ph[qp] = operand_tr(xt + 0 * XT + (32 * qp) * XS, 16 * XS, two);
            sh[qp] = operand_tr(xt + (F16 ? 1 : 2) * XT + (32 * qp) * XS, 16 * XS, two);
            if constexpr (!F16) {
                pl[qp] = operand_tr(xt + 1 * XT + (32 * qp) * XS, 16 * XS, two);
                sl[qp] = operand_tr(xt + 3 * XT + (32 * qp) * XS, 16 * XS, two);
            }
        }
        const uint16_t* lq16 = reinterpret_cast<const uint16_t*>(sa) + trs;
        const uint16_t* lg16 = reinterpret_cast<const uint16_t*>(sb) + trs;
        const __amdgpu_buffer_rsrc_t rdv = make_rsrc((char*)p.dv + tile_d, tile_bytes_d);
        const __amdgpu_buffer_rsrc_t rdk = make_rsrc((char*)p.dk + tile_d, tile_bytes_d);
        u32x2 kwait[4];
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) {
            f32x4 av = zero, ak = zero;  // dV, dK [16 jb + n][16 cb + 4g + r]
#pragma unroll
            for (int qp = 0; qp < NB2; ++qp) {
                const bool two = 2 * qp + 1 < NB;
                const bf16x8 gt = operand_tr(lg16 + (32 * qp) * SROW + 16 * cb, 16 * SROW, two);
                const bf16x8 qt = operand_tr(lq16 + (32 * qp) * SROW + 16 * cb, 16 * SROW, two);
                av = mfma_e<F16>(gt, ph[qp], av);
                ak = mfma_e<F16>(qt, sh[qp], ak);
                if constexpr (!F16) {
                    av = mfma_bf16(gt, pl[qp], av);
                    ak = mfma_bf16(qt, sl[qp], ak);
                }
            }
            const u32x2 vv = {pack_e<F16>(av[0], av[1]), pack_e<F16>(av[2], av[3])};
            const u32x2 vk = {pack_e<F16>(ak[0] * p.scale, ak[1] * p.scale), pack_e<F16>(ak[2] * p.scale, ak[3] * p.scale)};
            // dV through the cells block by block; dK waits in registers and follows
            gather(vv, cb);
            kwait[cb & 3] = vk;
            if ((cb & 3) == 3) {
                flush(rdv, jb, cb);
#pragma unroll
                for (int t = 0; t < 4; ++t) gather(kwait[t], t);
                flush(rdk, jb, cb);
            }
        }
    }
    if (has_next) __syncthreads();  // slabs and tiles are rewritten for the next window
    }

    if (DB && active) {
        // partial sums in register order: [slot][head][qb][jb][lane] float4 -- contiguous 16-byte stores
        f32x4* dst = reinterpret_cast<f32x4*>(p.partial) + ((size_t)bw * p.heads + h) * (NB * NB * 64) + lane;
#pragma unroll
        for (int jb = 0; jb < NB; ++jb) dst[(role * NB + jb) * 64] = dbacc[jb];
    }
}

template <int NB, int D, bool BM, bool DB, bool F16>
hipError_t launch_wide_one(const BwdArgs& a, unsigned G, hipStream_t st) {
    // K, V (then Q, dO) slabs; the P / dS tiles (two for half data, four hi / lo tiles for bf16); output cells
    const size_t lds = (size_t)2 * 16 * NB * (D / 8 + 1) * 16 + (size_t)(F16 ? 2 : 4) * 16 * NB * 64 * 2 + (size_t)4 * 16 * 144;
    const hipError_t e = allow_lds(reinterpret_cast<const void*>(&bwd_bf16_wide_kernel<NB, D, BM, DB, F16>), lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((bwd_bf16_wide_kernel<NB, D, BM, DB, F16>), dim3(G * (unsigned)a.heads), dim3(256), lds, st, a, G);
    return hipGetLastError();
}

template <int NB, int D, bool F16>
hipError_t launch_wide_nb(const BwdArgs& a, hipStream_t st) {
    const bool bm = a.bias || has_mask(a);
    if (a.dbias == nullptr) {
        // Width 256 (100 KB of LDS: one workgroup per CU): as many window positions as workgroups stay
        // resident, 5 % faster than one window per workgroup; narrower heads (2-3 workgroups per
        // CU) are 5-8 % faster with one window each.
        long long G0 = a.N;
        const long long per_head = cu_count() / a.heads;
        if (D == 256 && a.N > per_head) G0 = per_head > 0 ? per_head : 1;
        return bm ? launch_wide_one<NB, D, true, false, F16>(a, (unsigned)G0, st)
                  : launch_wide_one<NB, D, false, false, F16>(a, (unsigned)G0, st);
    }
    const unsigned G = (unsigned)a.slots;
    const hipError_t e = bm ? launch_wide_one<NB, D, true, true, F16>(a, G, st)
                            : launch_wide_one<NB, D, false, true, F16>(a, G, st);
    return e != hipSuccess ? e : launch_dbias_reduce(a, st);
}

template <int D>
hipError_t launch_wide_d(const BwdArgs& a, hipStream_t s) {
    switch ((a.L + 15) / 16) {
        case 1: return a.f16 ? launch_wide_nb<1, D, true>(a, s) : launch_wide_nb<1, D, false>(a, s);
        case 2: return a.f16 ? launch_wide_nb<2, D, true>(a, s) : launch_wide_nb<2, D, false>(a, s);
        case 3: return a.f16 ? launch_wide_nb<3, D, true>(a, s) : launch_wide_nb<3, D, false>(a, s);
        case 4: return a.f16 ? launch_wide_nb<4, D, true>(a, s) : launch_wide_nb<4, D, false>(a, s);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace

// Window positions walked in parallel (= dBias slots) when dBias is wanted: two or three resident
// workgroups per CU; never more than the single-wave kernel's count, which sizes the workspace.
int backward_wide_slots(long long N, int heads) {
    long long G = 2 * cu_count() / heads;
    if (G < 1) G = 1;
    return (int)(G > N ? N : G);
}

hipError_t launch_backward_bf16_wide(const BwdArgs& a, hipStream_t s) {
    switch (a.C / a.heads) {
        case 64: return launch_wide_d<64>(a, s);
        case 128: return launch_wide_d<128>(a, s);
        case 256: return launch_wide_d<256>(a, s);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace fwa
