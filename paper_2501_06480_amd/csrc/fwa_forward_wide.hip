// Forward for head widths 64, 128 and 256 at L <= 64: the shapes of the paper's own kernel
// benchmark (section 3.1: L = 64, 4 heads, the width per head swept upwards).
//
// This is where the paper's feature-dimension loop (eq. 5-6) does real work: the score product
// is accumulated over D / 32 chunks of 32 channels (one matrix-core k-step each), and the output
// is produced in D / 16 blocks of 16 channels.  One workgroup per (window, head), one wave per
// 16-query block.  The head's K and V rows (D * 2 bytes each: whole 128-byte lines) go to LDS
// with coalesced 16-byte loads, one after the other through the same slab; a wave reads its own
// Q rows straight from global memory as operands, one 16-byte load per chunk.  Register
// layouts are those of the other forward kernels ("query on the lane"): S^T = K Q^T chunk by
// chunk into the same accumulators, softmax across the 4 lanes that share a query, and
// O^T = V^T P^T channel block by channel block with V^T from the transposing LDS read.
#include "fwa_device.h"
#include "fwa_internal.h"
#include "fwa_softmax.h"

namespace fwa {
namespace {

// F16: the data are IEEE half instead of bf16 (the precision the paper's Section 3.3 comparison runs in);
// same bytes, same layouts, the other matrix instruction and conversion.
template <int NB, int D, bool BM, bool F16>
__global__ void __launch_bounds__(256) fwd_bf16_wide_kernel(FwdArgs p) {
    constexpr int NB2 = (NB + 1) / 2;
    constexpr int ROWS = 16 * NB;
    constexpr int CH = D / 32;               // chunks of the score product
    constexpr int CB = D / 16;               // 16-channel blocks of the output
    constexpr uint32_t STRIDE = D / 8 + 1;   // slab row in 16-byte units: D * 2 bytes of data + 16 of padding
    constexpr uint32_t SROW = STRIDE * 8;    // the same in bf16 elements
    constexpr int TPR = D / 8;               // threads that move one slab row
    constexpr int RPP = 256 / TPR;           // rows per pass of the workgroup
    constexpr int PASSES = (ROWS + RPP - 1) / RPP;
    extern __shared__ __attribute__((aligned(16))) uint4 lds[];  // one slab [ROWS][STRIDE]: K, then V
    const int tid = threadIdx.x, lane = tid & 63;
    const int n = lane & 15, g = lane >> 4;
    const int qb = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bool active = qb < NB;  // the other waves only move slab rows
    const uint32_t w = blockIdx.x / (uint32_t)p.heads, h = blockIdx.x % (uint32_t)p.heads;
    const int L = p.L;
    const uint32_t row_bytes = (uint32_t)p.ldq * 2u, row_out = (uint32_t)p.ldo * 2u;  // token rows: ldq / ldo elements apart
    const size_t tile = ((size_t)w * L * p.ldq + (size_t)h * D) * 2u;
    const uint32_t tile_bytes = (uint32_t)(L - 1) * row_bytes + 2u * D;  // rows beyond L read as zero

    // K and V take turns in one slab: V is requested once K is parked, waits in registers while the
    // scores are made, and is parked behind a barrier.  Half the LDS of two slabs means twice the
    // workgroups per CU at widths 128 and 256, where LDS is what limits them.
    const uint32_t srow = (uint32_t)tid / TPR, scol = (uint32_t)tid % TPR;
    u32x4 slab[PASSES];
    {
        const __amdgpu_buffer_rsrc_t rk = make_rsrc((const char*)p.k + tile, tile_bytes);
#pragma unroll
        for (int t = 0; t < PASSES; ++t)
            slab[t] = __builtin_amdgcn_raw_buffer_load_b128(rk, (RPP * t + srow) * row_bytes + scol * 16u, 0, 0);
    }
    // Q rows of this wave's block as operands: lane (g, n) takes channels 32 c + 8g .. + 7 of row n
    bf16x8 qop[CH];
    {
        const __amdgpu_buffer_rsrc_t rq = make_rsrc((const char*)p.q + tile, tile_bytes);
        const uint32_t off = (uint32_t)(16 * qb + n) * row_bytes + 16u * g;
#pragma unroll
        for (int c = 0; c < CH; ++c) qop[c] = as_bf16x8(__builtin_amdgcn_raw_buffer_load_b128(rq, off + 64 * c, 0, 0));
    }
    auto park = [&]() {
#pragma unroll
        for (int t = 0; t < PASSES; ++t) {
            const uint32_t row = RPP * t + srow;
            if (row < (uint32_t)ROWS) lds[row * STRIDE + scol] = __builtin_bit_cast(uint4, slab[t]);
        }
    };
    park();
    {
        const __amdgpu_buffer_rsrc_t rv = make_rsrc((const char*)p.v + tile, tile_bytes);
#pragma unroll
        for (int t = 0; t < PASSES; ++t)
            slab[t] = __builtin_amdgcn_raw_buffer_load_b128(rv, (RPP * t + srow) * row_bytes + scol * 16u, 0, 0);
    }
    __syncthreads();

    // scores: S[16 qb + n][16 jb + 4g + r], accumulated over the chunks
    f32x4 s[NB];
#pragma unroll
    for (int jb = 0; jb < NB; ++jb) s[jb] = f32x4{0.f, 0.f, 0.f, 0.f};
    if (active) {
        const uint4* const lkh = lds + n * STRIDE + g;  // K[16 jb + n][32 c + 8g ..] at lkh[16 jb STRIDE + 4 c]
#pragma unroll
        for (int c = 0; c < CH; ++c)
#pragma unroll
            for (int jb = 0; jb < NB; ++jb)
                s[jb] = mfma_e<F16>(__builtin_bit_cast(bf16x8, lkh[16 * jb * STRIDE + 4 * c]), qop[c], s[jb]);
    }
    __syncthreads();  // every wave has read its K operands
    park();

    const float sl2 = p.scale * kLog2e;
    float inv = 1.f;
    if (active) {
        if (BM) {
            const BiasSrc rb = bias_of_head(p, h);
            const AddendGlobal addend = addend_at(rb, mask_of_window(p, w), (uint32_t)(16 * qb + n), 4u * g, (uint32_t)L);
            inv = softmax_block<NB, true>(s, sl2, addend, L, g);
        } else {
            inv = softmax_block<NB, false>(s, sl2, AddendNone{}, L, g);
        }
    }
    __syncthreads();  // V is in place
    if (!active) return;  // no barrier follows
    bf16x8 pop[NB2];
#pragma unroll
    for (int kp = 0; kp < NB2; ++kp) pop[kp] = prob_operand<NB, F16>(s, kp);

    // O^T = V^T P^T, 16 channels at a time: o[r] = O[16 qb + n][16 cb + 4g + r]
    const uint16_t* const lvh = reinterpret_cast<const uint16_t*>(lds) + (4 * g + (n >> 2)) * SROW + 4 * (n & 3);
    const __amdgpu_buffer_rsrc_t ro = make_rsrc((char*)p.o + ((size_t)w * L * p.ldo + (size_t)h * D) * 2u,
                                                (uint32_t)(L - 1) * row_out + 2u * D);
    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
    char* const mine = reinterpret_cast<char*>(lds + ROWS * STRIDE) + qb * (16 * 144);  // behind the slab
#pragma unroll
    for (int cb = 0; cb < CB; ++cb) {
        f32x4 o = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kp = 0; kp < NB2; ++kp)
            o = mfma_e<F16>(operand_tr(lvh + (32 * kp) * SROW + 16 * cb, 16 * SROW, 2 * kp + 1 < NB), pop[kp], o);
        const u32x2 v = {pack_e<F16>(o[0] * inv, o[1] * inv), pack_e<F16>(o[2] * inv, o[3] * inv)};
        // Four channel blocks (64 channels, a 128-byte line per row) are gathered in LDS cells of this wave's
        // own -- rows 144 bytes apart -- and leave as two 16-byte-per-lane stores of 8 whole lines each,
        // instead of four stores of 32-byte pieces.
        *reinterpret_cast<u32x2*>(mine + n * 144 + (cb & 3) * 32 + g * 8) = v;
        if ((cb & 3) == 3) {
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const uint32_t r = (uint32_t)(8 * i + (lane >> 3)), c = (uint32_t)(lane & 7);
                const u32x4 rows = *reinterpret_cast<const u32x4*>(mine + r * 144 + c * 16);
                __builtin_amdgcn_raw_buffer_store_b128(rows, ro, (uint32_t)(16 * qb + r) * row_out + 128u * (uint32_t)(cb >> 2) + 16u * c, 0, 0);
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
        }
    }
}

template <int NB, int D, bool BM, bool F16>
hipError_t launch_wide_one(const FwdArgs& a, hipStream_t st) {
    const unsigned grid = (unsigned)(a.N * a.heads);
    const size_t lds = (size_t)16 * NB * (D / 8 + 1) * 16 + (size_t)4 * 16 * 144;  // one slab (K, then V); output cells of the waves
    const hipError_t e = allow_lds(reinterpret_cast<const void*>(&fwd_bf16_wide_kernel<NB, D, BM, F16>), lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((fwd_bf16_wide_kernel<NB, D, BM, F16>), dim3(grid), dim3(256), lds, st, a);
    return hipGetLastError();
}

template <int NB, int D>
hipError_t launch_wide_nb(const FwdArgs& a, hipStream_t st) {
    const bool bm = a.bias || has_mask(a);
    if (a.f16) return bm ? launch_wide_one<NB, D, true, true>(a, st) : launch_wide_one<NB, D, false, true>(a, st);
    return bm ? launch_wide_one<NB, D, true, false>(a, st) : launch_wide_one<NB, D, false, false>(a, st);
}

template <int D>
hipError_t launch_wide_d(const FwdArgs& a, hipStream_t s) {
    switch ((a.L + 15) / 16) {
        case 1: return launch_wide_nb<1, D>(a, s);
        case 2: return launch_wide_nb<2, D>(a, s);
        case 3: return launch_wide_nb<3, D>(a, s);
        case 4: return launch_wide_nb<4, D>(a, s);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace

bool forward_wide_supported(int L, int head_dim) {
    return L <= kMaxWideL && (head_dim == 64 || head_dim == 128 || head_dim == 256);
}

hipError_t launch_forward_bf16_wide(const FwdArgs& a, hipStream_t s) {
    switch (a.C / a.heads) {
        case 64: return launch_wide_d<64>(a, s);
        case 128: return launch_wide_d<128>(a, s);
        case 256: return launch_wide_d<256>(a, s);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace fwa
