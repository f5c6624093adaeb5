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
//   * in that layout the probabilities of a lane are already the A operand of
//     P V (its k-slots are keys 4g..4g+3 of two neighbouring tiles); V is
//     loaded as dwords (channel pair 2n, 2n+1 of those same keys) and split
//     into an even-channel and an odd-channel B operand, so the two output
//     accumulators of a lane are neighbouring channels and are stored as one
//     packed dword;
//   * rows/columns beyond L (L is padded to a multiple of 16 on chip only)
//     load as zero, padded score columns are set to -inf, padded rows are
//     never stored.  Nothing is read or written outside [N, L, C].
#include "fwa_device.h"
#include "fwa_internal.h"

namespace fwa {
namespace {

// ---------------------------------------------------------------- bf16 ----
// NB = ceil(L / 16) key/query blocks; BM = a bias and/or mask is present.
template <int NB, bool BM>
__global__ void __launch_bounds__(64 * kWavesPerBlock)
fwd_bf16_kernel(FwdArgs p, int qsplit, int qb_per_split, long long ntasks) {
    constexpr int NB2 = (NB + 1) / 2;
    const int lane = threadIdx.x & 63;
    const int n = lane & 15, g = lane >> 4;
    const long long task = (long long)blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6);
    if (task >= ntasks) return;  // wave-uniform; the kernel has no barriers
    const int qs = (int)(task % qsplit);
    const long long wh = task / qsplit;
    const int h = (int)(wh % p.heads);
    const long long w = wh / p.heads;
    const int L = p.L, C = p.C;
    const size_t tile = (size_t)w * L * C + (size_t)h * kHeadDim;
    const uint16_t* Qw = (const uint16_t*)p.q + tile;
    const uint16_t* Kw = (const uint16_t*)p.k + tile;
    const uint16_t* Vw = (const uint16_t*)p.v + tile;
    uint16_t* Ow = (uint16_t*)p.o + tile;

    // K: A operands, lane (g, n) = K[16 jb + n][8g .. 8g+7]
    bf16x8 kop[NB];
#pragma unroll
    for (int jb = 0; jb < NB; ++jb) {
        const int row = 16 * jb + n;
        uint4 t = {0u, 0u, 0u, 0u};
        if (row < L) t = *(const uint4*)(Kw + (size_t)row * C + 8 * g);
        kop[jb] = as_bf16x8(t);
    }
    // V: B operands for key pairs of blocks, even and odd channel
    bf16x8 vop[NB2][2];
#pragma unroll
    for (int kp = 0; kp < NB2; ++kp) {
        uint32_t d[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int key = 32 * kp + slot_row(g, e);
            d[e] = 0u;
            if (key < L) d[e] = *(const uint32_t*)(Vw + (size_t)key * C + 2 * n);
        }
        split_pairs(d, vop[kp][0], vop[kp][1]);
    }

    const float sl2 = p.scale * kLog2e;
    const float* bias_h = BM && p.bias ? p.bias + (size_t)h * L * L : nullptr;
    const float* mask_w = BM && p.mask ? p.mask + (size_t)(w % p.nW) * L * L : nullptr;

    const int qb_end = min(NB, (qs + 1) * qb_per_split);
    for (int qb = qs * qb_per_split; qb < qb_end; ++qb) {
        const int i = 16 * qb + n;  // the query row this lane's scores belong to
        uint4 t = {0u, 0u, 0u, 0u};
        if (i < L) t = *(const uint4*)(Qw + (size_t)i * C + 8 * g);
        const bf16x8 qop = as_bf16x8(t);

        f32x4 s[NB];
        float m = -INFINITY;
#pragma unroll
        for (int jb = 0; jb < NB; ++jb) {
            const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
            s[jb] = mfma_bf16(kop[jb], qop, zero);
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int j = 16 * jb + 4 * g + r;
                float x = s[jb][r] * sl2;
                if (BM) {
                    float add = 0.f;
                    if (i < L && j < L) {
                        if (bias_h) add += bias_h[(size_t)i * L + j];
                        if (mask_w) add += mask_w[(size_t)i * L + j];
                    }
                    x = fmaf(add, kLog2e, x);
                }
                if (jb == NB - 1 && j >= L) x = -INFINITY;
                s[jb][r] = x;
                m = fmaxf(m, x);
            }
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
        const float inv = 1.0f / sum;

        f32x4 oe = {0.f, 0.f, 0.f, 0.f}, oo = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kp = 0; kp < NB2; ++kp) {
            uint4 a;
            a.x = pack_bf16(s[2 * kp][0], s[2 * kp][1]);
            a.y = pack_bf16(s[2 * kp][2], s[2 * kp][3]);
            const int j1 = 2 * kp + 1 < NB ? 2 * kp + 1 : 0;  // odd NB: the last pair has no second tile
            a.z = 2 * kp + 1 < NB ? pack_bf16(s[j1][0], s[j1][1]) : 0u;
            a.w = 2 * kp + 1 < NB ? pack_bf16(s[j1][2], s[j1][3]) : 0u;
            const bf16x8 pop = as_bf16x8(a);
            oe = mfma_bf16(pop, vop[kp][0], oe);
            oo = mfma_bf16(pop, vop[kp][1], oo);
        }
        // accumulators: oe[r] = O[16 qb + 4g + r][2n], oo[r] = ...[2n+1];
        // the row sum of query 4g + r sits in lane 4g + r (any row).
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const float inv_r = __shfl(inv, 4 * g + r);
            const int io = 16 * qb + 4 * g + r;
            if (io < L) *(uint32_t*)(Ow + (size_t)io * C + 2 * n) = pack_bf16(oe[r] * inv_r, oo[r] * inv_r);
        }
    }
}

// ---------------------------------------------------------------- fp32 ----
// Same tile ownership and layouts with v_mfma_f32_16x16x4_f32 (true fp32
// products): k-slot g of step kk stands for channel 8g + kk in QK^T and for
// key 16 jb + 4g + r in step (jb, r) of PV.  V is streamed from cache per
// query block instead of being held in registers.
template <int NB, bool BM>
__global__ void __launch_bounds__(64 * kWavesPerBlock)
fwd_f32_kernel(FwdArgs p, int qsplit, int qb_per_split, long long ntasks) {
    const int lane = threadIdx.x & 63;
    const int n = lane & 15, g = lane >> 4;
    const long long task = (long long)blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6);
    if (task >= ntasks) return;
    const int qs = (int)(task % qsplit);
    const long long wh = task / qsplit;
    const int h = (int)(wh % p.heads);
    const long long w = wh / p.heads;
    const int L = p.L, C = p.C;
    const size_t tile = (size_t)w * L * C + (size_t)h * kHeadDim;
    const float* Qw = (const float*)p.q + tile;
    const float* Kw = (const float*)p.k + tile;
    const float* Vw = (const float*)p.v + tile;
    float* Ow = (float*)p.o + tile;

    float kop[NB][8];
#pragma unroll
    for (int jb = 0; jb < NB; ++jb) {
        const int row = 16 * jb + n;
        float4 a = {0.f, 0.f, 0.f, 0.f}, b = {0.f, 0.f, 0.f, 0.f};
        if (row < L) {
            a = *(const float4*)(Kw + (size_t)row * C + 8 * g);
            b = *(const float4*)(Kw + (size_t)row * C + 8 * g + 4);
        }
        kop[jb][0] = a.x; kop[jb][1] = a.y; kop[jb][2] = a.z; kop[jb][3] = a.w;
        kop[jb][4] = b.x; kop[jb][5] = b.y; kop[jb][6] = b.z; kop[jb][7] = b.w;
    }
    const float* bias_h = BM && p.bias ? p.bias + (size_t)h * L * L : nullptr;
    const float* mask_w = BM && p.mask ? p.mask + (size_t)(w % p.nW) * L * L : nullptr;

    const int qb_end = min(NB, (qs + 1) * qb_per_split);
    for (int qb = qs * qb_per_split; qb < qb_end; ++qb) {
        const int i = 16 * qb + n;
        float qop[8];
        {
            float4 a = {0.f, 0.f, 0.f, 0.f}, b = {0.f, 0.f, 0.f, 0.f};
            if (i < L) {
                a = *(const float4*)(Qw + (size_t)i * C + 8 * g);
                b = *(const float4*)(Qw + (size_t)i * C + 8 * g + 4);
            }
            qop[0] = a.x; qop[1] = a.y; qop[2] = a.z; qop[3] = a.w;
            qop[4] = b.x; qop[5] = b.y; qop[6] = b.z; qop[7] = b.w;
        }
        f32x4 s[NB];
        float m = -INFINITY;
#pragma unroll
        for (int jb = 0; jb < NB; ++jb) {
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kk = 0; kk < 8; ++kk) acc = mfma_f32(kop[jb][kk], qop[kk], acc);
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int j = 16 * jb + 4 * g + r;
                float x = acc[r] * p.scale;
                if (BM) {
                    if (i < L && j < L) {
                        if (bias_h) x += bias_h[(size_t)i * L + j];
                        if (mask_w) x += mask_w[(size_t)i * L + j];
                    }
                }
                if (jb == NB - 1 && j >= L) x = -INFINITY;
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
                const int key = 16 * jb + 4 * g + r;
                float v0 = 0.f, v1 = 0.f;
                if (key < L) {
                    v0 = Vw[(size_t)key * C + n];
                    v1 = Vw[(size_t)key * C + 16 + n];
                }
                o0 = mfma_f32(s[jb][r], v0, o0);
                o1 = mfma_f32(s[jb][r], v1, o1);
            }
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const float sum_r = __shfl(sum, 4 * g + r);
            const int io = 16 * qb + 4 * g + r;
            if (io < L) {
                Ow[(size_t)io * C + n] = o0[r] / sum_r;
                Ow[(size_t)io * C + 16 + n] = o1[r] / sum_r;
            }
        }
    }
}

struct Split {
    int qsplit, qb_per_split;
};
// How many waves share the query blocks of one tile.
inline Split choose_split(int nb) {
    Split s;
    s.qb_per_split = nb <= 4 ? nb : 4;
    s.qsplit = (nb + s.qb_per_split - 1) / s.qb_per_split;
    return s;
}

template <int NB>
hipError_t launch_bf16_nb(const FwdArgs& a, hipStream_t st) {
    const Split sp = choose_split(NB);
    const long long ntasks = a.N * a.heads * sp.qsplit;
    const unsigned grid = (unsigned)((ntasks + kWavesPerBlock - 1) / kWavesPerBlock);
    if (a.bias || a.mask)
        hipLaunchKernelGGL((fwd_bf16_kernel<NB, true>), dim3(grid), dim3(64 * kWavesPerBlock), 0, st, a,
                           sp.qsplit, sp.qb_per_split, ntasks);
    else
        hipLaunchKernelGGL((fwd_bf16_kernel<NB, false>), dim3(grid), dim3(64 * kWavesPerBlock), 0, st, a,
                           sp.qsplit, sp.qb_per_split, ntasks);
    return hipGetLastError();
}

template <int NB>
hipError_t launch_f32_nb(const FwdArgs& a, hipStream_t st) {
    const Split sp = choose_split(NB);
    const long long ntasks = a.N * a.heads * sp.qsplit;
    const unsigned grid = (unsigned)((ntasks + kWavesPerBlock - 1) / kWavesPerBlock);
    if (a.bias || a.mask)
        hipLaunchKernelGGL((fwd_f32_kernel<NB, true>), dim3(grid), dim3(64 * kWavesPerBlock), 0, st, a,
                           sp.qsplit, sp.qb_per_split, ntasks);
    else
        hipLaunchKernelGGL((fwd_f32_kernel<NB, false>), dim3(grid), dim3(64 * kWavesPerBlock), 0, st, a,
                           sp.qsplit, sp.qb_per_split, ntasks);
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

hipError_t launch_forward_bf16(const FwdArgs& a, hipStream_t s) {
    const int nb = (a.L + 15) / 16;
    FWA_NB_SWITCH(launch_bf16_nb, nb, a, s)
}

hipError_t launch_forward_f32(const FwdArgs& a, hipStream_t s) {
    const int nb = (a.L + 15) / 16;
    FWA_NB_SWITCH(launch_f32_nb, nb, a, s)
}

}  // namespace fwa
