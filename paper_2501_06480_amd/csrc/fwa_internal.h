// Internal declarations shared by the HIP translation units of libfwa.
// Nothing here is part of the public ABI (see include/fwa.h for that).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <atomic>

namespace fwa {

constexpr int kHeadDim = 32;   // head width of every path but the wide-head kernels
constexpr int kMaxWideL = 64;  // wide-head kernels (head widths 64, 128, 256): the tile of one window
constexpr int kMaxL = 256;     // 16 key blocks of 16 rows
constexpr int kMaxBackwardL = 64;  // backward: largest window whose score tile stays on chip (and that has dBias)
constexpr int kWavesPerBlock = 4;

struct FwdArgs {
    const void* q;
    const void* k;
    const void* v;
    void* o;
    const void* bias;    // [heads, L, L], fp32 or (bias_bf16) bf16, or nullptr
    int bias_bf16;
    const float* mask;   // [nW, L, L] or nullptr
    const int32_t* labels;  // [nW, L] region labels standing for the mask, or nullptr; never together with mask
    float mask_value;       // what labels that differ add to a score
    long long N;
    int L;
    int C;
    int heads;
    int nW;
    float scale;
    int ldq;             // elements between consecutive token rows of q, k, v (C when contiguous)
    int ldo;             // the same for o
    int f16;             // the 16-bit data are IEEE half, not bf16 (wide-head kernels only)
};

struct BwdArgs {
    const void* q;
    const void* k;
    const void* v;
    const void* d_o;
    void* dq;
    void* dk;
    void* dv;
    float* dbias;        // [heads, L, L] or nullptr
    float* partial;      // workspace for per-slot dS sums, or nullptr
    float* stats;        // workspace [N, heads, 2, 16 * ceil(L / 16)] for the row statistics (L > 64 with dbias), or nullptr
    const void* bias;    // as in FwdArgs
    int bias_bf16;
    const float* mask;
    const int32_t* labels;  // as in FwdArgs
    float mask_value;
    long long N;
    int L;
    int C;
    int heads;
    int nW;
    float scale;
    int slots;           // number of partial-sum slots per head in `partial`
    int per_window;      // cooperative kernel for L <= 64: the mask is formed per window from the labels (a period
                         // that no slot count is a multiple of); only the bias stays in registers
    int ldq;             // elements between consecutive token rows of q, k, v (C when contiguous)
    int ldg;             // the same for d_o
    int ldd;             // the same for dq, dk, dv
    int f16;             // the 16-bit data are IEEE half, not bf16 (wide-head kernels only)
};

// Whether the scores get a mask, in either form, and its period over the windows (1 without one).
template <class Args>
inline bool has_mask(const Args& a) { return a.mask != nullptr || a.labels != nullptr; }
template <class Args>
inline int mask_period(const Args& a) { return has_mask(a) ? a.nW : 1; }

// Compute units of the current device, asked from the runtime once per device (256 on MI355X; the
// same figure stands in when no device answers, e.g. a workspace-size query on a machine without a
// GPU).  Workgroup counts of the persistent kernels and dBias slot counts are derived from it.
int cu_count();

// Lifts the 64 KB limit on dynamic LDS for kernel `fn` on the current device (to the 160 KB of a
// compute unit), once per kernel and device; a no-op for requests of at most 64 KB.  Lock-free: two
// threads racing through a kernel's first call merely ask the runtime twice.
hipError_t allow_lds(const void* fn, size_t lds_bytes);

// Each returns a hipError_t from the launch (hipSuccess when enqueued).
hipError_t launch_forward_bf16(const FwdArgs& a, hipStream_t s);
hipError_t launch_forward_f32(const FwdArgs& a, hipStream_t s);
hipError_t launch_forward_f32_tile(const FwdArgs& a, hipStream_t s);
int staged_heads_per_block(int L, int heads);
hipError_t launch_forward_bf16_staged(const FwdArgs& a, hipStream_t s);
bool forward_wide_supported(int L, int head_dim);
hipError_t launch_forward_bf16_wide(const FwdArgs& a, hipStream_t s);
hipError_t launch_backward_bf16(const BwdArgs& a, hipStream_t s);
hipError_t launch_backward_f32(const BwdArgs& a, hipStream_t s);
int backward_slots(long long N, int heads, int nW);
int backward_max_slots(long long N, int heads);
int coop_slots(long long N, int heads, int nW);
hipError_t launch_backward_bf16_coop(const BwdArgs& a, hipStream_t s);
hipError_t launch_backward_bf16_single(const BwdArgs& a, hipStream_t s);
hipError_t launch_backward_bf16_large(const BwdArgs& a, hipStream_t s);
hipError_t launch_backward_bf16_wide(const BwdArgs& a, hipStream_t s);
int backward_wide_slots(long long N, int heads);
hipError_t launch_dbias_reduce(const BwdArgs& a, hipStream_t s, bool key_on_lane = false);
int backward_large_slots(long long N, int heads, int L);
hipError_t launch_zero_f32(float* dst, size_t count, hipStream_t s);
hipError_t launch_widen_bf16(const void* src, float* dst, size_t count, hipStream_t s);
hipError_t launch_bias_gather(const float* table, float* bias, int heads, int k, hipStream_t s);
hipError_t launch_bias_scatter(const float* dbias, float* dtable, int heads, int k, hipStream_t s);

}  // namespace fwa
