// extern "C" entry points of libfwa: argument validation and dispatch.
// Every check happens before any HIP call, so an error never launches work.
#include "../../include/fwa.h"
#include "fwa_internal.h"

namespace fwa {

namespace {
constexpr int kDeviceSlots = 64;
std::atomic<int> g_cu_count[kDeviceSlots];  // 0 = not asked yet

// kernel -> devices on which its dynamic-LDS limit has been lifted: an open-addressing table that
// only ever grows (a few hundred kernels exist), filled with compare-and-swap
constexpr unsigned kKernelSlots = 4096;
std::atomic<const void*> g_lds_kernel[kKernelSlots];
std::atomic<uint64_t> g_lds_devices[kKernelSlots];
}  // namespace

int cu_count() {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0) {
        (void)hipGetLastError();  // no device: not an error the next call should see
        return 256;
    }
    std::atomic<int>& slot = g_cu_count[dev % kDeviceSlots];
    int n = slot.load(std::memory_order_relaxed);
    if (n > 0) return n;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1) {
        (void)hipGetLastError();
        return 256;
    }
    slot.store(n, std::memory_order_relaxed);
    return n;
}

hipError_t allow_lds(const void* fn, size_t lds_bytes) {
    if (lds_bytes <= 64 * 1024) return hipSuccess;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const uint64_t bit = (uint64_t)1 << (dev & 63);
    unsigned i = (unsigned)((reinterpret_cast<uintptr_t>(fn) >> 4) * 2654435761u) % kKernelSlots;
    for (unsigned probes = 0; probes < kKernelSlots; ++probes, i = (i + 1) % kKernelSlots) {
        const void* key = g_lds_kernel[i].load(std::memory_order_acquire);
        if (key == nullptr) {
            const void* expected = nullptr;
            if (g_lds_kernel[i].compare_exchange_strong(expected, fn, std::memory_order_acq_rel)) key = fn;
            else key = expected;
        }
        if (key != fn) continue;
        if (g_lds_devices[i].load(std::memory_order_acquire) & bit) return hipSuccess;
        e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e == hipSuccess) g_lds_devices[i].fetch_or(bit, std::memory_order_release);
        return e;
    }
    // table full (cannot happen with this library's kernel count): ask every time
    return hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
}

}  // namespace fwa

namespace {

inline bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

// Shape checks shared by forward, backward and the workspace query.
// Head width 32 everywhere; 64, 128 and 256 for L <= 64 (`wide_ok`: every forward and backward call).
int check_shape(int64_t N, int L, int C, int heads, int dtype, bool wide_ok) {
    if (N < 0 || L < 1 || C < 1 || heads < 1) return FWA_ERR_SHAPE;
    if (C % heads != 0) return FWA_ERR_SHAPE;
    if (dtype != FWA_F32 && dtype != FWA_BF16 && dtype != FWA_F16) return FWA_ERR_UNSUPPORTED;
    if (C / heads != fwa::kHeadDim &&
        !(wide_ok && fwa::forward_wide_supported(L, C / heads)))
        return FWA_ERR_UNSUPPORTED;
    // half data: the wide-head kernels only (head widths 64, 128, 256 at L <= 64)
    if (dtype == FWA_F16 && C / heads == fwa::kHeadDim) return FWA_ERR_UNSUPPORTED;
    if (L > fwa::kMaxL) return FWA_ERR_UNSUPPORTED;
    // one launch: the number of wave tasks (at most 4 per window-head) must fit a 32-bit grid.  The other grids
    // are bounded through the row stride: C <= 2^20 elements (check_row_stride) means at most 2^15 heads of
    // width 32, so the dBias reduction's heads * 16 * 16 * 4 workgroups stay below 2^25.
    if ((double)N * heads * 4.0 > 2.0e9) return FWA_ERR_UNSUPPORTED;
    return FWA_OK;
}

// The backward covers bf16 data in every shape of the forward, and fp32 data for windows of up to
// 64 tokens without dBias.
int check_backward_support(int L, int dtype, bool want_dbias) {
    if (dtype == FWA_F32 && (L > fwa::kMaxWideL || want_dbias)) return FWA_ERR_UNSUPPORTED;
    return FWA_OK;
}

// Row statistics the large-window backward leaves for its dBias kernel: [N, heads, 2, 16 nb] floats
size_t large_stats_bytes(int64_t N, int L, int heads) {
    const size_t nb = (size_t)(L + 15) / 16;
    return (size_t)N * heads * 2 * 16 * nb * sizeof(float);
}

// fp32 copy of a bf16 bias for the large-window backward, which reads the bias once per window and
// query block (a copy made once per call costs less than widening it at every use): [heads, L, L]
// floats, rounded up to 256 bytes
size_t large_bias_copy_bytes(int L, int heads) {
    return (((size_t)heads * L * L * sizeof(float)) + 255) & ~(size_t)255;
}

// Row stride of a strided tensor, in elements: at least C, rows 16-byte aligned, and small enough
// that the byte offsets inside one window fit 32 bits with room to spare.
int check_row_stride(int64_t ld, int C, int dtype) {
    const int64_t per16 = dtype == FWA_F32 ? 4 : 8;
    if (ld < C) return FWA_ERR_SHAPE;
    if (ld % per16 != 0) return FWA_ERR_ALIGN;
    if (ld > (int64_t)1 << 20) return FWA_ERR_UNSUPPORTED;
    return FWA_OK;
}

// A row-strided [N, L, C] tensor as the bytes it touches: rows of `width` bytes every `ld` bytes.
struct Span {
    uintptr_t base;
    uint64_t ld, width, rows;
    uintptr_t end() const { return base + (rows - 1) * ld + width; }
};
Span span_of(const void* p, int64_t N, int L, int C, int64_t ld, int dtype) {
    const uint64_t e = dtype == FWA_F32 ? 4 : 2;
    return Span{reinterpret_cast<uintptr_t>(p), (uint64_t)ld * e, (uint64_t)C * e, (uint64_t)N * (uint64_t)L};
}
// Whether two such tensors share a byte.  Tensors whose extents are disjoint do not.  With equal row
// strides (the views of one fused [N, L, 3, heads, d] buffer) the test is exact: rows interleave
// without touching iff the bases differ, modulo the stride, by at least a row width either way.
// Extents that intersect under different strides are reported as overlapping (conservative).
bool overlaps(const Span& a, const Span& b) {
    if (a.end() <= b.base || b.end() <= a.base) return false;
    if (a.ld != b.ld) return true;
    const uint64_t d = (a.base >= b.base ? a.base - b.base : b.base - a.base) % a.ld;
    return d < a.width || a.ld - d < a.width;
}

// The mask comes as a dense tile per window position or as region labels, never both.
int check_mask(int64_t N, const void* mask, const void* labels, int nW) {
    if (mask == nullptr && labels == nullptr) return FWA_OK;
    if (nW < 1 || N % nW != 0) return FWA_ERR_SHAPE;
    return FWA_OK;
}

int forward_impl(const void* q, const void* k, const void* v, void* o, int64_t N, int L, int C, int heads,
                 float scale, int64_t ld_qkv, int64_t ld_o, const void* bias, int bias_dtype, const float* mask,
                 const int32_t* labels, float mask_value, int nW, int dtype, void* stream) {
    int rc = check_shape(N, L, C, heads, dtype, true);
    if (rc != FWA_OK) return rc;
    if (bias && bias_dtype != FWA_F32 && bias_dtype != FWA_BF16) return FWA_ERR_UNSUPPORTED;
    rc = check_mask(N, mask, labels, nW);
    if (rc != FWA_OK) return rc;
    rc = check_row_stride(ld_qkv, C, dtype);
    if (rc != FWA_OK) return rc;
    rc = check_row_stride(ld_o, C, dtype);
    if (rc != FWA_OK) return rc;
    if (N == 0) return FWA_OK;
    if (!q || !k || !v || !o) return FWA_ERR_NULL;
    if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(o) || misaligned(bias) || misaligned(mask) ||
        misaligned(labels))
        return FWA_ERR_ALIGN;
    {
        const Span so = span_of(o, N, L, C, ld_o, dtype);
        const void* ins[3] = {q, k, v};
        for (const void* in : ins)
            if (overlaps(so, span_of(in, N, L, C, ld_qkv, dtype))) return FWA_ERR_ALIAS;
    }
    fwa::FwdArgs a;
    a.q = q; a.k = k; a.v = v; a.o = o;
    a.bias = bias; a.bias_bf16 = bias && bias_dtype == FWA_BF16;
    a.mask = mask; a.labels = labels; a.mask_value = mask_value;
    a.N = N; a.L = L; a.C = C; a.heads = heads; a.nW = (mask || labels) ? nW : 1; a.scale = scale;
    a.ldq = (int)ld_qkv; a.ldo = (int)ld_o; a.f16 = dtype == FWA_F16;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const bool wide = C / heads != fwa::kHeadDim;
    const hipError_t e = dtype == FWA_F32 ? (wide || L <= fwa::kMaxWideL ? fwa::launch_forward_f32_tile(a, st) : fwa::launch_forward_f32(a, st))
                                           : (wide ? fwa::launch_forward_bf16_wide(a, st) : fwa::launch_forward_bf16(a, st));
    return e == hipSuccess ? FWA_OK : FWA_ERR_LAUNCH;
}

int backward_impl(const void* q, const void* k, const void* v, const void* d_o, void* dq, void* dk, void* dv,
                  float* dbias, int64_t N, int L, int C, int heads, float scale, int64_t ld_qkv, int64_t ld_do,
                  int64_t ld_dqkv, const void* bias, int bias_dtype, const float* mask, const int32_t* labels,
                  float mask_value, int nW, int dtype, void* workspace, size_t workspace_bytes, void* stream,
                  bool static_scratch = false);

}  // namespace

extern "C" {

const char* fwa_status_string(int code) {
    switch (code) {
        case FWA_OK: return "ok";
        case FWA_ERR_NULL: return "a required pointer is NULL";
        case FWA_ERR_SHAPE: return "inconsistent shape arguments";
        case FWA_ERR_UNSUPPORTED: return "unsupported head dim, window length or dtype";
        case FWA_ERR_ALIGN: return "a base pointer is not 16-byte aligned";
        case FWA_ERR_WORKSPACE: return "workspace missing or too small";
        case FWA_ERR_LAUNCH: return "the HIP runtime refused the launch";
        case FWA_ERR_ALIAS: return "an output aliases another argument";
        default: return "unknown status code";
    }
}

int fwa_forward_strided(const void* q, const void* k, const void* v, void* o, int64_t N, int L, int C, int heads,
                        float scale, int64_t ld_qkv, int64_t ld_o, const float* bias, const float* mask, int nW,
                        int dtype, void* stream) {
    return forward_impl(q, k, v, o, N, L, C, heads, scale, ld_qkv, ld_o, bias, FWA_F32, mask, nullptr, 0.f, nW, dtype,
                        stream);
}

int fwa_forward_labels(const void* q, const void* k, const void* v, void* o, int64_t N, int L, int C, int heads,
                       float scale, int64_t ld_qkv, int64_t ld_o, const void* bias, int bias_dtype,
                       const int32_t* labels, float mask_value, int nW, int dtype, void* stream) {
    return forward_impl(q, k, v, o, N, L, C, heads, scale, ld_qkv, ld_o, bias, bias_dtype, nullptr, labels, mask_value,
                        nW, dtype, stream);
}

int fwa_forward(const void* q, const void* k, const void* v, void* o, int64_t N, int L, int C, int heads,
                float scale, const float* bias, const float* mask, int nW, int dtype, void* stream) {
    return fwa_forward_strided(q, k, v, o, N, L, C, heads, scale, C, C, bias, mask, nW, dtype, stream);
}

size_t fwa_backward_workspace_bytes(int64_t N, int L, int C, int heads, int dtype, int want_dbias) {
    if (check_shape(N, L, C, heads, dtype, true) != FWA_OK || check_backward_support(L, dtype, want_dbias != 0) != FWA_OK)
        return 0;
    if (N == 0) return 0;
    // the slot count depends on the mask period; this is its upper bound over all periods
    const size_t nb = (size_t)(L + 15) / 16;  // partial sums are kept per 16 x 16 block, padded
    if (L > fwa::kMaxBackwardL) {
        // room for the fp32 copy of a bf16 bias whether or not the call will pass one
        const size_t copy = large_bias_copy_bytes(L, heads);
        if (!want_dbias) return copy;
        return copy + large_stats_bytes(N, L, heads) +
               (size_t)fwa::backward_large_slots(N, heads, L) * heads * nb * nb * 256 * sizeof(float);
    }
    if (!want_dbias) return 0;
    return (size_t)fwa::backward_max_slots(N, heads) * heads * nb * nb * 256 * sizeof(float);
}

int fwa_backward_strided(const void* q, const void* k, const void* v, const void* d_o, void* dq, void* dk, void* dv,
                         float* dbias, int64_t N, int L, int C, int heads, float scale, int64_t ld_qkv,
                         int64_t ld_do, int64_t ld_dqkv, const float* bias, const float* mask, int nW, int dtype,
                         void* workspace, size_t workspace_bytes, void* stream) {
    return backward_impl(q, k, v, d_o, dq, dk, dv, dbias, N, L, C, heads, scale, ld_qkv, ld_do, ld_dqkv, bias, FWA_F32,
                         mask, nullptr, 0.f, nW, dtype, workspace, workspace_bytes, stream);
}

int fwa_backward_labels(const void* q, const void* k, const void* v, const void* d_o, void* dq, void* dk, void* dv,
                        float* dbias, int64_t N, int L, int C, int heads, float scale, int64_t ld_qkv,
                        int64_t ld_do, int64_t ld_dqkv, const void* bias, int bias_dtype, const int32_t* labels,
                        float mask_value, int nW, int dtype, void* workspace, size_t workspace_bytes, void* stream) {
    return backward_impl(q, k, v, d_o, dq, dk, dv, dbias, N, L, C, heads, scale, ld_qkv, ld_do, ld_dqkv, bias, bias_dtype,
                         nullptr, labels, mask_value, nW, dtype, workspace, workspace_bytes, stream);
}

}  // extern "C"

namespace {

// Scratch of fwa_backward_noalloc: the workspace of a backward call, held by the library itself so
// that the call allocates nothing.  Every device the library runs on holds its own copy of the
// array until the process ends; host code must address it through the pointer the runtime reports
// for the current device, never through the array's name.
__device__ __attribute__((used)) __align__(256) unsigned char scratch[FWA_NOALLOC_SCRATCH_BYTES];
std::atomic<void*> g_scratch_ptr[64];  // per device; nullptr = not asked yet

void* scratch_of_current_device() {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return nullptr;
    void* ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (ptr != nullptr) return ptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) return nullptr;
    g_scratch_ptr[dev].store(ptr, std::memory_order_release);
    return ptr;
}

int backward_impl(const void* q, const void* k, const void* v, const void* d_o, void* dq, void* dk, void* dv,
                  float* dbias, int64_t N, int L, int C, int heads, float scale, int64_t ld_qkv, int64_t ld_do,
                  int64_t ld_dqkv, const void* bias, int bias_dtype, const float* mask, const int32_t* labels,
                  float mask_value, int nW, int dtype, void* workspace, size_t workspace_bytes, void* stream,
                  bool static_scratch) {
    int rc = check_shape(N, L, C, heads, dtype, true);
    if (rc != FWA_OK) return rc;
    if (bias && bias_dtype != FWA_F32 && bias_dtype != FWA_BF16) return FWA_ERR_UNSUPPORTED;
    rc = check_row_stride(ld_qkv, C, dtype);
    if (rc != FWA_OK) return rc;
    rc = check_row_stride(ld_do, C, dtype);
    if (rc != FWA_OK) return rc;
    rc = check_row_stride(ld_dqkv, C, dtype);
    if (rc != FWA_OK) return rc;
    rc = check_backward_support(L, dtype, dbias != nullptr);
    if (rc != FWA_OK) return rc;
    rc = check_mask(N, mask, labels, nW);
    if (rc != FWA_OK) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (N == 0) {
        // the sum over zero windows: dbias is still "overwritten"
        if (dbias) {
            if (misaligned(dbias)) return FWA_ERR_ALIGN;
            if (fwa::launch_zero_f32(dbias, (size_t)heads * L * L, st) != hipSuccess) return FWA_ERR_LAUNCH;
        }
        return FWA_OK;
    }
    if (!q || !k || !v || !d_o || !dq || !dk || !dv) return FWA_ERR_NULL;
    if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(d_o) || misaligned(dq) || misaligned(dk) ||
        misaligned(dv) || misaligned(dbias) || misaligned(bias) || misaligned(mask) || misaligned(labels) ||
        misaligned(workspace))
        return FWA_ERR_ALIGN;
    {
        const Span ins[4] = {span_of(q, N, L, C, ld_qkv, dtype), span_of(k, N, L, C, ld_qkv, dtype),
                             span_of(v, N, L, C, ld_qkv, dtype), span_of(d_o, N, L, C, ld_do, dtype)};
        const Span outs[3] = {span_of(dq, N, L, C, ld_dqkv, dtype), span_of(dk, N, L, C, ld_dqkv, dtype),
                              span_of(dv, N, L, C, ld_dqkv, dtype)};
        for (int a = 0; a < 3; ++a) {
            for (int b = 0; b < 4; ++b)
                if (overlaps(outs[a], ins[b])) return FWA_ERR_ALIAS;
            for (int b = a + 1; b < 3; ++b)
                if (overlaps(outs[a], outs[b])) return FWA_ERR_ALIAS;
        }
        if (dbias) {  // one contiguous row of heads * L * L floats
            const uint64_t bytes = (uint64_t)heads * L * L * sizeof(float);
            const Span sd = Span{reinterpret_cast<uintptr_t>(dbias), bytes, bytes, 1};
            for (int b = 0; b < 4; ++b)
                if (overlaps(sd, ins[b])) return FWA_ERR_ALIAS;
            for (int b = 0; b < 3; ++b)
                if (overlaps(sd, outs[b])) return FWA_ERR_ALIAS;
            const uint64_t bias_bytes = bias_dtype == FWA_BF16 ? bytes / 2 : bytes;
            if (bias && overlaps(sd, Span{reinterpret_cast<uintptr_t>(bias), bias_bytes, bias_bytes, 1})) return FWA_ERR_ALIAS;
        }
    }
    fwa::BwdArgs a;
    a.q = q; a.k = k; a.v = v; a.d_o = d_o;
    a.dq = dq; a.dk = dk; a.dv = dv; a.dbias = dbias;
    a.mask = mask; a.labels = labels; a.mask_value = mask_value;
    a.N = N; a.L = L; a.C = C; a.heads = heads; a.nW = (mask || labels) ? nW : 1; a.scale = scale;
    // A mask period that no slot count of the cooperative kernel is a multiple of: with the mask as
    // labels the kernel forms each window's mask itself and its workgroups walk the windows as if
    // there were no period; with a dense mask the one-wave-per-tile kernel takes the call.
    const bool large = L > fwa::kMaxBackwardL;
    const bool small = dtype == FWA_BF16 && C / heads == fwa::kHeadDim && !large;
    a.per_window = small && labels && fwa::coop_slots(N, heads, a.nW) == 0 && fwa::coop_slots(N, heads, 1) > 0;
    a.slots = C / heads != fwa::kHeadDim ? fwa::backward_wide_slots(N, heads)
              : large                    ? fwa::backward_large_slots(N, heads, L)
                                         : fwa::backward_slots(N, heads, a.per_window ? 1 : a.nW);
    // workspace: [fp32 copy of a bf16 bias (large windows only)] [row statistics (large windows
    // with dBias)] [partial sums of dBias]; a call needs the parts it uses
    const bool copy_bias = large && bias && bias_dtype == FWA_BF16;
    const size_t copy_room = large ? large_bias_copy_bytes(L, heads) : 0;
    if (static_scratch) {
        // the parts at their exact sizes for this call, out of the library's own array
        const size_t nb = (size_t)(L + 15) / 16;
        const size_t exact = (copy_bias ? copy_room : 0) + (dbias && large ? large_stats_bytes(N, L, heads) : 0) +
                             (dbias ? (size_t)a.slots * heads * nb * nb * 256 * sizeof(float) : 0);
        if (exact > FWA_NOALLOC_SCRATCH_BYTES) return FWA_ERR_WORKSPACE;
        workspace = nullptr;
        if (exact > 0) {
            workspace = scratch_of_current_device();
            if (workspace == nullptr) return FWA_ERR_LAUNCH;
        }
    } else {
        const size_t full = fwa_backward_workspace_bytes(N, L, C, heads, dtype, dbias != nullptr);
        const size_t need = (dbias ? full - copy_room : 0) + (copy_bias ? copy_room : 0);
        if (need > 0 && (workspace == nullptr || workspace_bytes < need)) return FWA_ERR_WORKSPACE;
    }
    char* ws = static_cast<char*>(workspace);
    if (copy_bias) {
        if (fwa::launch_widen_bf16(bias, reinterpret_cast<float*>(ws), (size_t)heads * L * L, st) != hipSuccess)
            return FWA_ERR_LAUNCH;
        bias = ws;
        bias_dtype = FWA_F32;
        ws += copy_room;
    }
    a.partial = dbias ? reinterpret_cast<float*>(ws) : nullptr;
    a.stats = nullptr;
    if (dbias && large) {  // [row statistics][partial sums]
        a.stats = reinterpret_cast<float*>(ws);
        a.partial = reinterpret_cast<float*>(ws + large_stats_bytes(N, L, heads));
    }
    a.bias = bias; a.bias_bf16 = bias && bias_dtype == FWA_BF16;
    a.ldq = (int)ld_qkv; a.ldg = (int)ld_do; a.ldd = (int)ld_dqkv; a.f16 = dtype == FWA_F16;
    // the one-wave-per-tile kernel takes fp32 biases only
    if (a.bias_bf16 && small && !a.per_window && fwa::coop_slots(N, heads, a.nW) == 0)
        return FWA_ERR_UNSUPPORTED;
    const hipError_t e = dtype != FWA_F32 ? fwa::launch_backward_bf16(a, st) : fwa::launch_backward_f32(a, st);
    return e == hipSuccess ? FWA_OK : FWA_ERR_LAUNCH;
}

}  // namespace

extern "C" {

int fwa_backward(const void* q, const void* k, const void* v, const void* d_o, void* dq, void* dk, void* dv,
                 float* dbias, int64_t N, int L, int C, int heads, float scale, const float* bias,
                 const float* mask, int nW, int dtype, void* workspace, size_t workspace_bytes, void* stream) {
    return fwa_backward_strided(q, k, v, d_o, dq, dk, dv, dbias, N, L, C, heads, scale, C, C, C, bias, mask, nW,
                                dtype, workspace, workspace_bytes, stream);
}

int fwa_backward_noalloc(const void* q, const void* k, const void* v, const void* d_o, void* dq, void* dk, void* dv,
                         float* dbias, int64_t N, int L, int C, int heads, float scale, const float* bias,
                         const float* mask, int nW, int dtype, void* stream) {
    return backward_impl(q, k, v, d_o, dq, dk, dv, dbias, N, L, C, heads, scale, C, C, C, bias, FWA_F32, mask, nullptr,
                         0.f, nW, dtype, nullptr, 0, stream, true);
}

int fwa_bias_gather(const float* table, float* bias, int heads, int k, void* stream) {
    if (heads < 1 || k < 1) return FWA_ERR_SHAPE;
    if (k > 16) return FWA_ERR_UNSUPPORTED;
    if (!table || !bias) return FWA_ERR_NULL;
    if (misaligned(table) || misaligned(bias)) return FWA_ERR_ALIGN;
    if (table == bias) return FWA_ERR_ALIAS;
    return fwa::launch_bias_gather(table, bias, heads, k, static_cast<hipStream_t>(stream)) == hipSuccess
               ? FWA_OK : FWA_ERR_LAUNCH;
}

int fwa_bias_scatter(const float* dbias, float* dtable, int heads, int k, void* stream) {
    if (heads < 1 || k < 1) return FWA_ERR_SHAPE;
    if (k > 16) return FWA_ERR_UNSUPPORTED;
    if (!dbias || !dtable) return FWA_ERR_NULL;
    if (misaligned(dbias) || misaligned(dtable)) return FWA_ERR_ALIGN;
    if (dbias == dtable) return FWA_ERR_ALIAS;
    return fwa::launch_bias_scatter(dbias, dtable, heads, k, static_cast<hipStream_t>(stream)) == hipSuccess
               ? FWA_OK : FWA_ERR_LAUNCH;
}

}  // extern "C"
