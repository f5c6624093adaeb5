// Relative-position bias helpers: table [heads, (2k-1)^2] <-> bias [heads, L, L].
// Pure index work (the paper defers to Swin Transformer for the bias; this is
// that published indexing): pair (i, j) of a k x k window reads table column
// (y_i - y_j + k - 1) * (2k - 1) + (x_i - x_j + k - 1).
#include "fwa_internal.h"

namespace fwa {
namespace {

__global__ void bias_gather_kernel(const float* __restrict__ table, float* __restrict__ bias, int heads, int k) {
    const int L = k * k, T = (2 * k - 1) * (2 * k - 1);
    const long long total = (long long)heads * L * L;
    for (long long e = (long long)blockIdx.x * blockDim.x + threadIdx.x; e < total;
         e += (long long)gridDim.x * blockDim.x) {
        const int j = (int)(e % L);
        const int i = (int)((e / L) % L);
        const int h = (int)(e / ((long long)L * L));
        const int dy = i / k - j / k + k - 1;
        const int dx = i % k - j % k + k - 1;
        bias[e] = table[(size_t)h * T + dy * (2 * k - 1) + dx];
    }
}

// One thread per table entry; it adds its (k-|dy|)(k-|dx|) contributions in a
// fixed order, so the result is bit-reproducible.
__global__ void bias_scatter_kernel(const float* __restrict__ dbias, float* __restrict__ dtable, int heads, int k) {
    const int L = k * k, W = 2 * k - 1, T = W * W;
    const int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= heads * T) return;
    const int h = e / T;
    const int dy = (e % T) / W - (k - 1);
    const int dx = (e % T) % W - (k - 1);
    const float* src = dbias + (size_t)h * L * L;
    float acc = 0.f;
    for (int yi = max(0, dy); yi < min(k, k + dy); ++yi)
        for (int xi = max(0, dx); xi < min(k, k + dx); ++xi) {
            const int i = yi * k + xi;
            const int j = (yi - dy) * k + (xi - dx);
            acc += src[(size_t)i * L + j];
        }
    dtable[e] = acc;
}

__global__ void zero_f32_kernel(float* __restrict__ dst, size_t count) {
    for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < count; e += (size_t)gridDim.x * blockDim.x)
        dst[e] = 0.f;
}

// bf16 -> fp32 (exact: the 16 bits become the upper half of the word)
__global__ void widen_bf16_kernel(const uint16_t* __restrict__ src, float* __restrict__ dst, size_t count) {
    for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < count; e += (size_t)gridDim.x * blockDim.x)
        dst[e] = __builtin_bit_cast(float, (uint32_t)src[e] << 16);
}

}  // namespace

hipError_t launch_widen_bf16(const void* src, float* dst, size_t count, hipStream_t s) {
    const size_t blocks = (count + 255) / 256;
    hipLaunchKernelGGL(widen_bf16_kernel, dim3((unsigned)(blocks > 1024 ? 1024 : blocks)), dim3(256), 0, s,
                       static_cast<const uint16_t*>(src), dst, count);
    return hipGetLastError();
}

// A fill kernel rather than a memset node, so that callers may capture it in a graph.
hipError_t launch_zero_f32(float* dst, size_t count, hipStream_t s) {
    const size_t blocks = (count + 255) / 256;
    hipLaunchKernelGGL(zero_f32_kernel, dim3((unsigned)(blocks > 1024 ? 1024 : blocks)), dim3(256), 0, s, dst, count);
    return hipGetLastError();
}

hipError_t launch_bias_gather(const float* table, float* bias, int heads, int k, hipStream_t s) {
    const long long total = (long long)heads * k * k * k * k;
    const unsigned grid = (unsigned)((total + 255) / 256 > 4096 ? 4096 : (total + 255) / 256);
    hipLaunchKernelGGL(bias_gather_kernel, dim3(grid), dim3(256), 0, s, table, bias, heads, k);
    return hipGetLastError();
}

hipError_t launch_bias_scatter(const float* dbias, float* dtable, int heads, int k, hipStream_t s) {
    const int total = heads * (2 * k - 1) * (2 * k - 1);
    hipLaunchKernelGGL(bias_scatter_kernel, dim3((total + 127) / 128), dim3(128), 0, s, dbias, dtable, heads, k);
    return hipGetLastError();
}

}  // namespace fwa
