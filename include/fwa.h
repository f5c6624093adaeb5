/*
 * fwa.h -- C ABI of the Flash Window Attention library for AMD MI355X (gfx950).
 *
 * The library computes fused, batched short-sequence attention over
 * window-partitioned tensors (paper Section 2.1, eq. 1-4):
 *
 *     O[n, :, head h] = softmax(scale * Q_nh K_nh^T + B[h] + M[n mod nW]) V_nh
 *
 * with the whole L x L score/probability tile kept on chip and Q, K, V, O
 * crossing device memory exactly once (paper Algorithm 1), and its backward
 * (paper Algorithm 2) which recomputes P on chip and needs nothing saved from
 * the forward.  The paper's equations carry no scale, bias or mask; they are
 * additive extensions: scale multiplies QK^T before B and M are added.
 *
 * Conventions shared by every entry point
 * ---------------------------------------
 *  - Every pointer is a DEVICE pointer owned by the caller.  The library
 *    never allocates, frees or synchronises; it enqueues kernels on `stream`
 *    (a hipStream_t passed as void*; NULL = the default stream) and returns.
 *  - Tensors are contiguous, row-major.  Q, K, V, O, dO, dQ, dK, dV are
 *    [N, L, C]; head h owns channels [h*d, (h+1)*d) with d = C / heads.
 *    Supported: d == 32 with 1 <= L <= 256; d == 64, 128, 256 with
 *    1 <= L <= 64 (the feature-dimension loop of paper eq. 5-6; the shapes of
 *    its Section 3.1 benchmark), in fp32 and bf16 (half: the wider heads only,
 *    see dtype).  N >= 0 (N == 0 is a no-op).
 *  - dtype is FWA_F32 (fp32 data, fp32 arithmetic), FWA_BF16 (bf16 data,
 *    bf16 matrix-core products with fp32 accumulation, fp32 softmax, one final
 *    round-to-nearest-even to bf16) or FWA_F16 (IEEE half data, handled like
 *    bf16 with half products; head widths 64, 128 and 256 only, i.e. the
 *    shapes and the precision of the paper's Section 3 comparisons;
 *    FWA_ERR_UNSUPPORTED at head width 32).  With half data every intermediate
 *    that enters a matrix product -- P, dS -- must stay inside the half range.
 *  - mask and dbias are always fp32; bias is fp32, or bf16 through the
 *    *_labels entry points (bias_dtype).
 *  - Base pointers must be 16-byte aligned.  No output may share a byte with an
 *    input or with another output (FWA_ERR_ALIAS).  For row-strided tensors of
 *    one stride -- the q/k/v or dq/dk/dv views of one fused buffer -- the test is
 *    exact: rows may interleave.  Tensors of different strides whose address
 *    extents intersect are rejected even if their rows happen not to touch.
 *  - The return value is FWA_OK or an error code; on error nothing has been
 *    launched.
 *  - Calls are thread-safe.  The only state the library keeps is per kernel and
 *    device, behind atomics: whether the runtime has been told that the kernel
 *    may use more than 64 KB of LDS (hipFuncSetAttribute), how many of its
 *    workgroups fit a compute unit, and the device's compute-unit count.  These
 *    are asked on the first call that needs them, so a caller that records calls
 *    into a HIP graph makes one call of the same shape outside the capture first.
 *    (fwa_backward_noalloc also shares one scratch array per device: see there.)
 */
#ifndef FWA_H
#define FWA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { FWA_F32 = 0, FWA_BF16 = 1, FWA_F16 = 2 };

enum {
    FWA_OK = 0,
    FWA_ERR_NULL = 1,        /* a required pointer is NULL                          */
    FWA_ERR_SHAPE = 2,       /* negative N, L < 1, C % heads != 0, N % nW != 0, ... */
    FWA_ERR_UNSUPPORTED = 3, /* head dim, L, dtype or dbias outside the ranges above */
    FWA_ERR_ALIGN = 4,       /* a base pointer is not 16-byte aligned               */
    FWA_ERR_WORKSPACE = 5,   /* workspace missing or smaller than required          */
    FWA_ERR_LAUNCH = 6,      /* the HIP runtime refused the launch                  */
    FWA_ERR_ALIAS = 7        /* an output shares memory with another argument       */
};

/*
 * Forward pass (paper Algorithm 1; eq. 2-4).
 *   q, k, v : in,  [N, L, C], dtype
 *   o       : out, [N, L, C], dtype, fully overwritten
 *   bias    : NULL, or in [heads, L, L] fp32 (already gathered per token pair)
 *   mask    : NULL, or in [nW, L, L] fp32, added to the scores of window n as
 *             mask[n % nW]; requires nW >= 1 and N % nW == 0.  nW is ignored
 *             when mask is NULL.
 */
int fwa_forward(const void* q, const void* k, const void* v, void* o,
                int64_t N, int L, int C, int heads, float scale,
                const float* bias, const float* mask, int nW,
                int dtype, void* stream);

/*
 * The same with row strides: token row (n, l) of q, k and v starts ld_qkv elements after row
 * (n, l) - 1 (window n begins at row n*L), and likewise ld_o for o; ld == C is the contiguous
 * case above.  This reads Q, K, V in place out of a fused projection output [N, L, 3, heads, d]
 * (q = base, k = base + C, v = base + 2C elements, ld_qkv = 3C), saving the permute and copy in
 * front of the kernel.  Strides must be >= C and keep rows 16-byte aligned (FWA_ERR_SHAPE /
 * FWA_ERR_ALIGN otherwise).
 */
int fwa_forward_strided(const void* q, const void* k, const void* v, void* o,
                        int64_t N, int L, int C, int heads, float scale,
                        int64_t ld_qkv, int64_t ld_o,
                        const float* bias, const float* mask, int nW,
                        int dtype, void* stream);

/*
 * Backward pass (paper Algorithm 2).  Inputs are Q, K, V and dO only.
 * Supported: FWA_BF16 and FWA_F16 in every shape the forward takes them;
 * FWA_F32 for L <= 64 without dbias (FWA_ERR_UNSUPPORTED otherwise).
 *   d_o        : in,  [N, L, C], dtype
 *   dq, dk, dv : out, [N, L, C], dtype, fully overwritten
 *   dbias      : NULL, or out [heads, L, L] fp32 = sum over all N windows of
 *                dS; overwritten, not accumulated.  The mask gets no gradient.
 *   workspace  : device scratch of at least fwa_backward_workspace_bytes(...)
 *                bytes, 16-byte aligned.  It holds per-workgroup partial sums
 *                of dbias and, for L > 64, the softmax statistics of every row
 *                and the fp32 copy of a bf16 bias (fwa_backward_labels).  It
 *                may be NULL when dbias is NULL, unless L > 64 and the bias is
 *                bf16.  Contents on entry are ignored and undefined on exit.
 * Results are bit-reproducible from run to run for fixed arguments.
 */
int fwa_backward(const void* q, const void* k, const void* v, const void* d_o,
                 void* dq, void* dk, void* dv, float* dbias,
                 int64_t N, int L, int C, int heads, float scale,
                 const float* bias, const float* mask, int nW,
                 int dtype, void* workspace, size_t workspace_bytes, void* stream);

/* The same with row strides (see fwa_forward_strided): ld_qkv for q, k, v; ld_do for d_o;
 * ld_dqkv for dq, dk, dv, so that the three gradients can be written straight into a fused
 * [N, L, 3, heads, d] gradient buffer. */
int fwa_backward_strided(const void* q, const void* k, const void* v, const void* d_o,
                         void* dq, void* dk, void* dv, float* dbias,
                         int64_t N, int L, int C, int heads, float scale,
                         int64_t ld_qkv, int64_t ld_do, int64_t ld_dqkv,
                         const float* bias, const float* mask, int nW,
                         int dtype, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Forward and backward with the shift mask given as region labels instead of a dense tile,
 * and optionally a bf16 bias
 * (paper Section 2.1: shifted blocks mask attention between tokens that were not neighbours
 * before the cyclic shift; the labels name the regions of the shifted token map):
 *   labels     : NULL (no mask), or in [nW, L] int32; the scores of window n receive
 *                M[i][j] = labels[n % nW][i] == labels[n % nW][j] ? 0 : mask_value,
 *                formed inside the kernels.  This reads L * 4 bytes per window position
 *                instead of L * L * 4.  Requires nW >= 1 and N % nW == 0; 16-byte aligned.
 *   mask_value : what a pair of tokens with different labels adds to its score (-100 in
 *                the Swin Transformer); ignored when labels is NULL.
 *   bias       : NULL, or in [heads, L, L] of type bias_dtype: FWA_F32 as everywhere else, or
 *                FWA_BF16 (half the bytes; the values are used as they are, i.e. the result is
 *                that of the fp32 call on the same values).  dbias stays fp32.
 * Everything else (shapes, strides, dtype, workspace, error codes, supported ranges) is as in
 * fwa_forward_strided / fwa_backward_strided, and the results are those of the same call with
 * the dense mask written out from the labels: bit for bit while nW is small enough for a
 * workgroup to keep one mask tile for life (nW <= 256 / heads-per-workgroup, roughly), and to
 * within a rounding of the additive term beyond, where the dense form falls back to slower
 * kernels and this form does not (each window's mask is formed from its labels).
 */
int fwa_forward_labels(const void* q, const void* k, const void* v, void* o,
                       int64_t N, int L, int C, int heads, float scale,
                       int64_t ld_qkv, int64_t ld_o,
                       const void* bias, int bias_dtype, const int32_t* labels, float mask_value, int nW,
                       int dtype, void* stream);

int fwa_backward_labels(const void* q, const void* k, const void* v, const void* d_o,
                        void* dq, void* dk, void* dv, float* dbias,
                        int64_t N, int L, int C, int heads, float scale,
                        int64_t ld_qkv, int64_t ld_do, int64_t ld_dqkv,
                        const void* bias, int bias_dtype, const int32_t* labels, float mask_value, int nW,
                        int dtype, void* workspace, size_t workspace_bytes, void* stream);

/*
 * fwa_backward for callers that cannot allocate: code under HIP graph capture, serving loops,
 * harnesses that forbid hipMalloc.  It is fwa_backward without the workspace arguments: the
 * workspace (dBias partial sums; for L > 64 also the row statistics) lives in an array of
 * FWA_NOALLOC_SCRATCH_BYTES bytes inside the library's code object, of which every device the
 * library runs on holds its own copy until the process ends.  The call itself allocates and frees
 * nothing, and runs the same kernels with the same results, bit for bit, as fwa_backward.
 *   - A call whose workspace would exceed the array returns FWA_ERR_WORKSPACE.  Every bf16 call
 *     with L <= 64 and head width 32 fits (at most 3 x compute-units tiles of 16 KB = 12 MiB);
 *     large windows with dbias mostly do not.  Without dbias no scratch is used at all.
 *   - All calls on one device share that device's array, which keeps the previous call's contents;
 *     the kernels overwrite every element they later read, so nothing needs clearing.  Calls that
 *     overlap in time on one device (two streams, two threads) race on it: serialise them.
 *   - The array's device address is looked up on the first call on each device
 *     (hipGetSymbolAddress, no allocation).
 */
#define FWA_NOALLOC_SCRATCH_BYTES (16u * 1024u * 1024u)
int fwa_backward_noalloc(const void* q, const void* k, const void* v, const void* d_o,
                         void* dq, void* dk, void* dv, float* dbias,
                         int64_t N, int L, int C, int heads, float scale,
                         const float* bias, const float* mask, int nW,
                         int dtype, void* stream);

/* Bytes of workspace that suffice for any backward call with these arguments
 * (0 if none is needed; for L > 64 the size includes room for the fp32 copy of
 * a bf16 bias whether or not one will be passed).  Returns 0 for arguments
 * fwa_backward would reject. */
size_t fwa_backward_workspace_bytes(int64_t N, int L, int C, int heads, int dtype, int want_dbias);

/*
 * Relative-position bias helpers for k x k windows (L = k*k).  Token i sits
 * at (i / k, i % k); pair (i, j) maps to table column
 * (y_i - y_j + k - 1) * (2k - 1) + (x_i - x_j + k - 1).  The paper only says
 * its baseline follows Swin Transformer; this is that published indexing.
 *   fwa_bias_gather : table [heads, (2k-1)^2] -> bias [heads, L, L]
 *   fwa_bias_scatter: dbias [heads, L, L] -> dtable [heads, (2k-1)^2]
 *                     (adjoint of the gather; overwritten; fixed summation
 *                     order, bit-reproducible)
 * All fp32 device pointers.  Requires heads >= 1 and 1 <= k <= 16.
 */
int fwa_bias_gather(const float* table, float* bias, int heads, int k, void* stream);
int fwa_bias_scatter(const float* dbias, float* dtable, int heads, int k, void* stream);

/* Static, NUL-terminated description of an error code. */
const char* fwa_status_string(int code);

#ifdef __cplusplus
}
#endif
#endif /* FWA_H */
