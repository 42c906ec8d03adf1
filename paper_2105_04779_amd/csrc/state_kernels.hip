// State maintenance between decode steps: gather of whole batch elements of H (section 3.1.1: the
// state EL-attention keeps is the hidden states themselves; Algorithm 3 leaves re-ordering it after a
// beam-search step, and dropping finished sentences, to the caller).  Pure data movement, bound by HBM:
// every valid row is read once and written once, 16 bytes per lane, rows at or beyond the element's
// length are neither read nor written.
#include <cstdint>
#include "el_internal.h"

namespace el {

typedef unsigned int u4v __attribute__((ext_vector_type(4)));

// grid: (row chunks, B_dst).  A workgroup copies kRowsPerBlock consecutive rows of one destination element.
constexpr int kRowsPerBlock = 32;

__global__ void __launch_bounds__(256)
k_gather_batch(const char *__restrict__ src, int64_t src_stride_b, const int32_t *__restrict__ len_src, int B_src,
               char *__restrict__ dst, int64_t dst_stride_b, int32_t *__restrict__ len_dst,
               const int32_t *__restrict__ index, int n, int row_bytes)
{
    const int i = blockIdx.y;
    const int from = index[i];
    const bool ok = from >= 0 && from < B_src;
    int len = 0;
    if (ok) { len = len_src ? len_src[from] : n; len = min(max(len, 0), n); }
    if (blockIdx.x == 0 && threadIdx.x == 0 && len_dst) len_dst[i] = len;
    const int r0 = blockIdx.x * kRowsPerBlock;
    if (r0 >= len) return;
    const int rows = min(kRowsPerBlock, len - r0);
    // the rows of one element are contiguous: one flat 16-byte-granular copy of rows * row_bytes bytes
    const u4v *s = (const u4v *)(src + (size_t)from * src_stride_b + (size_t)r0 * row_bytes);
    u4v *d = (u4v *)(dst + (size_t)i * dst_stride_b + (size_t)r0 * row_bytes);
    const int chunks = rows * (row_bytes >> 4);
    int c = threadIdx.x;
    // four independent loads in flight per lane
    for (; c + 3 * 256 < chunks; c += 4 * 256) {
        const u4v a = s[c], b = s[c + 256], e = s[c + 512], f = s[c + 768];
        d[c] = a; d[c + 256] = b; d[c + 512] = e; d[c + 768] = f;
    }
    for (; c < chunks; c += 256) d[c] = s[c];
}

} // namespace el

extern "C" el_status el_attn_gather_batch(el_dtype dtype, int32_t d_model,
                                          const void *H_src, int64_t src_batch_stride, const int32_t *lengths_src, int32_t B_src,
                                          void *H_dst, int64_t dst_batch_stride, int32_t *lengths_dst, int32_t B_dst,
                                          const int32_t *index, int32_t n, void *stream)
{
    if (!H_src || !H_dst || !index) return EL_ERR_INVALID_ARG;
    if (dtype != EL_F32 && dtype != EL_F16 && dtype != EL_BF16) return EL_ERR_INVALID_ARG;
    if (d_model < 1 || B_src < 1 || B_dst < 1 || n < 1) return EL_ERR_INVALID_ARG;
    const int64_t es = (int64_t)el::dtype_size(dtype);
    const int64_t row_bytes = (int64_t)d_model * es;
    if (row_bytes % 16 != 0 || row_bytes > (1 << 30)) return EL_ERR_INVALID_ARG;
    if (src_batch_stride < (int64_t)n * d_model || dst_batch_stride < (int64_t)n * d_model) return EL_ERR_INVALID_ARG;
    if (((uintptr_t)H_src | (uintptr_t)H_dst) & 15) return EL_ERR_INVALID_ARG;
    if ((src_batch_stride * es) % 16 != 0 || (dst_batch_stride * es) % 16 != 0) return EL_ERR_INVALID_ARG;
    if (B_dst > 65535) return EL_ERR_INVALID_ARG;      // grid.y
    const dim3 grid((n + el::kRowsPerBlock - 1) / el::kRowsPerBlock, B_dst), block(256);
    hipLaunchKernelGGL(el::k_gather_batch, grid, block, 0, (hipStream_t)stream,
                       (const char *)H_src, src_batch_stride * es, lengths_src, B_src,
                       (char *)H_dst, dst_batch_stride * es, lengths_dst, index, n, (int)row_bytes);
    return hipGetLastError() == hipSuccess ? EL_OK : EL_ERR_HIP;
}
