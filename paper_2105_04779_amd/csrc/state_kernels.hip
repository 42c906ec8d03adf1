// Context-free passes over the hidden states.
// (1) State maintenance between decode steps: gather of whole batch elements of H (section 3.1.1: the
// state EL-attention keeps is the hidden states themselves; Algorithm 3 leaves re-ordering it after a
// beam-search step, and dropping finished sentences, to the caller).  Pure data movement, bound by HBM:
// every valid row is read once and written once, 16 bytes per lane, rows at or beyond the element's
// length are neither read nor written.
// (2) Input check: what the decode step assumes about its inputs and does not verify on the hot path (lengths
// inside [1, n]; finite hidden states; in the 16-bit MFMA path, magnitudes inside the fp16 range, since bf16
// operands are converted to fp16), counted in one read of the valid rows.
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

// ---------------------------------------------------------------------------------------------
__global__ void k_zero_report(unsigned long long *report)
{
    if (threadIdx.x < 4) report[threadIdx.x] = 0ull;
}

// non-finite / beyond the fp16 range (finite, |v| > 65504), from the raw bits of a value widened to fp32 layout
__device__ __forceinline__ unsigned is_nonfinite32(unsigned u) { return (u & 0x7fffffffu) >= 0x7f800000u ? 1u : 0u; }
__device__ __forceinline__ unsigned is_large32(unsigned u)
{
    const unsigned mag = u & 0x7fffffffu;
    return (mag > 0x477fe000u && mag < 0x7f800000u) ? 1u : 0u;     // 0x477fe000 = 65504.0f
}

constexpr int kRowsPerCheckBlock = 128;

// grid: (row chunks, B).  report[0] lengths outside [1, n]; [1] non-finite elements; [2] finite elements beyond
// the fp16 range; [3] elements examined.  Rows at or beyond the (clamped) length are not read.
template <int DT>
__global__ void __launch_bounds__(256)
k_check_inputs(const char *__restrict__ H, int64_t stride_b, const int32_t *__restrict__ lengths, int n,
               int row_bytes, unsigned long long *__restrict__ report)
{
    const int b = blockIdx.y;
    const int raw = lengths ? lengths[b] : n;
    if (blockIdx.x == 0 && threadIdx.x == 0 && (raw < 1 || raw > n)) atomicAdd(&report[0], 1ull);
    const int len = min(max(raw, 0), n);
    const int r0 = blockIdx.x * kRowsPerCheckBlock;
    if (r0 >= len) return;
    const int rows = min(kRowsPerCheckBlock, len - r0);
    const u4v *s = (const u4v *)(H + (size_t)b * stride_b + (size_t)r0 * row_bytes);
    const int chunks = rows * (row_bytes >> 4);
    unsigned nonfinite = 0, large = 0;
    auto word = [&](unsigned x) {
        if (DT == EL_F32) { nonfinite += is_nonfinite32(x); large += is_large32(x); }
        else if (DT == EL_BF16) {
            nonfinite += is_nonfinite32(x << 16) + is_nonfinite32(x & 0xffff0000u);
            large += is_large32(x << 16) + is_large32(x & 0xffff0000u);
        } else {
            nonfinite += ((x & 0x7c00u) == 0x7c00u ? 1u : 0u) + ((x & 0x7c000000u) == 0x7c000000u ? 1u : 0u);
        }
    };
    auto chunk = [&](const u4v v) { word(v.x); word(v.y); word(v.z); word(v.w); };
    int c = threadIdx.x;
    // eight independent loads in flight per lane, non-temporal: the rows are read once
    for (; c + 7 * 256 < chunks; c += 8 * 256) {
        u4v v[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) v[k] = __builtin_nontemporal_load(s + c + k * 256);
#pragma unroll
        for (int k = 0; k < 8; ++k) chunk(v[k]);
    }
    for (; c < chunks; c += 256) chunk(__builtin_nontemporal_load(s + c));
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        nonfinite += __shfl_xor(nonfinite, o, 64);
        large += __shfl_xor(large, o, 64);
    }
    if ((threadIdx.x & 63) == 0) {
        if (nonfinite) atomicAdd(&report[1], (unsigned long long)nonfinite);
        if (large) atomicAdd(&report[2], (unsigned long long)large);
    }
    if (threadIdx.x == 0) atomicAdd(&report[3], (unsigned long long)rows * (unsigned long long)(row_bytes / (DT == EL_F32 ? 4 : 2)));
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
    (void)hipGetLastError();      // errors other libraries left behind in this thread are not this launch's
    hipLaunchKernelGGL(el::k_gather_batch, grid, block, 0, (hipStream_t)stream,
                       (const char *)H_src, src_batch_stride * es, lengths_src, B_src,
                       (char *)H_dst, dst_batch_stride * es, lengths_dst, index, n, (int)row_bytes);
    return hipGetLastError() == hipSuccess ? EL_OK : EL_ERR_HIP;
}

extern "C" el_status el_attn_check_inputs(el_dtype dtype, int32_t d_model,
                                          const void *H, int64_t H_batch_stride, const int32_t *lengths,
                                          int32_t B, int32_t n, uint64_t *report, void *stream)
{
    if (!H || !report) return EL_ERR_INVALID_ARG;
    if (dtype != EL_F32 && dtype != EL_F16 && dtype != EL_BF16) return EL_ERR_INVALID_ARG;
    if (d_model < 1 || B < 1 || n < 1 || B > 65535) return EL_ERR_INVALID_ARG;
    const int64_t es = (int64_t)el::dtype_size(dtype);
    const int64_t row_bytes = (int64_t)d_model * es;
    if (row_bytes % 16 != 0 || row_bytes > (1 << 30)) return EL_ERR_INVALID_ARG;
    if (H_batch_stride < (int64_t)n * d_model) return EL_ERR_INVALID_ARG;
    if (((uintptr_t)H & 15) || ((uintptr_t)report & 7) || (H_batch_stride * es) % 16 != 0) return EL_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    unsigned long long *rep = (unsigned long long *)report;
    (void)hipGetLastError();      // errors other libraries left behind in this thread are not this launch's
    hipLaunchKernelGGL(el::k_zero_report, dim3(1), dim3(64), 0, s, rep);
    const dim3 grid((n + el::kRowsPerCheckBlock - 1) / el::kRowsPerCheckBlock, B), block(256);
    const char *Hc = (const char *)H;
    if (dtype == EL_F32) hipLaunchKernelGGL((el::k_check_inputs<EL_F32>), grid, block, 0, s, Hc, H_batch_stride * es, lengths, n, (int)row_bytes, rep);
    else if (dtype == EL_F16) hipLaunchKernelGGL((el::k_check_inputs<EL_F16>), grid, block, 0, s, Hc, H_batch_stride * es, lengths, n, (int)row_bytes, rep);
    else hipLaunchKernelGGL((el::k_check_inputs<EL_BF16>), grid, block, 0, s, Hc, H_batch_stride * es, lengths, n, (int)row_bytes, rep);
    return hipGetLastError() == hipSuccess ? EL_OK : EL_ERR_HIP;
}
