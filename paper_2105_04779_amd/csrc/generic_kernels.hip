// Plain fp32-arithmetic kernels for every step of the EL-attention decode step.
//
// They cover every dtype and shape (the fp32 configuration runs on them alone) and are
// the fallback wherever no MFMA kernel applies.  Arithmetic is fp32 fused multiply-add on
// storage values widened exactly; nothing is rounded to the storage type in between.
//
// Steps follow Algorithm 3's attention routine (appendix A) and Eq. 5 / Eq. 9:
//   qproj  a1  Qp = (q W^Q + b^Q) / sqrt(d_k)
//   elq    a2  EL-Q_i = Qp_i (W_i^K)^T                      rows r = i*beam + j
//   core   a3-a5  scores against H, softmax over the valid prefix, weighted sum of H
//   merge     log-sum-exp combination of key-range partials
//   vproj  a6  A_i = X_i W_i^V
//   oproj  a7  out = A W^O + c_out,  c_out = b^O + sum_i b_i^V W_i^O (Eq. 8/9)
#include "el_internal.h"

namespace el {

constexpr int kBlock = 256;
constexpr int kChunk = 512; // key positions scored per pass of the generic core

// ---------------------------------------------------------------------------------------------
template <typename T>
__global__ void k_cout(const T *__restrict__ bv, const T *__restrict__ bo, const T *__restrict__ Wo,
                       float *__restrict__ c_out, int hd, int d_m)
{
    int d = blockIdx.x * kBlock + threadIdx.x;
    if (d >= d_m) return;
    float acc = bo ? to_f32(bo[d]) : 0.f;
    if (bv)
        for (int c = 0; c < hd; ++c) acc = fmaf(to_f32(bv[c]), to_f32(Wo[(size_t)c * d_m + d]), acc);
    c_out[d] = acc;
}

// a1: Qp[row, c] = (sum_k q[row,k] Wq[k,c] + bq[c]) * scale
template <typename T>
__global__ void k_qproj(const T *__restrict__ q, const T *__restrict__ Wq, const T *__restrict__ bq,
                        float *__restrict__ Qp, int d_m, int hd, float scale)
{
    int c = blockIdx.x * kBlock + threadIdx.x;
    int row = blockIdx.y;
    if (c >= hd) return;
    const T *qr = q + (size_t)row * d_m;
    float acc = 0.f;
    for (int k = 0; k < d_m; ++k) acc = fmaf(to_f32(qr[k]), to_f32(Wq[(size_t)k * hd + c]), acc);
    if (bq) acc += to_f32(bq[c]);
    Qp[(size_t)row * hd + c] = acc * scale;
}

// a2: ELQ[b, r=i*beam+j, d] = sum_c Qp[b*beam+j, i*d_k+c] * Wk[d, i*d_k+c]
template <typename T>
__global__ void k_elq(const float *__restrict__ Qp, const T *__restrict__ Wk, float *__restrict__ elq,
                      int beam, int d_m, int d_k, int hd, int R)
{
    int d = blockIdx.x * kBlock + threadIdx.x;
    int r = blockIdx.y, b = blockIdx.z;
    if (d >= d_m) return;
    int i = r / beam, j = r % beam;
    const float *qp = Qp + ((size_t)b * beam + j) * hd + (size_t)i * d_k;
    const T *wk = Wk + (size_t)d * hd + (size_t)i * d_k;
    float acc = 0.f;
    for (int c = 0; c < d_k; ++c) acc = fmaf(qp[c], to_f32(wk[c]), acc);
    elq[((size_t)b * R + r) * d_m + d] = acc;
}

// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ float wave_sum(float v)
{
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ float wave_max(float v)
{
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

// a3-a5 for one (row r, key-range part p, batch element b) per workgroup.
// Writes the un-normalised weighted sum, and the running max / sum of its range.
template <typename T, int MAXD>
__global__ void __launch_bounds__(kBlock)
k_core_generic(const float *__restrict__ elq, const T *__restrict__ H, int64_t h_stride,
               const int32_t *__restrict__ lengths, int n, int d_m, int R, int Rstride, int parts,
               float *__restrict__ Xp, float *__restrict__ ML)
{
    extern __shared__ float smem[];
    float *q_s = smem;          // [d_m]
    float *s_s = smem + d_m;    // [kChunk]
    __shared__ float red[8];

    const int r = blockIdx.x, p = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int len = lengths ? lengths[b] : n;
    len = min(max(len, 1), n);
    const int t0 = (int)(((int64_t)len * p) / parts);
    const int t1 = (int)(((int64_t)len * (p + 1)) / parts);
    const T *Hb = H + (size_t)b * h_stride;

    for (int d = tid; d < d_m; d += kBlock) q_s[d] = elq[((size_t)b * R + r) * d_m + d];
    __syncthreads();

    float m = -INFINITY, l = 0.f;
    float acc[MAXD];
#pragma unroll
    for (int k = 0; k < MAXD; ++k) acc[k] = 0.f;

    for (int c0 = t0; c0 < t1; c0 += kChunk) {
        const int cnt = min(kChunk, t1 - c0);
        // scores of this chunk: one wave per key position, lanes over d
        for (int t = wave; t < cnt; t += kBlock / 64) {
            const T *hr = Hb + (size_t)(c0 + t) * d_m;
            float dot = 0.f;
            for (int d = lane; d < d_m; d += 64) dot = fmaf(q_s[d], to_f32(hr[d]), dot);
            dot = wave_sum(dot);
            if (lane == 0) s_s[t] = dot;
        }
        __syncthreads();
        float cm = -INFINITY;
        for (int t = tid; t < cnt; t += kBlock) cm = fmaxf(cm, s_s[t]);
        cm = wave_max(cm);
        if (lane == 0) red[wave] = cm;
        __syncthreads();
        cm = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
        const float m_new = fmaxf(m, cm);
        const float alpha = (m == -INFINITY) ? 0.f : expf(m - m_new);
        float ps = 0.f;
        for (int t = tid; t < cnt; t += kBlock) {
            float e = expf(s_s[t] - m_new);
            s_s[t] = e;
            ps += e;
        }
        ps = wave_sum(ps);
        if (lane == 0) red[4 + wave] = ps;
        __syncthreads();
        l = l * alpha + (red[4] + red[5] + red[6] + red[7]);
        m = m_new;
#pragma unroll
        for (int k = 0; k < MAXD; ++k) {
            const int d = tid + k * kBlock;
            if (d < d_m) {
                float a = acc[k] * alpha;
                for (int t = 0; t < cnt; ++t) a = fmaf(s_s[t], to_f32(Hb[(size_t)(c0 + t) * d_m + d]), a);
                acc[k] = a;
            }
        }
        __syncthreads();
    }

    float *xo = Xp + (((size_t)b * parts + p) * Rstride + r) * d_m;
#pragma unroll
    for (int k = 0; k < MAXD; ++k) {
        const int d = tid + k * kBlock;
        if (d < d_m) xo[d] = acc[k];
    }
    if (tid == 0) {
        float *ml = ML + (((size_t)b * parts + p) * Rstride + r) * 2;
        ml[0] = m;
        ml[1] = l;
    }
}

// Log-sum-exp merge of the partials of one row, normalised: Xn[b,r,:].
__global__ void k_merge(const float *__restrict__ Xp, const float *__restrict__ ML, float *__restrict__ Xn,
                        int d_m, int R, int Rstride, int parts)
{
    const int d = blockIdx.x * kBlock + threadIdx.x;
    const int r = blockIdx.y, b = blockIdx.z;
    if (d >= d_m) return;
    float M = -INFINITY;
    for (int p = 0; p < parts; ++p) M = fmaxf(M, ML[(((size_t)b * parts + p) * Rstride + r) * 2]);
    float num = 0.f, den = 0.f;
    for (int p = 0; p < parts; ++p) {
        const size_t row = ((size_t)b * parts + p) * Rstride + r;
        const float mp = ML[row * 2], lp = ML[row * 2 + 1];
        if (lp > 0.f) {
            const float w = expf(mp - M);
            num = fmaf(w, Xp[row * d_m + d], num);
            den = fmaf(w, lp, den);
        }
    }
    Xn[((size_t)b * R + r) * d_m + d] = num / den;
}

// a6: A[b*beam+j, i*d_k+c] = sum_d Xn[b, i*beam+j, d] * Wv[d, i*d_k+c]
template <typename T>
__global__ void k_vproj(const float *__restrict__ Xn, const T *__restrict__ Wv, float *__restrict__ A,
                        int beam, int d_m, int d_k, int hd, int R)
{
    const int cg = blockIdx.x * kBlock + threadIdx.x;
    const int row = blockIdx.y;
    if (cg >= hd) return;
    const int b = row / beam, j = row % beam, i = cg / d_k;
    const float *x = Xn + ((size_t)b * R + (size_t)i * beam + j) * d_m;
    float acc = 0.f;
    for (int d = 0; d < d_m; ++d) acc = fmaf(x[d], to_f32(Wv[(size_t)d * hd + cg]), acc);
    A[(size_t)row * hd + cg] = acc;
}

// a7: out[row, d] = sum_c A[row,c] * Wo[c,d] + c_out[d]
template <typename T, typename TO>
__global__ void k_oproj(const float *__restrict__ A, const T *__restrict__ Wo, const float *__restrict__ c_out,
                        TO *__restrict__ out, int d_m, int hd)
{
    const int d = blockIdx.x * kBlock + threadIdx.x;
    const int row = blockIdx.y;
    if (d >= d_m) return;
    const float *a = A + (size_t)row * hd;
    float acc = 0.f;
    for (int c = 0; c < hd; ++c) acc = fmaf(a[c], to_f32(Wo[(size_t)c * d_m + d]), acc);
    from_f32(acc + c_out[d], out + (size_t)row * d_m + d);
}

// ---------------------------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------------------------
#define EL_DISPATCH_DTYPE(dt, ...)                                                   \
    switch (dt) {                                                                    \
    case EL_F32: { using T = float; __VA_ARGS__; } break;                            \
    case EL_F16: { using T = f16_t; __VA_ARGS__; } break;                            \
    default:     { using T = bf16_t; __VA_ARGS__; } break;                           \
    }

static inline int cdiv(int a, int b) { return (a + b - 1) / b; }

hipError_t launch_cout(const el_attn_ctx *ctx, const void *bv, const void *bo, hipStream_t s)
{
    const int d_m = ctx->cfg.d_model, hd = ctx->hd;
    EL_DISPATCH_DTYPE(ctx->cfg.dtype,
        hipLaunchKernelGGL((k_cout<T>), dim3(cdiv(d_m, kBlock)), dim3(kBlock), 0, s,
                           (const T *)bv, (const T *)bo, (const T *)ctx->w.Wo, ctx->w.c_out, hd, d_m));
    return hipGetLastError();
}

hipError_t launch_qproj_generic(const el_attn_ctx *ctx, const Problem &p, const Workspace &ws, hipStream_t s)
{
    const float scale = 1.0f / sqrtf((float)p.d_k);
    EL_DISPATCH_DTYPE(p.dtype,
        hipLaunchKernelGGL((k_qproj<T>), dim3(cdiv(p.hd, kBlock), p.B * p.beam), dim3(kBlock), 0, s,
                           (const T *)p.queries, (const T *)ctx->w.Wq, (const T *)ctx->w.bq, ws.Qp,
                           p.d_m, p.hd, scale));
    return hipGetLastError();
}

hipError_t launch_elq_generic(const el_attn_ctx *ctx, const Problem &p, const float *Qp, float *elq, hipStream_t s)
{
    EL_DISPATCH_DTYPE(p.dtype,
        hipLaunchKernelGGL((k_elq<T>), dim3(cdiv(p.d_m, kBlock), p.R, p.B), dim3(kBlock), 0, s,
                           Qp, (const T *)ctx->w.Wk, elq, p.beam, p.d_m, p.d_k, p.hd, p.R));
    return hipGetLastError();
}

template <typename T>
static hipError_t launch_core_t(const Problem &p, const Workspace &ws, int parts, hipStream_t s)
{
    const size_t smem = (size_t)(p.d_m + kChunk) * sizeof(float);
    const dim3 grid(p.R, parts, p.B), block(kBlock);
    const float *elq = (const float *)ws.ELQ;
    const T *H = (const T *)p.H;
#define EL_CORE_CASE(MAXD)                                                                          \
    hipLaunchKernelGGL((k_core_generic<T, MAXD>), grid, block, smem, s, elq, H, p.H_batch_stride,   \
                       p.lengths, p.n, p.d_m, p.R, p.R, parts, ws.Xp, ws.ML)
    if (p.d_m <= 1 * kBlock) EL_CORE_CASE(1);
    else if (p.d_m <= 2 * kBlock) EL_CORE_CASE(2);
    else if (p.d_m <= 4 * kBlock) EL_CORE_CASE(4);
    else if (p.d_m <= 8 * kBlock) EL_CORE_CASE(8);
    else if (p.d_m <= 16 * kBlock) EL_CORE_CASE(16);
    else EL_CORE_CASE(32);
#undef EL_CORE_CASE
    return hipGetLastError();
}

hipError_t launch_core_generic(const el_attn_ctx *, const Problem &p, const Workspace &ws, int parts, hipStream_t s)
{
    EL_DISPATCH_DTYPE(p.dtype, return launch_core_t<T>(p, ws, parts, s));
    return hipErrorUnknown;
}

hipError_t launch_merge_generic(const el_attn_ctx *, const Problem &p, const Workspace &ws, int parts, int Rstride,
                                hipStream_t s)
{
    hipLaunchKernelGGL(k_merge, dim3(cdiv(p.d_m, kBlock), p.R, p.B), dim3(kBlock), 0, s,
                       (const float *)ws.Xp, (const float *)ws.ML, ws.Xn, p.d_m, p.R, Rstride, parts);
    return hipGetLastError();
}

hipError_t launch_vproj_generic(const el_attn_ctx *ctx, const Problem &p, const Workspace &ws, hipStream_t s)
{
    EL_DISPATCH_DTYPE(p.dtype,
        hipLaunchKernelGGL((k_vproj<T>), dim3(cdiv(p.hd, kBlock), p.B * p.beam), dim3(kBlock), 0, s,
                           (const float *)ws.Xn, (const T *)ctx->w.Wv, ws.A, p.beam, p.d_m, p.d_k, p.hd, p.R));
    return hipGetLastError();
}

hipError_t launch_oproj_generic(const el_attn_ctx *ctx, const Problem &p, const Workspace &ws, const float *bias32, hipStream_t s)
{
    const dim3 grid(cdiv(p.d_m, kBlock), p.B * p.beam), block(kBlock);
    EL_DISPATCH_DTYPE(p.dtype,
        if (p.out_dtype == EL_F32)
            hipLaunchKernelGGL((k_oproj<T, float>), grid, block, 0, s, (const float *)ws.A, (const T *)ctx->w.Wo,
                               bias32, (float *)p.out, p.d_m, p.hd);
        else
            hipLaunchKernelGGL((k_oproj<T, T>), grid, block, 0, s, (const float *)ws.A, (const T *)ctx->w.Wo,
                               bias32, (T *)p.out, p.d_m, p.hd));
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// fp32 copy of a bias vector (zeros when it is absent)
template <typename T>
__global__ void k_vec_f32(const T *__restrict__ src, float *__restrict__ dst, int n)
{
    const int i = blockIdx.x * kBlock + threadIdx.x;
    if (i < n) dst[i] = src ? to_f32(src[i]) : 0.f;
}

hipError_t launch_vec_f32(int dtype, const void *src, float *dst, int n, hipStream_t s)
{
    EL_DISPATCH_DTYPE(dtype,
        hipLaunchKernelGGL((k_vec_f32<T>), dim3(cdiv(n, kBlock)), dim3(kBlock), 0, s, (const T *)src, dst, n));
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Segment form of the step (section 3.2: one softmax over EL-attention on a shared prefix and ordinary
// attention on each beam's own continuation).  After a1..a6 on one key set, per (query row, head):
//   seg_A   = A + b^V           the segment's own normalised head output (Eq. 8 with the probabilities
//                               summing to one inside the segment)
//   seg_lse = log sum_t exp s_t for s = Q_i K_i^T / sqrt(d_k) INCLUDING Eq. 7's key-bias term Q_i (b_i^K)^T,
//                               which is constant inside a segment (and is dropped by the step itself) but
//                               is part of the scores ordinary attention reports
// The key-range statistics (reference exponent, sum relative to it) are folded by the log-sum-exp rule
// exactly as the merge of the partials does.
template <typename TA, typename TQ>
__global__ void k_seg_finish(const SegFinishArgs a)
{
    const int cg = blockIdx.x * kBlock + threadIdx.x;
    const int m = blockIdx.y;
    if (cg >= a.hd) return;
    a.seg_A[(size_t)m * a.hd + cg] = to_f32(((const TA *)a.A)[(size_t)m * a.hd + cg]) + a.bv32[cg];
    if (cg % a.d_k != 0) return;
    const int i = cg / a.d_k, b = m / a.beam, j = m % a.beam, r = i * a.beam + j;
    int slot0, np;
    piece_range(a.pm, b, slot0, np);
    float M = -INFINITY;
    for (int p = 0; p < np; ++p) {
        const float *ml = a.ML + (((size_t)slot0 + p) * a.Rstride + r) * 2;
        if (ml[1] > 0.f) M = fmaxf(M, ml[0]);
    }
    float L = 0.f;
    for (int p = 0; p < np; ++p) {
        const float *ml = a.ML + (((size_t)slot0 + p) * a.Rstride + r) * 2;
        if (ml[1] > 0.f) L += expf((ml[0] - M) * a.ml_to_nat) * ml[1];
    }
    float c = 0.f;
    const TQ *q = (const TQ *)a.Qp + (size_t)m * a.hd + (size_t)i * a.d_k;
    for (int k = 0; k < a.d_k; ++k) c = fmaf(to_f32(q[k]), a.bk32[i * a.d_k + k], c);
    a.seg_lse[(size_t)m * a.heads + i] = L > 0.f ? M * a.ml_to_nat + logf(L) + c * a.c_to_nat : -INFINITY;
}

hipError_t launch_seg_finish(const SegFinishArgs &a, bool a_f16, bool qp_f16, int rows, hipStream_t s)
{
    const dim3 grid(cdiv(a.hd, kBlock), rows), block(kBlock);
    if (a_f16 && qp_f16) hipLaunchKernelGGL((k_seg_finish<f16_t, f16_t>), grid, block, 0, s, a);
    else if (!a_f16 && !qp_f16) hipLaunchKernelGGL((k_seg_finish<float, float>), grid, block, 0, s, a);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

// One softmax over the union of the segments' keys, per (row, head):
//   w_s = exp(lse_s - max_s' lse_s') / sum_s' exp(lse_s' - max),   A = sum_s w_s seg_A_s      (then a7 on A)
template <typename TO>
__global__ void k_seg_merge(const SegMergeArgs a)
{
    const int cg = blockIdx.x * kBlock + threadIdx.x;
    const int m = blockIdx.y;
    if (cg >= a.hd) return;
    const int i = cg / a.d_k;
    float ls[kMaxSegments], M = -INFINITY;
#pragma unroll
    for (int s = 0; s < kMaxSegments; ++s) {
        ls[s] = s < a.nseg ? a.lse[s][(size_t)m * a.heads + i] : -INFINITY;
        M = fmaxf(M, ls[s]);
    }
    float num = 0.f, den = 0.f;
#pragma unroll
    for (int s = 0; s < kMaxSegments; ++s) {
        if (s < a.nseg && ls[s] > -INFINITY) {
            const float w = expf(ls[s] - M);
            num = fmaf(w, a.A[s][(size_t)m * a.hd + cg], num);
            den += w;
        }
    }
    from_f32(den > 0.f ? num / den : 0.f, (TO *)a.A_out + (size_t)m * a.hd + cg);
}

hipError_t launch_seg_merge(const SegMergeArgs &a, bool out_f16, int rows, hipStream_t s)
{
    const dim3 grid(cdiv(a.hd, kBlock), rows), block(kBlock);
    if (out_f16) hipLaunchKernelGGL((k_seg_merge<f16_t>), grid, block, 0, s, a);
    else hipLaunchKernelGGL((k_seg_merge<float>), grid, block, 0, s, a);
    return hipGetLastError();
}

} // namespace el
