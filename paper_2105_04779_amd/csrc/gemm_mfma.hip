// Small-M MFMA GEMMs for the projection steps of the EL-attention decode step (steps a1, a2, a6,
// a7 of Algorithm 3's attention routine; group 2 of Table 1 -- O(d_m^2) per query, weight-read
// bound).  All four are C[m, n] = sum_k A[m, k] * Bt[n, k]: both operands contiguous along k, so
// every MFMA operand fragment is one 16-byte load straight from global memory (the weights W^Q,
// W^V, W^O are stored transposed at prepare time for exactly this; W^K already has that shape).
//
//   a1  Qp   = q . W^Q + b^Q              A = queries (storage dtype),    Bt = (W^Q)^T
//   a2  ELQ_i = Qp_i . (W_i^K)^T          A = Qp (fp32),                  Bt = W^K        per head
//   a6  A_i  = X_i . W_i^V                A = merge of split partials,    Bt = (W^V)^T    per head
//   a7  out  = A . W^O + c_out            A = A (fp32),                   Bt = (W^O)^T
//
// Storage-dtype operands enter the MFMA exactly.  fp32 activations are split into a high and a
// low half in the weights' 16-bit type (two MFMAs per fragment), so nothing wider than the final
// fp16 EL-Q is ever rounded to 16 bits: 16 (bf16 pair) or 22 (fp16 pair) significant bits survive.
// Accumulation is fp32 (v_mfma_f32_16x16x32_{f16,bf16}).
#include "el_internal.h"

namespace el {

typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef __bf16 b8 __attribute__((ext_vector_type(8)));
typedef float f4 __attribute__((ext_vector_type(4)));
typedef unsigned int u4 __attribute__((ext_vector_type(4)));

enum { A_STORAGE = 0, A_F32 = 1, A_MERGE = 2 };
enum { C_F32 = 0, C_F16 = 1, C_BF16 = 2 };

struct GemmArgs {
    const void *A;        // activations (see a_kind)
    const void *Bt;       // weights [N rows, K contiguous], storage dtype
    void *C;
    const void *bias;     // per output column, storage dtype, may be null
    const float *bias32;  // per output column, fp32, may be null
    float scale;          // applied to (acc + bias)
    int M, N, K;          // per batch (head)
    int lda, ldb, ldc;    // row strides in elements
    int x;                // beam: logical row m = b*x + j
    // physical row of logical row m in batch z:  (m / x) * rB + (m % x) * rJ + z * rI
    int a_rB, a_rJ, a_rI, c_rB, c_rJ, c_rI;
    int a_col_z, bt_row_z, bt_col_z, c_col_z;   // per-batch offsets (elements / rows)
    // A_MERGE: A points at the normalised fp16 split partials Xp [B, parts, Rs, d_m]; ML [B, parts, Rs, 2]
    const float *ML;
    int parts, Rs;
};

template <bool BF> struct Frag;
template <> struct Frag<false> {
    typedef h8 type;
    static __device__ __forceinline__ f4 mfma(h8 a, h8 b, f4 c) { return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0); }
    static __device__ __forceinline__ void split(const float *v, h8 &hi, h8 &lo) {
#pragma unroll
        for (int e = 0; e < 8; ++e) { const _Float16 h = (_Float16)v[e]; hi[e] = h; lo[e] = (_Float16)(v[e] - (float)h); }
    }
};
template <> struct Frag<true> {
    typedef b8 type;
    static __device__ __forceinline__ f4 mfma(b8 a, b8 b, f4 c) { return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0); }
    static __device__ __forceinline__ void split(const float *v, b8 &hi, b8 &lo) {
#pragma unroll
        for (int e = 0; e < 8; ++e) { const __bf16 h = (__bf16)v[e]; hi[e] = h; lo[e] = (__bf16)(v[e] - (float)h); }
    }
};

// One wavefront computes a 16 x (16*NT) tile over a K range.  A workgroup is KS x WM x WN wavefronts
// (KS * WM * WN = 4): KS wavefronts split K for the same tile and add up through LDS -- these GEMMs
// are a few MFLOP per tile and latency-bound, so the point is to have every load of a tile in
// flight at once (U k-steps are fetched before the first MFMA of a round).
template <bool BF, int AK, int CK, int NT, int WN, int KS, int U>
__global__ void __launch_bounds__(256)
k_gemm_nt(const GemmArgs g)
{
    typedef typename Frag<BF>::type frag_t;
    constexpr int WM = 4 / (WN * KS);
    static_assert(WM >= 1 && WM * WN * KS == 4, "four wavefronts per workgroup");
    __shared__ float red[KS > 1 ? (KS - 1) * WM * WN * NT * 256 : 1];

    const int l = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int r16 = l & 15, q4 = l >> 4;
    const int z = blockIdx.z;
    const int ks = w % KS, wt = w / KS;              // K slice, tile slot inside the workgroup
    const int m0 = (blockIdx.y * WM + wt / WN) * 16;
    const int n0 = (blockIdx.x * WN + wt % WN) * 16 * NT;
    const bool live = m0 < g.M && n0 < g.N;          // dead slots still reach the barrier below

    // A row of this lane (clamped: lanes past M recompute the last row and never store)
    const int m = min(m0 + r16, g.M - 1);
    const size_t a_row = (size_t)(m / g.x) * g.a_rB + (size_t)(m % g.x) * g.a_rJ + (size_t)z * g.a_rI;

    float wgt[kMaxParts];
    if (AK == A_MERGE) {
        // log-sum-exp weights of this row's key-range partials (reference maxima in log2 units)
        const int b = m / g.x, r = (m % g.x) * g.a_rJ + z * g.a_rI;
        float Mx = -INFINITY;
        for (int p = 0; p < g.parts; ++p) {
            const float *ml = g.ML + (((size_t)b * g.parts + p) * g.Rs + r) * 2;
            if (ml[1] > 0.f) Mx = fmaxf(Mx, ml[0]);
        }
        float den = 0.f;
#pragma unroll
        for (int p = 0; p < kMaxParts; ++p) {
            wgt[p] = 0.f;
            if (p < g.parts) {
                const float *ml = g.ML + (((size_t)b * g.parts + p) * g.Rs + r) * 2;
                if (ml[1] > 0.f) { wgt[p] = exp2f(ml[0] - Mx) * ml[1]; den += wgt[p]; }
            }
        }
        const float inv = 1.0f / den;
#pragma unroll
        for (int p = 0; p < kMaxParts; ++p) wgt[p] *= inv;
    }

    const char *Bt = (const char *)g.Bt;
    size_t bt_off[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const int n = min(n0 + 16 * t + r16, g.N - 1);
        bt_off[t] = ((size_t)(g.bt_row_z * z + n) * g.ldb + (size_t)g.bt_col_z * z + 8 * q4) * 2;
    }

    f4 acc[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) acc[t] = f4{0.f, 0.f, 0.f, 0.f};

    const int kspan = g.K / KS;                       // K is a multiple of 32 * KS (checked by the host)
    const int kbeg = ks * kspan, kend = kbeg + kspan;

    if (live)
    for (int kr = kbeg; kr < kend; kr += 32 * U) {
        // ---- fetch U k-steps of A and Bt fragments ----
        u4 a_raw[U][AK == A_STORAGE ? 1 : 2];
        u4 b_raw[U][NT];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int k0 = min(kr + 32 * u, kend - 32);    // rounds that overrun re-read the last step (and skip its MFMAs)
            if (AK == A_STORAGE) {
                a_raw[u][0] = *(const u4 *)((const char *)g.A + (a_row * g.lda + (size_t)g.a_col_z * z + k0 + 8 * q4) * 2);
            } else if (AK == A_F32) {
                const float *ap = (const float *)g.A + a_row * g.lda + (size_t)g.a_col_z * z + k0 + 8 * q4;
                a_raw[u][0] = *(const u4 *)ap;
                a_raw[u][1] = *(const u4 *)(ap + 4);
            }
#pragma unroll
            for (int t = 0; t < NT; ++t) b_raw[u][t] = *(const u4 *)(Bt + bt_off[t] + (size_t)k0 * 2);
        }
        // ---- multiply ----
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int k0 = kr + 32 * u;
            if (k0 >= kend) break;
            frag_t a_hi, a_lo;
            if (AK == A_STORAGE) {
                a_hi = __builtin_bit_cast(frag_t, a_raw[u][0]);
            } else {
                float v[8];
                if (AK == A_F32) {
                    const f4 v0 = __builtin_bit_cast(f4, a_raw[u][0]), v1 = __builtin_bit_cast(f4, a_raw[u][1]);
                    v[0] = v0[0]; v[1] = v0[1]; v[2] = v0[2]; v[3] = v0[3];
                    v[4] = v1[0]; v[5] = v1[1]; v[6] = v1[2]; v[7] = v1[3];
                } else {
                    const int b = m / g.x, r = (m % g.x) * g.a_rJ + z * g.a_rI;
#pragma unroll
                    for (int e = 0; e < 8; ++e) v[e] = 0.f;
#pragma unroll
                    for (int p = 0; p < kMaxParts; ++p) {
                        if (p < g.parts && wgt[p] != 0.f) {
                            const h8 xv = *(const h8 *)((const f16_t *)g.A + (((size_t)b * g.parts + p) * g.Rs + r) * g.lda + k0 + 8 * q4);
#pragma unroll
                            for (int e = 0; e < 8; ++e) v[e] = fmaf(wgt[p], (float)xv[e], v[e]);
                        }
                    }
                }
                Frag<BF>::split(v, a_hi, a_lo);
            }
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                const frag_t bf = __builtin_bit_cast(frag_t, b_raw[u][t]);
                acc[t] = Frag<BF>::mfma(a_hi, bf, acc[t]);
                if (AK != A_STORAGE) acc[t] = Frag<BF>::mfma(a_lo, bf, acc[t]);
            }
        }
    }

    // ---- add the K slices of a tile (slice 0 collects) ----
    if (KS > 1) {
        if (ks > 0) {
#pragma unroll
            for (int t = 0; t < NT; ++t)
                *(f4 *)(red + ((((ks - 1) * (WM * WN) + wt) * NT + t) * 64 + l) * 4) = acc[t];
        }
        __syncthreads();
        if (ks > 0) return;
#pragma unroll
        for (int s = 1; s < KS; ++s)
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                const f4 o = *(const f4 *)(red + ((((s - 1) * (WM * WN) + wt) * NT + t) * 64 + l) * 4);
                acc[t][0] += o[0]; acc[t][1] += o[1]; acc[t][2] += o[2]; acc[t][3] += o[3];
            }
    }
    if (!live) return;

    // C layout of the MFMA: lane holds rows 4*q4 + j (j = 0..3) of column l%16
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const int n = n0 + 16 * t + r16;
        if (n >= g.N) continue;
        float badd = 0.f;
        if (g.bias) badd = BF ? to_f32(((const bf16_t *)g.bias)[g.c_col_z * z + n]) : to_f32(((const f16_t *)g.bias)[g.c_col_z * z + n]);
        if (g.bias32) badd += g.bias32[g.c_col_z * z + n];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int mm = m0 + 4 * q4 + j;
            if (mm < g.M) {
                const size_t c_row = (size_t)(mm / g.x) * g.c_rB + (size_t)(mm % g.x) * g.c_rJ + (size_t)z * g.c_rI;
                const size_t ci = c_row * g.ldc + (size_t)g.c_col_z * z + n;
                const float val = (acc[t][j] + badd) * g.scale;
                if (CK == C_F32) ((float *)g.C)[ci] = val;
                else if (CK == C_F16) ((f16_t *)g.C)[ci] = (f16_t)val;
                else from_f32(val, (bf16_t *)g.C + ci);
            }
        }
    }
}

// Transpose a [rows, cols] matrix of 16-bit elements (prepare-time packing of W^Q, W^V, W^O).
__global__ void k_transpose16(const uint16_t *__restrict__ src, uint16_t *__restrict__ dst, int rows, int cols)
{
    __shared__ uint16_t tile[32][33];
    const int bx = blockIdx.x * 32, by = blockIdx.y * 32;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;   // 32 x 8
    for (int i = ty; i < 32; i += 8)
        if (by + i < rows && bx + tx < cols) tile[i][tx] = src[(size_t)(by + i) * cols + bx + tx];
    __syncthreads();
    for (int i = ty; i < 32; i += 8)
        if (bx + i < cols && by + tx < rows) dst[(size_t)(bx + i) * rows + by + tx] = tile[tx][i];
}

hipError_t launch_transpose16(const void *src, void *dst, int rows, int cols, hipStream_t s)
{
    hipLaunchKernelGGL(k_transpose16, dim3((cols + 31) / 32, (rows + 31) / 32), dim3(256), 0, s,
                       (const uint16_t *)src, (uint16_t *)dst, rows, cols);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
template <int AK, int CK, int NT, int WN, int KS, int U>
static hipError_t launch_gemm(const GemmArgs &g, bool bf, int batches, hipStream_t s)
{
    constexpr int WM = 4 / (WN * KS);
    const dim3 grid((g.N + 16 * NT * WN - 1) / (16 * NT * WN), (g.M + 16 * WM - 1) / (16 * WM), batches), block(256);
    if (bf) hipLaunchKernelGGL((k_gemm_nt<true, AK, CK, NT, WN, KS, U>), grid, block, 0, s, g);
    else hipLaunchKernelGGL((k_gemm_nt<false, AK, CK, NT, WN, KS, U>), grid, block, 0, s, g);
    return hipGetLastError();
}

bool gemm_mfma_supported(int dtype, int d_m, int d_k)
{
    return (dtype == EL_F16 || dtype == EL_BF16) && d_m % 128 == 0 && d_k % 64 == 0;
}

static GemmArgs base_args(const Problem &p)
{
    GemmArgs g{};
    g.scale = 1.0f;
    g.x = p.beam;
    g.M = p.B * p.beam;
    return g;
}

// a1: Qp = (q . W^Q + b^Q) * scale        [B*beam, hd] fp32
hipError_t launch_qproj_mfma(const el_attn_ctx *ctx, const Problem &p, const Workspace &ws, float scale, hipStream_t s)
{
    GemmArgs g = base_args(p);
    g.A = p.queries; g.Bt = ctx->w.WqT; g.C = ws.Qp; g.bias = ctx->w.bq; g.scale = scale;
    g.N = p.hd; g.K = p.d_m; g.lda = p.d_m; g.ldb = p.d_m; g.ldc = p.hd;
    g.a_rB = p.beam; g.a_rJ = 1; g.c_rB = p.beam; g.c_rJ = 1;
    return launch_gemm<A_STORAGE, C_F32, 2, 1, 4, 8>(g, p.dtype == EL_BF16, 1, s);
}

// a2: ELQ[b, i*beam+j, :] = Qp[b*beam+j, head i] . (W_i^K)^T      fp16, row stride d_m, Rs rows per b
hipError_t launch_elq_mfma(const el_attn_ctx *ctx, const Problem &p, const Workspace &ws, int Rs, hipStream_t s)
{
    GemmArgs g = base_args(p);
    g.A = ws.Qp; g.Bt = ctx->w.Wk; g.C = ws.ELQ;
    g.N = p.d_m; g.K = p.d_k; g.lda = p.hd; g.ldb = p.hd; g.ldc = p.d_m;
    g.a_rB = p.beam; g.a_rJ = 1; g.a_col_z = p.d_k;
    g.bt_col_z = p.d_k;
    g.c_rB = Rs; g.c_rJ = 1; g.c_rI = p.beam;
    const bool bf = p.dtype == EL_BF16;
    if (p.d_m % 512 == 0) return launch_gemm<A_F32, C_F16, 8, 4, 1, 2>(g, bf, p.heads, s);
    return launch_gemm<A_F32, C_F16, 2, 4, 1, 2>(g, bf, p.heads, s);
}

// merge + a6: A[b*beam+j, head i] = (sum_p w_p Xp[b,p,i*beam+j,:]) . W_i^V       fp32
hipError_t launch_vproj_mfma(const el_attn_ctx *ctx, const Problem &p, const Workspace &ws, int parts, int Rs,
                             hipStream_t s)
{
    GemmArgs g = base_args(p);
    g.A = ws.Xp; g.Bt = ctx->w.WvT; g.C = ws.A; g.ML = ws.ML; g.parts = parts; g.Rs = Rs;
    g.N = p.d_k; g.K = p.d_m; g.lda = p.d_m; g.ldb = p.d_m; g.ldc = p.hd;
    g.a_rJ = 1; g.a_rI = p.beam;            // row inside the batch element: i*beam + j
    g.bt_row_z = p.d_k;
    g.c_rB = p.beam; g.c_rJ = 1; g.c_col_z = p.d_k;
    const bool bf = p.dtype == EL_BF16;
    // one workgroup covers a head's whole d_k = 64 columns, so every partial row is read by one workgroup only
    return launch_gemm<A_MERGE, C_F32, 4, 1, 4, 4>(g, bf, p.heads, s);
}

// a7: out = A . W^O + c_out
hipError_t launch_oproj_mfma(const el_attn_ctx *ctx, const Problem &p, const Workspace &ws, hipStream_t s)
{
    GemmArgs g = base_args(p);
    g.A = ws.A; g.Bt = ctx->w.WoT; g.C = p.out; g.bias32 = ctx->w.c_out;
    g.N = p.d_m; g.K = p.hd; g.lda = p.hd; g.ldb = p.hd; g.ldc = p.d_m;
    g.a_rB = p.beam; g.a_rJ = 1; g.c_rB = p.beam; g.c_rJ = 1;
    const bool bf = p.dtype == EL_BF16;
    if (p.out_dtype == EL_F32) return launch_gemm<A_F32, C_F32, 2, 1, 4, 8>(g, bf, 1, s);
    if (bf) return launch_gemm<A_F32, C_BF16, 2, 1, 4, 8>(g, true, 1, s);
    return launch_gemm<A_F32, C_F16, 2, 1, 4, 8>(g, false, 1, s);
}

} // namespace el
