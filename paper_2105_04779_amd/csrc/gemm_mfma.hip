// Small-M MFMA GEMMs for the projection steps of the EL-attention decode step (steps a1, a2, a6,
// a7 of Algorithm 3's attention routine; group 2 of Table 1 -- O(d_m^2) per query, weight-read
// bound).  All four are C[m, n] = sum_k A[m, k] * Bt[n, k] with both operands contiguous along k
// (W^Q, W^V, W^O are stored transposed at prepare time for exactly this; W^K already has that shape).
//
//   a1  Qp    = (q . W^Q + b^Q) * scale   k_gemm_slab  A = queries (storage dtype), Bt = (W^Q)^T (storage dtype)
//   a2  ELQ_i = Qp_i . (W_i^K)^T          k_elq_slab   A = Qp (fp16),               Bt = W^K in fp16     per head
//                                                      (result as a high + low pair of planes in the storage type)
//   a6  A_i   = X_i . W_i^V               k_vproj_slab A = merge of the pieces,     Bt = (W^V)^T in fp16 per head
//   a7  out   = A . W^O + c_out           k_gemm_slab  A = A (fp16),                Bt = (W^O)^T in fp16
//
// Storage-dtype operands enter the MFMA exactly (a1 runs in the storage type).  From a2 on everything
// is fp16: bf16 weights are converted once at prepare time (exact above 2^-14, |error| <= 2^-25 below),
// and the intermediates Qp, merged X and A are rounded to fp16 once each (2^-12 relative; the
// measured end-to-end error stays several times under the 2e-3 bar).  Accumulation is fp32.
//
// k_gemm_slab: a workgroup stages 32 rows of A and 32 rows of Bt over the whole K in LDS with 1 KB
// LDS-DMA pieces (full cache lines, every byte fetched once per workgroup), then its four wavefronts
// split K.  k_vproj_slab: the same with the A rows built in LDS from the key-range partials.
// k_elq_slab: the weight slice stays in registers, operand fragments come straight from global memory
// (a2: K = d_k is tiny).
#include "el_internal.h"

namespace el {

typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef __bf16 b8 __attribute__((ext_vector_type(8)));
typedef float f4 __attribute__((ext_vector_type(4)));
typedef unsigned int u4 __attribute__((ext_vector_type(4)));

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
    int c_rB;             // k_elq_slab: padded rows per batch element of the output (logical row m, head i -> row i * x + m % x of element m / x)
    // k_vproj_slab: A points at the normalised fp16 pieces Xp [slot, Rs, d_m]; ML [slot, Rs, 2]; pm says which
    // slots belong to a batch element, parts bounds their number
    const float *ML;
    PieceMap pm;
    int parts, Rs;
    int N_heads;          // k_vproj_slab: heads (the grid is one-dimensional, see the kernel)
};

template <bool BF> struct Frag;
template <> struct Frag<false> {
    typedef h8 type;
    static __device__ __forceinline__ f4 mfma(h8 a, h8 b, f4 c) { return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0); }
};
template <> struct Frag<true> {
    typedef b8 type;
    static __device__ __forceinline__ f4 mfma(b8 a, b8 b, f4 c) { return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0); }
};

// ---------------------------------------------------------------------------------------------
// Slab GEMM: C[M, N] = A[M, K] . Bt[N, K]^T for K = 512, 768 or 1024 (rows of 1, 1.5 or 2 KB).  One workgroup
// owns a 32 x 32 output tile.  Its 64 operand rows are fetched once, whole, into LDS (row r lands
// XOR-swizzled by row_swizzle(r % 16), see dma_piece), so global traffic is full cache lines and
// (M/32 + N/32) passes over the operands in total.  Then wavefront w multiplies k-steps
// [w K/128, (w+1) K/128) for all four 16 x 16 sub-tiles, the partial tiles are added through LDS
// and wavefront w finishes sub-tile w.
template <bool BF, int CK>
__global__ void __launch_bounds__(256)
k_gemm_slab(const GemmArgs g)
{
    typedef typename Frag<BF>::type frag_t;
    __shared__ __attribute__((aligned(1024))) char S[64 * 2048];
    const int tid = threadIdx.x, l = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r16 = l & 15, q4 = l >> 4;
    const int m0 = blockIdx.y * 32, n0 = blockIdx.x * 32;
    const int rowb = g.K * 2;
    const unsigned s_lds = (unsigned)(uintptr_t)(__attribute__((address_space(3))) char *)S;

    // ---- stage: wavefronts 0,1 fetch the A rows, 2,3 the Bt rows ----
    if (rowb == 1536) {
        // Rows of 1.5 KB do not split into 1 KB pieces: a wavefront's 16 rows are 24 KB of contiguous LDS, filled by
        // 24 requests; lane l of request j lands at chunk position p = 64 j + l of that block, which is row
        // r = p / 96, position q = p % 96, and must hold chunk q ^ swizzle(r) of the row.
        const char *mbase = w < 2 ? (const char *)g.A : (const char *)g.Bt;
        const int first = w < 2 ? m0 + 16 * w : n0 + 16 * (w - 2);
        const int lastv = (w < 2 ? g.M : g.N) - 1, ld = w < 2 ? g.lda : g.ldb;
#pragma unroll
        for (int j = 0; j < 24; ++j) {
            const int pz = 64 * j + l, r = pz / 96, q = pz - 96 * r;
            const unsigned voff = (unsigned)min(first + r, lastv) * (unsigned)(ld * 2) + (unsigned)((q ^ row_swizzle(r)) << 4);
            dma_piece(s_lds + 16 * w * rowb + 1024 * j, voff, mbase);
        }
    } else
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int rr = 16 * w + i;
        const char *sbase;
        if (w < 2) sbase = (const char *)g.A + (size_t)min(m0 + rr, g.M - 1) * g.lda * 2;
        else sbase = (const char *)g.Bt + (size_t)min(n0 + rr - 32, g.N - 1) * g.ldb * 2;
        const unsigned voff = (unsigned)((l ^ row_swizzle(i)) << 4);
        if (rowb == 2048) dma_row_2k(s_lds + rr * rowb, voff, sbase);
        else dma_piece(s_lds + rr * rowb, voff, sbase);
    }

    // bias of this lane's four output columns (sub-tile w), fetched while the slab is in flight
    const int mt = w >> 1, nt = w & 1;
    const int ncol = n0 + 16 * nt + 4 * q4;
    float badd[4] = {0.f, 0.f, 0.f, 0.f};
    if (ncol < g.N) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (g.bias) badd[j] = BF ? to_f32(((const bf16_t *)g.bias)[ncol + j]) : to_f32(((const f16_t *)g.bias)[ncol + j]);
            if (g.bias32) badd[j] += g.bias32[ncol + j];
        }
    }

    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();

    // ---- multiply: this wavefront's quarter of K ----
    const __attribute__((address_space(3))) char *Sl = (const __attribute__((address_space(3))) char *)S;
    const int fsw = row_swizzle(r16);
    f4 acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b) acc[a][b] = f4{0.f, 0.f, 0.f, 0.f};
    const int steps = g.K / 128;
    for (int st = 0; st < steps; ++st) {
        const int chunk = (4 * (w * steps + st) + q4) ^ fsw;
        const int off = r16 * rowb + (chunk << 4);
        const frag_t a0 = __builtin_bit_cast(frag_t, *(const __attribute__((address_space(3))) u4 *)(Sl + off));
        const frag_t a1 = __builtin_bit_cast(frag_t, *(const __attribute__((address_space(3))) u4 *)(Sl + off + 16 * rowb));
        const frag_t b0 = __builtin_bit_cast(frag_t, *(const __attribute__((address_space(3))) u4 *)(Sl + off + 32 * rowb));
        const frag_t b1 = __builtin_bit_cast(frag_t, *(const __attribute__((address_space(3))) u4 *)(Sl + off + 48 * rowb));
        // weights as the MFMA's A operand: the result is the transposed tile, so a lane holds four
        // consecutive output columns of one row
        acc[0][0] = Frag<BF>::mfma(b0, a0, acc[0][0]);
        acc[0][1] = Frag<BF>::mfma(b1, a0, acc[0][1]);
        acc[1][0] = Frag<BF>::mfma(b0, a1, acc[1][0]);
        acc[1][1] = Frag<BF>::mfma(b1, a1, acc[1][1]);
    }

    // ---- add the four K quarters: wavefront w collects sub-tile (mt, nt) ----
    __syncthreads();                                   // the slab is no longer needed
    float *red = (float *)S;
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b) *(f4 *)(red + (((w * 4) + a * 2 + b) * 64 + l) * 4) = acc[a][b];
    __syncthreads();
    f4 sum = f4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        const f4 o = *(const f4 *)(red + (((s * 4) + mt * 2 + nt) * 64 + l) * 4);
        sum[0] += o[0]; sum[1] += o[1]; sum[2] += o[2]; sum[3] += o[3];
    }
    const int mm = m0 + 16 * mt + r16;
    if (mm >= g.M || ncol >= g.N) return;
    float val[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) val[j] = (sum[j] + badd[j]) * g.scale;
    const size_t ci = (size_t)mm * g.ldc + ncol;
    if (CK == C_F32) {
        *(f4 *)((float *)g.C + ci) = f4{val[0], val[1], val[2], val[3]};
    } else if (CK == C_F16) {
        typedef _Float16 h4 __attribute__((ext_vector_type(4)));
        *(h4 *)((f16_t *)g.C + ci) = h4{(_Float16)val[0], (_Float16)val[1], (_Float16)val[2], (_Float16)val[3]};
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) from_f32(val[j], (bf16_t *)g.C + ci + j);
    }
}

// ---------------------------------------------------------------------------------------------
// Merge of the key-range partials fused with a6 (A_i = X_i . W_i^V, Eq. 5 / Eq. 8), one workgroup
// per (16 rows, head).  The head's 64 rows of (W^V)^T are fetched whole into LDS by LDS-DMA while
// the workgroup builds its 16 merged rows there: each wavefront reads the partials of 4 rows
// (full-row, coalesced), combines them with the log-sum-exp weights
//     X = sum_p (w_p l_p) Xhat_p / sum_p (w_p l_p),  w_p = 2^(m_p - M),
// and stores the row in fp16, XOR-swizzled like the weights.  Then the four wavefronts split K,
// add their 16 x 64 partial tiles through LDS, and wavefront w finishes columns [16w, 16w+16).
template <int DM>
__global__ void __launch_bounds__(256)
k_vproj_slab(const GemmArgs g)
{
    constexpr int ROWB = DM * 2;
    constexpr int A_BYTES = 16 * ROWB, B_BYTES = 64 * ROWB;
    __shared__ __attribute__((aligned(1024))) char S[A_BYTES + B_BYTES];
    const int tid = threadIdx.x, l = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r16 = l & 15, q4 = l >> 4;
    // Workgroup ids that differ by a multiple of 8 share an XCD and its L2.  Heads are dealt out so that an XCD
    // works on as few of them as possible (heads / 8 when that divides): it then pulls only those heads' weights
    // from memory, once, instead of every XCD pulling all of W^V.
    int m0, head;
    {
        const int heads = g.N_heads, xcd = blockIdx.x & 7, j = blockIdx.x >> 3;
        const int hp = (heads + 7) >> 3;                 // heads per XCD
        head = xcd * hp + j % hp;
        m0 = (j / hp) * 16;
        if (head >= heads || m0 >= g.M) return;
    }
    const unsigned s_lds = (unsigned)(uintptr_t)(__attribute__((address_space(3))) char *)S;

    // Order of the requests: the piece table first (a few scalars; the answer arrives while the first half of
    // the weights is being requested), then half of the weights, then the statistics and the partial rows
    // (which still have arithmetic ahead of them), then the rest of the weights (which go straight to LDS).
    int e_tot = 0, e_lo[4], e_hi[4], b_of[4];
#pragma unroll
    for (int ii = 0; ii < 4; ++ii) {
        b_of[ii] = __builtin_amdgcn_readfirstlane(min(m0 + 4 * w + ii, g.M - 1) / g.x);
        e_lo[ii] = e_hi[ii] = 0;
    }
    if (g.pm.E) {
        e_tot = g.pm.E[g.pm.B];
#pragma unroll
        for (int ii = 0; ii < 4; ++ii) { e_lo[ii] = g.pm.E[b_of[ii]]; e_hi[ii] = g.pm.E[b_of[ii] + 1]; }
    }
    // ---- weights of this head: rows 16w..16w+15 of its 64, straight into LDS ----
    auto weight_rows = [&](int i0, int i1) {
        if (ROWB == 1536) {                              // 1.5 KB rows: the rows as one block, see k_gemm_slab
            const char *sbase = (const char *)g.Bt + (size_t)(head * 64 + 16 * w + i0) * g.ldb * 2;
#pragma unroll
            for (int j = 0; j < (i1 - i0) * 3 / 2; ++j) {
                const int pz = 64 * j + l, r = pz / 96, q = pz - 96 * r;
                dma_piece(s_lds + A_BYTES + (16 * w + i0) * ROWB + 1024 * j,
                          (unsigned)(r * g.ldb * 2 + ((q ^ row_swizzle(i0 + r)) << 4)), sbase);
            }
            return;
        }
#pragma unroll
        for (int i = i0; i < i1; ++i) {
            const int rr = 16 * w + i;
            const char *sbase = (const char *)g.Bt + (size_t)(head * 64 + rr) * g.ldb * 2;
            const unsigned voff = (unsigned)((l ^ row_swizzle(i)) << 4);
            if (ROWB == 2048) dma_row_2k(s_lds + A_BYTES + rr * ROWB, voff, sbase);
            else dma_piece(s_lds + A_BYTES + rr * ROWB, voff, sbase);
        }
    };
    weight_rows(0, 8);

    // ---- merged activation rows 4w..4w+3 ----
    // Everything this needs is requested before anything is used: the statistics (one (row, part) pair
    // per lane), then all partial rows (four rows x the slots in use x both halves), so the whole merge
    // costs one round trip to memory.
    constexpr int HF = (ROWB + 1023) / 1024;             // 64-lane passes over a row of 16-byte chunks (the last may be half used)
    constexpr int CPR = ROWB / 16;
    int slot0[4], np[4];                                 // pieces of the four rows' batch elements (wave-uniform)
    {
        // integer divisions are long instruction sequences: the span length is worked out once, and rows of one
        // batch element (with a beam of four: all four rows of a wavefront) share one look-up
        const PieceCut cut = piece_cut(g.pm, e_tot);
#pragma unroll
        for (int ii = 0; ii < 4; ++ii) {
            if (ii > 0 && b_of[ii] == b_of[ii - 1]) { slot0[ii] = slot0[ii - 1]; np[ii] = np[ii - 1]; }
            else {
                piece_range(g.pm, cut, b_of[ii], e_lo[ii], e_hi[ii], slot0[ii], np[ii]);
                np[ii] = min(np[ii], kMaxParts);
            }
        }
    }
    auto row_src = [&](int ii, int p, int hf) {
        const int m = min(m0 + 4 * w + ii, g.M - 1);
        const int r = head * g.x + (m % g.x);
        return (const h8 *)((const f16_t *)g.A + (((size_t)slot0[ii] + p) * g.Rs + r) * g.lda + hf * 512 + 8 * l);
    };
    float mp, lp;
    {
        const int ii = l >> 4, p = l & 15;
        const int m = min(m0 + 4 * w + ii, g.M - 1);
        const int r = head * g.x + (m % g.x);
        const int s0 = ii == 0 ? slot0[0] : (ii == 1 ? slot0[1] : (ii == 2 ? slot0[2] : slot0[3]));
        const int n0 = ii == 0 ? np[0] : (ii == 1 ? np[1] : (ii == 2 ? np[2] : np[3]));
        const float *ml = g.ML + (((size_t)s0 + min(p, n0 - 1)) * g.Rs + r) * 2;
        mp = ml[0]; lp = ml[1];
        if (p >= n0) lp = 0.f;
    }

    h8 xv[4][HF][kMaxParts];
#pragma unroll
    for (int pp = 0; pp < kMaxParts; ++pp) {
        if (pp >= g.parts) continue;                     // uniform
#pragma unroll
        for (int ii = 0; ii < 4; ++ii) {
            if (pp >= np[ii]) continue;                  // uniform
#pragma unroll
            for (int hf = 0; hf < HF; ++hf)
                if (hf * 64 + l < CPR) xv[ii][hf][pp] = *row_src(ii, pp, hf);
        }
    }
    weight_rows(8, 16);
    float wgt_lane;
    {
        if (!(lp > 0.f)) { lp = 0.f; mp = -INFINITY; }       // an empty part (its maximum was never written)
        float Mx = mp;
#pragma unroll
        for (int o = 1; o < 16; o <<= 1) Mx = fmaxf(Mx, __shfl_xor(Mx, o, 64));
        float wp = lp > 0.f ? exp2f(mp - Mx) * lp : 0.f;
        float den = wp;
#pragma unroll
        for (int o = 1; o < 16; o <<= 1) den += __shfl_xor(den, o, 64);
        wgt_lane = den > 0.f ? wp / den : 0.f;
    }
#pragma unroll
    for (int ii = 0; ii < 4; ++ii) {
        const int ar = 4 * w + ii;
        float wrow[kMaxParts];
#pragma unroll
        for (int pp = 0; pp < kMaxParts; ++pp) {
            wrow[pp] = __shfl(wgt_lane, 16 * ii + pp, 64);
            if (pp >= np[ii]) wrow[pp] = 0.f;
        }
#pragma unroll
        for (int hf = 0; hf < HF; ++hf) {
            float v[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] = 0.f;
#pragma unroll
            for (int pp = 0; pp < kMaxParts; ++pp) {
                if (pp >= g.parts) continue;
                if (wrow[pp] != 0.f) {                   // an empty part's row was never written
#pragma unroll
                    for (int e = 0; e < 8; ++e) v[e] = fmaf(wrow[pp], (float)xv[ii][hf][pp][e], v[e]);
                }
            }
            h8 hv;
#pragma unroll
            for (int e = 0; e < 8; ++e) hv[e] = (_Float16)v[e];
            if (hf * 64 + l < CPR) *(h8 *)(S + ar * ROWB + (((hf * 64 + l) ^ row_swizzle(ar)) << 4)) = hv;
        }
    }

    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();

    // ---- multiply: this wavefront's quarter of K ----
    const __attribute__((address_space(3))) char *Sl = (const __attribute__((address_space(3))) char *)S;
    const int fsw = row_swizzle(r16);
    f4 acc[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) acc[t] = f4{0.f, 0.f, 0.f, 0.f};
    constexpr int STEPS = DM / 128;
#pragma unroll
    for (int st = 0; st < STEPS; ++st) {
        const int chunk = (4 * (w * STEPS + st) + q4) ^ fsw;
        const int off = r16 * ROWB + (chunk << 4);
        const h8 a0 = *(const __attribute__((address_space(3))) h8 *)(Sl + off);
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const h8 bt = *(const __attribute__((address_space(3))) h8 *)(Sl + A_BYTES + 16 * t * ROWB + off);
            acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(bt, a0, acc[t], 0, 0, 0);   // transposed tile: lane = row, 4 columns
        }
    }

    // ---- add the four K quarters; wavefront w finishes column block w ----
    __syncthreads();
    float *red = (float *)S;
#pragma unroll
    for (int t = 0; t < 4; ++t) *(f4 *)(red + ((w * 4 + t) * 64 + l) * 4) = acc[t];
    __syncthreads();
    f4 sum = f4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        const f4 o = *(const f4 *)(red + ((s * 4 + w) * 64 + l) * 4);
        sum[0] += o[0]; sum[1] += o[1]; sum[2] += o[2]; sum[3] += o[3];
    }
    const int mm = m0 + r16;
    if (mm >= g.M) return;
    typedef _Float16 h4 __attribute__((ext_vector_type(4)));
    *(h4 *)((f16_t *)g.C + (size_t)mm * g.ldc + head * 64 + 16 * w + 4 * q4) =
        h4{(_Float16)sum[0], (_Float16)sum[1], (_Float16)sum[2], (_Float16)sum[3]};
}

// bf16 -> fp16 copy of a weight matrix (prepare time).
__global__ void k_bf16_to_f16(const bf16_t *src, f16_t *dst, size_t n)   // src may equal dst
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) dst[i] = (f16_t)to_f32(src[i]);
}

hipError_t launch_bf16_to_f16(const void *src, void *dst, size_t n, hipStream_t s)
{
    hipLaunchKernelGGL(k_bf16_to_f16, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, (const bf16_t *)src, (f16_t *)dst, n);
    return hipGetLastError();
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
// ---------------------------------------------------------------------------------------------
// a2, query expansion (Eq. 9's Q_i (W_i^K)^T): ELQ[b, i*x + j, :] = Qp[b*x + j, head i] . (W_i^K)^T with
// d_k = 64.  One workgroup owns 64 output columns of one head for up to 256 logical rows: its slice
// of W^K (64 x 64, 8 KB) is read once and stays in registers as MFMA fragments while the four
// wavefronts walk over the row tiles, so W^K is read once per 256 rows instead of once per 16.
// Weights are the MFMA's A operand: a lane ends up with four consecutive columns of one row; the
// 16 x 64 tile then goes through LDS and leaves in the fragment order of the attention core (elq_frag_index),
// 64 contiguous bytes per row and 32-column fragment.
template <bool BF>
__global__ void __launch_bounds__(256)
k_elq_slab(const GemmArgs g)
{
    typedef uint16_t q4 __attribute__((ext_vector_type(4)));
    constexpr int MT = 4;                               // row tiles per wavefront
    __shared__ __attribute__((aligned(16))) uint16_t Ct[2][4][MT][16 * 72];   // [plane]; rows 144 bytes apart

    const int l = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int r16 = l & 15, qd = l >> 4;
    const int n0 = blockIdx.x * 64, head = blockIdx.y;
    const int mt0 = blockIdx.z * (4 * MT);              // first 16-row tile of this workgroup

    u4 bfr[4][2], afr[MT][2];
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int u = 0; u < 2; ++u)
            bfr[t][u] = *(const u4 *)((const f16_t *)g.Bt + (size_t)(n0 + 16 * t + r16) * g.ldb + head * 64 + 32 * u + 8 * qd);
#pragma unroll
    for (int mi = 0; mi < MT; ++mi) {
        const int m = min((mt0 + w + 4 * mi) * 16 + r16, g.M - 1);
#pragma unroll
        for (int u = 0; u < 2; ++u)
            afr[mi][u] = *(const u4 *)((const f16_t *)g.A + (size_t)m * g.lda + head * 64 + 32 * u + 8 * qd);
    }
#pragma unroll
    for (int mi = 0; mi < MT; ++mi) {
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            f4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int u = 0; u < 2; ++u)
                acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(h8, bfr[t][u]), __builtin_bit_cast(h8, afr[mi][u]), acc, 0, 0, 0);
            q4 hi, lo;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                uint16_t h, l2;
                split16<BF>(acc[e], h, l2);
                hi[e] = h; lo[e] = l2;
            }
            *(q4 *)(&Ct[0][w][mi][r16 * 72 + 16 * t + 4 * qd]) = hi;
            *(q4 *)(&Ct[1][w][mi][r16 * 72 + 16 * t + 4 * qd]) = lo;
        }
    }
    // a wavefront reads back only what it wrote: no barrier.  Eight lanes write one 128-byte row piece.
#pragma unroll
    for (int mi = 0; mi < MT; ++mi) {
#pragma unroll
        for (int hf = 0; hf < 2; ++hf) {
            const int row = 8 * hf + (l >> 3), m = (mt0 + w + 4 * mi) * 16 + row;
            if (m >= g.M) continue;
            uint16_t *dst = (uint16_t *)g.C + elq_frag_index(m / g.x, head * g.x + m % g.x, n0 + 8 * (l & 7), 0, g.c_rB, g.ldc);
            *(u4 *)dst = *(const u4 *)(&Ct[0][w][mi][row * 72 + 8 * (l & 7)]);
            *(u4 *)(dst + 512) = *(const u4 *)(&Ct[1][w][mi][row * 72 + 8 * (l & 7)]);
        }
    }
}

bool gemm_mfma_supported(int dtype, int d_m, int d_k)
{
    return (dtype == EL_F16 || dtype == EL_BF16) && (d_m == 512 || d_m == 768 || d_m == 1024) && d_k == 64;
}

static GemmArgs base_args(const Problem &p)
{
    GemmArgs g{};
    g.scale = 1.0f;
    g.x = p.beam;
    g.M = p.B * p.beam;
    return g;
}

template <bool BF, int CK>
static hipError_t launch_slab(const GemmArgs &g, hipStream_t s)
{
    hipLaunchKernelGGL((k_gemm_slab<BF, CK>), dim3((g.N + 31) / 32, (g.M + 31) / 32), dim3(256), 0, s, g);
    return hipGetLastError();
}

// a1: Qp = (q . W^Q + b^Q) * scale        [B*beam, hd] fp16
hipError_t launch_qproj_mfma(const el_attn_ctx *ctx, const Problem &p, const Workspace &ws, float scale, hipStream_t s)
{
    GemmArgs g = base_args(p);
    g.A = p.queries; g.Bt = ctx->w.WqT; g.C = ws.Qp; g.bias = ctx->w.bq; g.scale = scale;
    g.N = p.hd; g.K = p.d_m; g.lda = p.d_m; g.ldb = p.d_m; g.ldc = p.hd;
    return p.dtype == EL_BF16 ? launch_slab<true, C_F16>(g, s) : launch_slab<false, C_F16>(g, s);
}

// a2: ELQ[b, i*beam+j, :] = Qp[b*beam+j, head i] . (W_i^K)^T      high + low planes in fragment order, Rs rows per b
hipError_t launch_elq_mfma(const el_attn_ctx *ctx, const Problem &p, const Workspace &ws, int Rs, hipStream_t s)
{
    GemmArgs g = base_args(p);
    g.A = ws.Qp; g.Bt = ctx->w.WkH; g.C = ws.ELQ;
    g.N = p.d_m; g.K = p.d_k; g.lda = p.hd; g.ldb = p.hd; g.ldc = p.d_m;
    g.c_rB = Rs;
    const dim3 grid(p.d_m / 64, p.heads, (g.M + 255) / 256);
    if (p.dtype == EL_BF16) hipLaunchKernelGGL(k_elq_slab<true>, grid, dim3(256), 0, s, g);
    else hipLaunchKernelGGL(k_elq_slab<false>, grid, dim3(256), 0, s, g);
    return hipGetLastError();
}

// merge + a6: A[b*beam+j, head i] = (sum_p w_p Xp[b,p,i*beam+j,:]) . W_i^V       fp16   (d_k = 64)
hipError_t launch_vproj_mfma(const el_attn_ctx *ctx, const Problem &p, const Workspace &ws, const CorePlan &pl,
                             hipStream_t s)
{
    GemmArgs g = base_args(p);
    g.A = ws.Xp; g.Bt = ctx->w.WvT; g.C = ws.A; g.ML = ws.ML; g.parts = pl.parts; g.Rs = pl.Rs;
    g.pm = piece_map(pl, ws, p.B);
    g.N = p.d_k; g.K = p.d_m; g.lda = p.d_m; g.ldb = p.d_m; g.ldc = p.hd;
    g.N_heads = p.heads;
    const int hp = (p.heads + 7) / 8;                    // heads per XCD; 8 * hp * (row tiles) workgroups
    const dim3 grid(8 * hp * ((g.M + 15) / 16)), block(256);
    if (p.d_m == 1024) hipLaunchKernelGGL((k_vproj_slab<1024>), grid, block, 0, s, g);
    else if (p.d_m == 768) hipLaunchKernelGGL((k_vproj_slab<768>), grid, block, 0, s, g);
    else hipLaunchKernelGGL((k_vproj_slab<512>), grid, block, 0, s, g);
    return hipGetLastError();
}

// a7: out = A . W^O + c_out
hipError_t launch_oproj_mfma(const el_attn_ctx *ctx, const Problem &p, const Workspace &ws, const float *bias32, hipStream_t s)
{
    GemmArgs g = base_args(p);
    g.A = ws.A; g.Bt = ctx->w.WoT; g.C = p.out; g.bias32 = bias32;
    g.N = p.d_m; g.K = p.hd; g.lda = p.hd; g.ldb = p.hd; g.ldc = p.d_m;
    if (p.out_dtype == EL_F32) return launch_slab<false, C_F32>(g, s);
    if (p.dtype == EL_BF16) return launch_slab<false, C_BF16>(g, s);
    return launch_slab<false, C_F16>(g, s);
}

} // namespace el
