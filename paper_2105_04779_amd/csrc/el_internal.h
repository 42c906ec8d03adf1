// Internal declarations shared by the library's translation units (not installed).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "el_attn.h"

namespace el {

// ---- storage element types --------------------------------------------------------------
struct bf16_t { uint16_t bits; };
typedef _Float16 f16_t;

__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(f16_t v) { return (float)v; }
__device__ __forceinline__ float to_f32(bf16_t v) { return __uint_as_float(((uint32_t)v.bits) << 16); }

// round-to-nearest-even conversions for stores in the storage dtype
__device__ __forceinline__ void from_f32(float x, float *p) { *p = x; }
__device__ __forceinline__ void from_f32(float x, f16_t *p) { *p = (f16_t)x; }
__device__ __forceinline__ void from_f32(float x, bf16_t *p) {
    uint32_t u = __float_as_uint(x);
    if ((u & 0x7fffffffu) > 0x7f800000u) { p->bits = 0x7fc0; return; }
    u += 0x7fffu + ((u >> 16) & 1u);
    p->bits = (uint16_t)(u >> 16);
}

// x = high + low, both in the 16-bit storage type (the pair carries ~16 mantissa bits of x)
template <bool BF16>
__device__ __forceinline__ void split16(float x, uint16_t &hi, uint16_t &lo)
{
    if (BF16) {
        bf16_t h, l2;
        from_f32(x, &h);
        from_f32(x - to_f32(h), &l2);
        hi = h.bits; lo = l2.bits;
    } else {
        const f16_t h = (f16_t)x, l2 = (f16_t)(x - (float)h);
        hi = __builtin_bit_cast(uint16_t, h); lo = __builtin_bit_cast(uint16_t, l2);
    }
}

// ---- LDS staging helpers shared by the MFMA kernels ---------------------------------------
// 16-byte chunk swizzle inside a tile row: a bijection of the low four chunk bits that makes both
// the row-wise b128 reads and the transposing b64 reads spread over all LDS banks.
__device__ __forceinline__ int row_swizzle(int row) { return ((row & 7) << 1) | ((row >> 3) & 1); }

// One 1 KB piece of a row, fetched by one wavefront straight into LDS.  `lds_addr` is the
// LDS byte address the piece starts at (lane i lands at +16 i), `voff` the lane's byte offset from
// the wave-uniform global base.  Issued through inline assembly so that the compiler does not
// serialise later LDS reads of the *other* tile buffer behind it; completion is awaited
// explicitly (s_waitcnt vmcnt(0)) before the barrier that publishes the tile.
__device__ __forceinline__ void dma_piece(unsigned lds_addr, unsigned voff, const char *sbase)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(lds_addr), "v"(voff), "s"(sbase) : "memory", "m0");
}
__device__ __forceinline__ void dma_row_2k(unsigned lds_addr, unsigned voff, const char *sbase)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2\n\tglobal_load_lds_dwordx4 %1, %2 offset:1024"
                 :: "s"(lds_addr), "v"(voff), "s"(sbase) : "memory", "m0");
}

// The same requests with the non-temporal hint: the lines are not kept in L2 or in the memory-side cache.
// For a stream far larger than that cache this leaves it to the data that IS re-read (weights, expanded
// queries, partial results) and raises the streaming rate itself.
__device__ __forceinline__ void dma_piece_nt(unsigned lds_addr, unsigned voff, const char *sbase)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2 nt"
                 :: "s"(lds_addr), "v"(voff), "s"(sbase) : "memory", "m0");
}
__device__ __forceinline__ void dma_row_2k_nt(unsigned lds_addr, unsigned voff, const char *sbase)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2 nt\n\tglobal_load_lds_dwordx4 %1, %2 offset:1024 nt"
                 :: "s"(lds_addr), "v"(voff), "s"(sbase) : "memory", "m0");
}

static inline size_t dtype_size(int dt) { return dt == EL_F32 ? 4 : 2; }
static inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// EL-Q for the MFMA core is stored in the order its score wavefronts load it: 1 KB fragments of 16 rows x 32
// columns (row-major inside: element (r16, c32) at r16 * 32 + c32), ordered [batch element][row / 16][column / 32]
// [plane: 0 high, 1 low], so that one load instruction of a wavefront (lane = 4 r16 + column group) reads one
// contiguous fragment.  Returns the element index of (b, row, col) of a plane; Rs = padded row count, a multiple
// of 16.
__host__ __device__ __forceinline__ size_t elq_frag_index(int b, int row, int col, int plane, int Rs, int d_m)
{
    const size_t frag = (((size_t)b * (Rs >> 4) + (row >> 4)) * (d_m >> 5) + (col >> 5)) * 2 + plane;
    return frag * 512 + (size_t)(row & 15) * 32 + (col & 31);
}

// ---- compile-time limits -----------------------------------------------------------------
constexpr int kMaxParts = 8;        // key-range partials per (batch element, row) the workspace holds
constexpr int kGenericMaxDm = 8192; // widest d_model the generic core kernel covers
constexpr int kScanMax = 1024;      // most batch elements whose tiles the streaming core cuts as one list

// Where the partial results ("pieces") of batch element b live: `np` consecutive slots from `slot0` in the
// partial buffers Xp [slot, Rs, d_m] and ML [slot, Rs, 2].
//   fixed cut      every element is cut into `parts` key ranges: slots b*parts .. b*parts+parts-1;
//   flattened cut  the 16-row tiles of all elements lie on one axis, element after element, each element preceded
//                  by a gap of `kcost` units (what moving on to a new element costs a workgroup, in tiles): tile kt
//                  of element b sits at coordinate E[b] + kcost * (b + 1) + kt, where E [B+1] is the prefix sum of
//                  the elements' tile counts, written by the core.  The axis is cut into G spans of
//                  cspan = max(ceil(length / G), lfloor + kcost) units, so a span that crosses into a new element
//                  holds kcost tiles fewer; the piece of (span g, element b) is slot g + b (unique: along the
//                  axis, span and element never decrease and one of them grows from piece to piece).
struct PieceMap {
    const int32_t *E;       // null: fixed cut
    int parts;              // fixed cut: parts per element
    int G, lfloor, B, kcost; // flattened cut
};
__host__ __device__ __forceinline__ int flat_cspan(int total_tiles, int B, int G, int lfloor, int kcost)
{
    const int length = total_tiles + kcost * B;
    const int c = (length + G - 1) / G;
    return c > lfloor + kcost ? c : lfloor + kcost;
}
// What every look-up of one launch shares: the span length on the cost axis (a division, done once).
struct PieceCut { int cspan; };
__device__ __forceinline__ PieceCut piece_cut(const PieceMap &m, int E_total)       // E_total = E[B]
{
    return PieceCut{m.E ? flat_cspan(E_total, m.B, m.G, m.lfloor, m.kcost) : 1};
}
__device__ __forceinline__ PieceCut piece_cut(const PieceMap &m) { return piece_cut(m, m.E ? m.E[m.B] : 0); }
// (E_b, E_b1) = (E[b], E[b+1]), for callers that fetch them ahead of time
__device__ __forceinline__ void piece_range(const PieceMap &m, const PieceCut &c, int b, int E_b, int E_b1, int &slot0, int &np)
{
    if (!m.E) { slot0 = b * m.parts; np = m.parts; return; }
    const int first = E_b + m.kcost * (b + 1), last = E_b1 + m.kcost * (b + 1) - 1;
    const int g_lo = first / c.cspan;
    // an element has at most kMaxParts pieces: the last span is found by stepping, not by a second division
    int cnt = 1;
    for (int k = 1; k < kMaxParts; ++k) cnt += last >= (g_lo + k) * c.cspan ? 1 : 0;
    if (last >= (g_lo + kMaxParts) * c.cspan) cnt = last / c.cspan - g_lo + 1;     // never with a plan that respects kMaxParts
    slot0 = g_lo + b; np = cnt;
}
__device__ __forceinline__ void piece_range(const PieceMap &m, int b, int &slot0, int &np)
{
    if (!m.E) { slot0 = b * m.parts; np = m.parts; return; }
    piece_range(m, piece_cut(m), b, m.E[b], m.E[b + 1], slot0, np);
}

// ---- problem description handed to the launchers ------------------------------------------
struct Problem {
    int B, beam, n, heads, d_m, d_k, hd, R;
    int dtype, out_dtype;
    const void *H;
    int64_t H_batch_stride;
    const int32_t *lengths;
    const void *queries;
    void *out;
};

// Workspace carve-up (device pointers into the caller's buffer).
struct Workspace {
    float *Qp;      // [B*beam, hd]                 a1 result: fp32 (generic) or fp16 (MFMA GEMMs), scaled
    void *ELQ;      // [B, Rpad, d_m]               fp32 (generic) or fp16 (MFMA core)
    float *Xp;      // [B, parts, Rpad, d_m]        un-normalised partial weighted sums
    float *ML;      // [B, parts, Rpad, 2]          running max and sum of each partial
    float *Xn;      // [B, R, d_m]                  merged, normalised weighted sums (generic path)
    float *A;       // [B*beam, hd]                 a6 result: fp32 (generic) or fp16 (MFMA GEMMs)
    int32_t *E;     // [B+1]                        prefix sum of tile counts (flattened cut of the MFMA core)
    int slots;      // pieces Xp and ML have room for (batch elements the workspace was laid out for x kMaxParts)
};

struct Weights {    // library-owned copies in the storage dtype
    void *Wq, *Wk, *Wv, *Wo, *bq;   // original layout (x . W form)
    void *WqT;                      // (W^Q)^T in the storage dtype (16-bit dtypes only)
    void *WkH, *WvT, *WoT;          // W^K, (W^V)^T, (W^O)^T in fp16 (converted from bf16 when needed)
    float *c_out;                   // [d_m] = b_o + b_v . W_o, fp32
    float *bk32, *bv32, *bo32;      // [h*d_k], [h*d_k], [d_m] in fp32 (zeros when absent): only the segment form reads them
};

} // namespace el

// The context behind the opaque handle.
struct el_attn_ctx {
    el_attn_config cfg;
    int hd;                 // heads * d_k
    int Rpad_max;           // max_beam*heads rounded up to a multiple of 64
    el::Weights w;
    void *ws_base;
    size_t ws_bytes;        // bound size
    size_t ws_need;         // required size
    int splits_override;    // 0 = automatic
    int nrg_override;       // 0 = automatic
    int use_mfma_core;      // MFMA attention core available for this (dtype, d_m)
    int use_mfma_gemm;      // MFMA projection GEMMs available for this (dtype, d_m, d_k)
    int device;
    int num_cus;            // compute units of that device
    // optional event pairs around the core kernel (measurement aid)
    hipEvent_t *ev;         // 2 * ev_cap events, or null
    int ev_cap, ev_used;
};

namespace el {

// generic (fp32 arithmetic) kernels -- generic_kernels.hip
hipError_t launch_cout(const el_attn_ctx *ctx, const void *bv, const void *bo, hipStream_t s);
hipError_t launch_qproj_generic(const el_attn_ctx *ctx, const Problem &p, const Workspace &ws, hipStream_t s);
hipError_t launch_elq_generic(const el_attn_ctx *ctx, const Problem &p, const float *Qp, float *elq, hipStream_t s);
hipError_t launch_core_generic(const el_attn_ctx *ctx, const Problem &p, const Workspace &ws, int parts, hipStream_t s);
hipError_t launch_merge_generic(const el_attn_ctx *ctx, const Problem &p, const Workspace &ws, int parts, int Rstride, hipStream_t s);
hipError_t launch_vproj_generic(const el_attn_ctx *ctx, const Problem &p, const Workspace &ws, hipStream_t s);
hipError_t launch_oproj_generic(const el_attn_ctx *ctx, const Problem &p, const Workspace &ws, const float *bias32, hipStream_t s);
hipError_t launch_vec_f32(int dtype, const void *src, float *dst, int n, hipStream_t s);
// segment form (decoder-only models): statistics + biased head outputs of one segment; merge of several
struct SegFinishArgs {
    const void *A;            // [rows, hd] fp16 or fp32: the segment's normalised head outputs without b^V
    const void *Qp;           // [rows, hd] fp16 or fp32: projected queries as a1 left them (scaled)
    const float *ML;          // [slot, Rstride, 2] statistics of the pieces (see PieceMap)
    PieceMap pm;
    const float *bk32, *bv32;
    float *seg_A, *seg_lse;
    int beam, heads, d_k, hd, Rstride;
    float ml_to_nat, c_to_nat; // factors that turn ML's maxima / the key-bias dot product into natural-log units
};
constexpr int kMaxSegments = 4;
struct SegMergeArgs {
    const float *A[kMaxSegments];
    const float *lse[kMaxSegments];
    void *A_out;              // [rows, hd] fp16 or fp32
    int nseg, heads, d_k, hd;
};
hipError_t launch_seg_finish(const SegFinishArgs &a, bool a_f16, bool qp_f16, int rows, hipStream_t s);
hipError_t launch_seg_merge(const SegMergeArgs &a, bool out_f16, int rows, hipStream_t s);

// MFMA attention core -- core_stream.hip (the kernel), core_mfma.hip (planning, launch, helpers)
struct CorePlan {
    int nrg;      // 16-row groups per workgroup (1 or 2)
    int nblocks;  // row blocks (workgroups sharing one H range)
    int Rs;       // padded row count of ELQ / partial buffers = nblocks * 16 * nrg
    int flat;     // 1: the tiles of all elements are cut as one list into G spans; 0: one workgroup per (element, row block)
    int G;        // spans (flat) or batch elements (not flat)
    int lfloor;   // flat: floor on the span length in tiles, so that no element has more than kMaxParts pieces
    int kcost;    // flat: what crossing into a new element costs a workgroup, in tiles (see PieceMap)
    int parts;    // most pieces per (batch element, row)
    int slots;    // piece slots the partial buffers must hold
};
// Arguments of the streaming core (core_stream.hip)
struct StreamArgs {
    const void *H;
    int64_t h_stride;        // elements between batch elements
    const int32_t *lengths;
    const uint16_t *elq;     // EL-Q as high + low 16-bit planes in the storage type, scaled by log2(e)/sqrt(d_k),
                             //   in fragment order (see elq_frag_index)
    f16_t *Xp;               // [slot, Rs, DM] fp16, each piece already divided by its own sum
    float *ML;               // [slot, Rs, 2]  (reference max in log2 units, sum)
    int32_t *E;              // [B+1] prefix sum of tile counts (flat cut), written by the kernel; may be null
    int n, B, R, Rs, nblocks;
    int flat, G, lfloor, kcost;
    int stream_hint;         // nonzero: fetch H with the non-temporal hint (H far larger than the memory-side cache)
};
hipError_t launch_core_stream(const StreamArgs &a, int d_m, bool bf16, int rg, hipStream_t s, hipEvent_t ev0, hipEvent_t ev1);
bool core_mfma_supported(int dtype, int d_m);
CorePlan plan_core_mfma(const Problem &p, int splits_override, int nrg_override, int num_cus, int max_slots);
PieceMap piece_map(const CorePlan &pl, const Workspace &ws, int B);
hipError_t launch_elq_f16(const el_attn_ctx *ctx, const Problem &p, const Workspace &ws, const CorePlan &pl, hipStream_t s);
hipError_t launch_core_mfma(const el_attn_ctx *ctx, const Problem &p, const Workspace &ws, const CorePlan &pl, hipStream_t s,
                            hipEvent_t ev0, hipEvent_t ev1);   // events, if given, bracket the kernel itself
hipError_t launch_merge_exp2(const el_attn_ctx *ctx, const Problem &p, const Workspace &ws, const CorePlan &pl, hipStream_t s);

// MFMA projection GEMMs -- gemm_mfma.hip
bool gemm_mfma_supported(int dtype, int d_m, int d_k);
hipError_t launch_transpose16(const void *src, void *dst, int rows, int cols, hipStream_t s);
hipError_t launch_bf16_to_f16(const void *src, void *dst, size_t n, hipStream_t s);
hipError_t launch_qproj_mfma(const el_attn_ctx *ctx, const Problem &p, const Workspace &ws, float scale, hipStream_t s);
hipError_t launch_elq_mfma(const el_attn_ctx *ctx, const Problem &p, const Workspace &ws, int Rs, hipStream_t s);
hipError_t launch_vproj_mfma(const el_attn_ctx *ctx, const Problem &p, const Workspace &ws, const CorePlan &pl, hipStream_t s);
hipError_t launch_oproj_mfma(const el_attn_ctx *ctx, const Problem &p, const Workspace &ws, const float *bias32, hipStream_t s);

} // namespace el
