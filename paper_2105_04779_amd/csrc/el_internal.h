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

static inline size_t dtype_size(int dt) { return dt == EL_F32 ? 4 : 2; }
static inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// ---- compile-time limits -----------------------------------------------------------------
constexpr int kMaxParts = 8;        // key-range partials per (batch element, row) the workspace holds
constexpr int kGenericMaxDm = 8192; // widest d_model the generic core kernel covers

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
    float *Qp;      // [B*beam, hd]                 a1 result, fp32, already scaled by 1/sqrt(d_k)
    void *ELQ;      // [B, Rpad, d_m]               fp32 (generic) or fp16 (MFMA core)
    float *Xp;      // [B, parts, Rpad, d_m]        un-normalised partial weighted sums
    float *ML;      // [B, parts, Rpad, 2]          running max and sum of each partial
    float *Xn;      // [B, R, d_m]                  merged, normalised weighted sums (generic path)
    float *A;       // [B*beam, hd]                 a6 result, fp32
};

struct Weights {    // library-owned copies in the storage dtype
    void *Wq, *Wk, *Wv, *Wo, *bq;   // original layout (x . W form)
    void *WqT, *WvT, *WoT;          // transposed copies for the MFMA GEMMs (16-bit dtypes only)
    float *c_out;                   // [d_m] = b_o + b_v . W_o, fp32
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
hipError_t launch_oproj_generic(const el_attn_ctx *ctx, const Problem &p, const Workspace &ws, hipStream_t s);

// MFMA attention core -- core_mfma.hip
struct CorePlan {
    int nrg;      // 16-row groups per workgroup (1, 2 or 4)
    int nblocks;  // row blocks (workgroups sharing one H range)
    int Rs;       // padded row count of ELQ / partial buffers = nblocks * 16 * nrg
    int S;        // contiguous key-range splits per batch element
    int parts;    // partial results per (batch element, row) = S * 4 / nrg
};
bool core_mfma_supported(int dtype, int d_m);
CorePlan plan_core_mfma(const Problem &p, int splits_override, int nrg_override);
hipError_t launch_elq_f16(const el_attn_ctx *ctx, const Problem &p, const Workspace &ws, const CorePlan &pl, hipStream_t s);
hipError_t launch_core_mfma(const el_attn_ctx *ctx, const Problem &p, const Workspace &ws, const CorePlan &pl, hipStream_t s);
hipError_t launch_merge_exp2(const el_attn_ctx *ctx, const Problem &p, const Workspace &ws, const CorePlan &pl, hipStream_t s);

// MFMA projection GEMMs -- gemm_mfma.hip
bool gemm_mfma_supported(int dtype, int d_m, int d_k);
hipError_t launch_transpose16(const void *src, void *dst, int rows, int cols, hipStream_t s);
hipError_t launch_qproj_mfma(const el_attn_ctx *ctx, const Problem &p, const Workspace &ws, float scale, hipStream_t s);
hipError_t launch_elq_mfma(const el_attn_ctx *ctx, const Problem &p, const Workspace &ws, int Rs, hipStream_t s);
hipError_t launch_vproj_mfma(const el_attn_ctx *ctx, const Problem &p, const Workspace &ws, int parts, int Rs, hipStream_t s);
hipError_t launch_oproj_mfma(const el_attn_ctx *ctx, const Problem &p, const Workspace &ws, hipStream_t s);

} // namespace el
