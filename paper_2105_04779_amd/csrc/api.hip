// Host side of the C ABI declared in include/el_attn.h: argument validation, context and
// workspace bookkeeping, and the per-step launch sequence.  No kernel lives here.
#include <new>
#include <cmath>
#include <cstdlib>
#include <cstring>

#include "el_internal.h"

using namespace el;

// Scratch memory of el_attn_decode_step_static: every device the library's code object is loaded on holds its
// own copy of this array until the process ends.  In host code the name is only a handle for
// hipGetSymbolAddress; kernels get the resolved per-device address as an ordinary pointer argument.
constexpr size_t kStaticScratchBytes = EL_ATTN_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

constexpr int kMaxDevices = 64;
void *g_scratch_ptr[kMaxDevices];           // resolved address of `scratch` per device, null until resolved

// Resolve the array's address on `device` (which must be the current device).  Called from el_attn_prepare,
// so that the step itself finds it ready; returns null if the runtime cannot resolve it.
void *resolve_static_scratch(int device)
{
    if (device < 0 || device >= kMaxDevices) return nullptr;
    if (!g_scratch_ptr[device]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress((void **)&ptr, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
        g_scratch_ptr[device] = ptr;
    }
    return g_scratch_ptr[device];
}

void *static_scratch_of(int device) { return (device >= 0 && device < kMaxDevices) ? g_scratch_ptr[device] : nullptr; }

constexpr int32_t kVersion = 100; // 0.1.0

bool valid_dtype(int dt) { return dt == EL_F32 || dt == EL_F16 || dt == EL_BF16; }

int round_up64(int v) { return (v + 63) / 64 * 64; }

struct WsLayout {
    size_t off_Qp, off_ELQ, off_Xp, off_ML, off_Xn, off_A, off_E, total;
    int slots;
};

// Workspace of a step with at most `batch` batch elements of at most `beam` beams.
WsLayout ws_layout_for(const el_attn_ctx *c, int batch, int beam)
{
    const size_t mb = (size_t)batch, mx = (size_t)beam;
    const size_t d_m = (size_t)c->cfg.d_model, hd = (size_t)c->hd, Rp = (size_t)round_up64(c->cfg.heads * beam);
    WsLayout L;
    size_t o = 0;
    L.off_Qp = o;  o = align_up(o + mb * mx * hd * sizeof(float), 256);
    L.off_ELQ = o; o = align_up(o + mb * Rp * d_m * sizeof(float), 256);
    L.off_Xp = o;  o = align_up(o + mb * kMaxParts * Rp * d_m * sizeof(float), 256);
    L.off_ML = o;  o = align_up(o + mb * kMaxParts * Rp * 2 * sizeof(float), 256);
    L.off_Xn = o;  o = align_up(o + mb * Rp * d_m * sizeof(float), 256);
    L.off_A = o;   o = align_up(o + mb * mx * hd * sizeof(float), 256);
    L.off_E = o;   o = align_up(o + (mb + 1) * sizeof(int32_t), 256);
    L.total = o;
    L.slots = batch * kMaxParts;
    return L;
}

// Offsets of the bound workspace are those of the prepared maxima, so that it is valid for every smaller call.
WsLayout ws_layout(const el_attn_ctx *c) { return ws_layout_for(c, c->cfg.max_batch, c->cfg.max_beam); }

Workspace carve_from(void *ws_base, const WsLayout &L)
{
    char *base = (char *)ws_base;
    Workspace w;
    w.Qp = (float *)(base + L.off_Qp);
    w.ELQ = (void *)(base + L.off_ELQ);
    w.Xp = (float *)(base + L.off_Xp);
    w.ML = (float *)(base + L.off_ML);
    w.Xn = (float *)(base + L.off_Xn);
    w.A = (float *)(base + L.off_A);
    w.E = (int32_t *)(base + L.off_E);
    w.slots = L.slots;
    return w;
}

Workspace carve(const el_attn_ctx *c) { return carve_from(c->ws_base, ws_layout(c)); }

void free_weights(el_attn_ctx *c)
{
    void *ptrs[] = {c->w.Wq, c->w.Wk, c->w.Wv, c->w.Wo, c->w.bq, c->w.WqT, c->w.WkH, c->w.WvT, c->w.WoT, (void *)c->w.c_out,
                    (void *)c->w.bk32, (void *)c->w.bv32, (void *)c->w.bo32};
    for (void *p : ptrs)
        if (p) (void)hipFree(p);
    std::memset(&c->w, 0, sizeof(c->w));
}

// Number of key-range parts for the generic core: enough workgroups to occupy the chip
// when B*R is small, never more parts than 64-position slices of the shortest useful range.
int auto_parts_generic(const Problem &p)
{
    const long rows = (long)p.B * p.R;
    int parts = 1;
    if (rows < 1024) parts = (int)((1024 + rows - 1) / rows);
    const int by_len = p.n / 64 > 0 ? p.n / 64 : 1;
    if (parts > by_len) parts = by_len;
    if (parts > kMaxParts) parts = kMaxParts;
    return parts < 1 ? 1 : parts;
}

// The launchers report a failed launch through hipGetLastError(), which returns the last error ANY runtime call
// of this thread left behind, other libraries' included (a device probe that failed before the runtime was up,
// say).  Every entry point that launches starts from a clean slate.
void forget_foreign_errors() { (void)hipGetLastError(); }

bool aligned_to(const void *p, uintptr_t a) { return ((uintptr_t)p & (a - 1)) == 0; }

// Element alignment for every path; on the MFMA path operands are fetched and stored in 16-byte pieces.
uintptr_t operand_alignment(const el_attn_config &cfg, bool mfma) { return mfma ? 16 : dtype_size(cfg.dtype); }

// The shape and alignment rules of the queries (every call that takes them) ...
el_status check_queries(const el_attn_config &cfg, bool mfma, const void *queries, int32_t B, int32_t beam)
{
    if (!queries) return EL_ERR_INVALID_ARG;
    if (B < 1 || beam < 1) return EL_ERR_INVALID_ARG;
    if (B > cfg.max_batch || beam > cfg.max_beam) return EL_ERR_INVALID_ARG;
    if (!aligned_to(queries, operand_alignment(cfg, mfma))) return EL_ERR_INVALID_ARG;
    return EL_OK;
}

// ... and of the hidden states and their lengths
el_status check_hidden(const el_attn_config &cfg, bool mfma, const void *H, int64_t H_batch_stride, const int32_t *lengths, int32_t n)
{
    if (!H) return EL_ERR_INVALID_ARG;
    if (n < 1 || n > cfg.max_n) return EL_ERR_INVALID_ARG;
    if (H_batch_stride < (int64_t)n * cfg.d_model) return EL_ERR_INVALID_ARG;
    const uintptr_t al = operand_alignment(cfg, mfma);
    if (!aligned_to(H, al)) return EL_ERR_INVALID_ARG;
    if (((uint64_t)H_batch_stride * dtype_size(cfg.dtype)) % al != 0) return EL_ERR_INVALID_ARG;
    if (lengths && !aligned_to(lengths, sizeof(int32_t))) return EL_ERR_INVALID_ARG;
    return EL_OK;
}

el_status check_out(const el_attn_config &cfg, bool mfma, const void *out)
{
    if (!out) return EL_ERR_INVALID_ARG;
    return aligned_to(out, mfma ? 16 : dtype_size(cfg.out_dtype)) ? EL_OK : EL_ERR_INVALID_ARG;
}

el_status check_step_args(const el_attn_ctx *ctx, const void *queries, int32_t B, int32_t beam)
{
    if (!ctx) return EL_ERR_INVALID_ARG;
    return check_queries(ctx->cfg, el_attn_uses_mfma(ctx) != 0, queries, B, beam);
}

Problem make_problem(const el_attn_ctx *ctx, const void *H, int64_t stride, const int32_t *lengths,
                     const void *queries, void *out, int B, int beam, int n)
{
    Problem p;
    p.B = B; p.beam = beam; p.n = n;
    p.heads = ctx->cfg.heads; p.d_m = ctx->cfg.d_model; p.d_k = ctx->cfg.d_k; p.hd = ctx->hd;
    p.R = ctx->cfg.heads * beam;
    p.dtype = ctx->cfg.dtype; p.out_dtype = ctx->cfg.out_dtype;
    p.H = H; p.H_batch_stride = stride; p.lengths = lengths; p.queries = queries; p.out = out;
    return p;
}

// a1..a6 of one step; on return the workspace holds the projected queries, the key-range statistics and
// the head outputs A (without b^V), in the formats `fmt` names.
struct StepFormats {
    bool a_f16, qp_f16;     // element type of A and of the projected queries in the workspace
    PieceMap pm;            // which slots of the statistics [slot, Rstride, 2] belong to a batch element
    int Rstride;
    float ml_to_nat;        // ln 2 where the statistics' maxima are in log2 units
    float c_to_nat;         // ln 2 where the projected queries carry log2(e)
};

el_status run_a1_to_a6(el_attn_ctx *ctx, const Problem &p, const Workspace &ws, hipStream_t s, StepFormats *fmt)
{
    constexpr float kLn2 = 0.6931471805599453f;
    if (el_attn_uses_mfma(ctx)) {
        const CorePlan pl = plan_core_mfma(p, ctx->splits_override, ctx->nrg_override, ctx->num_cus, ws.slots);
        fmt->pm = piece_map(pl, ws, p.B); fmt->Rstride = pl.Rs; fmt->ml_to_nat = kLn2;
        // a1 + a2: expanded queries in fp16, pre-multiplied by log2(e)/sqrt(d_k) so the core's softmax is an exp2
        const float qscale = 1.4426950408889634f / sqrtf((float)p.d_k);
        if (ctx->use_mfma_gemm) {
            if (launch_qproj_mfma(ctx, p, ws, qscale, s) != hipSuccess) return EL_ERR_HIP;
            if (launch_elq_mfma(ctx, p, ws, pl.Rs, s) != hipSuccess) return EL_ERR_HIP;
        } else {
            if (launch_qproj_generic(ctx, p, ws, s) != hipSuccess) return EL_ERR_HIP;
            if (launch_elq_f16(ctx, p, ws, pl, s) != hipSuccess) return EL_ERR_HIP;
        }
        // a3-a5 on MFMA; key-range partials
        const bool timed = ctx->ev && ctx->ev_used < ctx->ev_cap;
        hipEvent_t ev0 = timed ? ctx->ev[2 * ctx->ev_used] : nullptr, ev1 = timed ? ctx->ev[2 * ctx->ev_used + 1] : nullptr;
        if (launch_core_mfma(ctx, p, ws, pl, s, ev0, ev1) != hipSuccess) return EL_ERR_HIP;
        if (timed) ctx->ev_used++;
        if (ctx->use_mfma_gemm) {
            // merge of the partials fused into a6
            if (launch_vproj_mfma(ctx, p, ws, pl, s) != hipSuccess) return EL_ERR_HIP;
            fmt->a_f16 = fmt->qp_f16 = true; fmt->c_to_nat = kLn2;
            return EL_OK;
        }
        if (launch_merge_exp2(ctx, p, ws, pl, s) != hipSuccess) return EL_ERR_HIP;
    } else {
        if (launch_qproj_generic(ctx, p, ws, s) != hipSuccess) return EL_ERR_HIP;
        if (launch_elq_generic(ctx, p, ws.Qp, (float *)ws.ELQ, s) != hipSuccess) return EL_ERR_HIP;
        const int parts = ctx->splits_override ? ctx->splits_override : auto_parts_generic(p);
        fmt->pm.E = nullptr; fmt->pm.parts = parts; fmt->pm.G = 0; fmt->pm.lfloor = 0; fmt->pm.B = p.B; fmt->pm.kcost = 0;
        fmt->Rstride = p.R; fmt->ml_to_nat = 1.f;
        const bool timed = ctx->ev && ctx->ev_used < ctx->ev_cap;
        if (timed && hipEventRecord(ctx->ev[2 * ctx->ev_used], s) != hipSuccess) return EL_ERR_HIP;
        if (launch_core_generic(ctx, p, ws, parts, s) != hipSuccess) return EL_ERR_HIP;
        if (timed) {
            if (hipEventRecord(ctx->ev[2 * ctx->ev_used + 1], s) != hipSuccess) return EL_ERR_HIP;
            ctx->ev_used++;
        }
        if (launch_merge_generic(ctx, p, ws, parts, p.R, s) != hipSuccess) return EL_ERR_HIP;
    }
    if (launch_vproj_generic(ctx, p, ws, s) != hipSuccess) return EL_ERR_HIP;
    fmt->a_f16 = fmt->qp_f16 = false; fmt->c_to_nat = 1.f;
    return EL_OK;
}

el_status run_a7(el_attn_ctx *ctx, const Problem &p, const Workspace &ws, const float *bias32, hipStream_t s)
{
    const hipError_t e = (el_attn_uses_mfma(ctx) && ctx->use_mfma_gemm) ? launch_oproj_mfma(ctx, p, ws, bias32, s)
                                                                       : launch_oproj_generic(ctx, p, ws, bias32, s);
    return e == hipSuccess ? EL_OK : EL_ERR_HIP;
}

el_status check_keys(const el_attn_ctx *ctx, const void *H, int64_t H_batch_stride, const int32_t *lengths, int32_t n)
{
    const el_status st = check_hidden(ctx->cfg, el_attn_uses_mfma(ctx) != 0, H, H_batch_stride, lengths, n);
    if (st != EL_OK) return st;
    if (!ctx->ws_base) return EL_ERR_WORKSPACE;
    return EL_OK;
}

} // namespace

extern "C" {

int32_t el_attn_version(void) { return kVersion; }

int32_t el_attn_max_splits(void) { return kMaxParts; }

const char *el_attn_status_string(el_status s)
{
    switch (s) {
    case EL_OK: return "ok";
    case EL_ERR_INVALID_ARG: return "invalid argument";
    case EL_ERR_UNSUPPORTED: return "unsupported shape or dtype";
    case EL_ERR_ALLOC: return "allocation failed";
    case EL_ERR_HIP: return "HIP runtime error";
    case EL_ERR_WORKSPACE: return "workspace missing or too small";
    default: return "unknown status";
    }
}

el_status el_attn_prepare(const el_attn_config *cfg,
                          const void *Wq, const void *bq, const void *Wk, const void *bk,
                          const void *Wv, const void *bv, const void *Wo, const void *bo,
                          void *stream, el_attn_ctx **out_ctx)
{
    if (out_ctx) *out_ctx = nullptr;
    if (!cfg || !out_ctx || !Wq || !Wk || !Wv || !Wo) return EL_ERR_INVALID_ARG;
    if (cfg->heads < 1 || cfg->d_model < 1 || cfg->d_k < 1) return EL_ERR_INVALID_ARG;
    if (cfg->max_batch < 1 || cfg->max_beam < 1 || cfg->max_n < 1) return EL_ERR_INVALID_ARG;
    if (!valid_dtype(cfg->dtype) || !valid_dtype(cfg->out_dtype)) return EL_ERR_UNSUPPORTED;
    if (cfg->out_dtype != EL_F32 && cfg->out_dtype != cfg->dtype) return EL_ERR_UNSUPPORTED;
    if ((int64_t)cfg->heads * cfg->d_k != cfg->d_model) return EL_ERR_UNSUPPORTED;
    if (cfg->d_model > kGenericMaxDm) return EL_ERR_UNSUPPORTED;
    if ((int64_t)cfg->heads * cfg->max_beam > 65535 || cfg->max_batch > 65535) return EL_ERR_UNSUPPORTED;

    el_attn_ctx *c = new (std::nothrow) el_attn_ctx;
    if (!c) return EL_ERR_ALLOC;
    std::memset(c, 0, sizeof(*c));
    c->cfg = *cfg;
    c->hd = cfg->heads * cfg->d_k;
    c->Rpad_max = round_up64(cfg->heads * cfg->max_beam);
    c->ws_need = ws_layout(c).total;
    c->use_mfma_core = core_mfma_supported(cfg->dtype, cfg->d_model) ? 1 : 0;

    hipStream_t s = (hipStream_t)stream;
    forget_foreign_errors();
    if (hipGetDevice(&c->device) != hipSuccess) { delete c; return EL_ERR_HIP; }
    if (hipDeviceGetAttribute(&c->num_cus, hipDeviceAttributeMultiprocessorCount, c->device) != hipSuccess || c->num_cus < 1) {
        delete c; return EL_ERR_HIP;
    }
    if (!resolve_static_scratch(c->device)) { delete c; return EL_ERR_HIP; }      // for el_attn_decode_step_static

    const size_t es = dtype_size(cfg->dtype);
    const size_t wbytes = (size_t)cfg->d_model * c->hd * es;
    struct { void **dst; const void *src; size_t bytes; } copies[] = {
        {&c->w.Wq, Wq, wbytes}, {&c->w.Wk, Wk, wbytes}, {&c->w.Wv, Wv, wbytes}, {&c->w.Wo, Wo, wbytes},
        {&c->w.bq, bq, (size_t)c->hd * es},
    };
    for (auto &cp : copies) {
        if (!cp.src) continue;
        if (hipMalloc(cp.dst, cp.bytes) != hipSuccess) { free_weights(c); delete c; return EL_ERR_ALLOC; }
        if (hipMemcpyAsync(*cp.dst, cp.src, cp.bytes, hipMemcpyDeviceToDevice, s) != hipSuccess) {
            free_weights(c); delete c; return EL_ERR_HIP;
        }
    }
    if (hipMalloc((void **)&c->w.c_out, (size_t)cfg->d_model * sizeof(float)) != hipSuccess) {
        free_weights(c); delete c; return EL_ERR_ALLOC;
    }
    if (launch_cout(c, bv, bo, s) != hipSuccess) { free_weights(c); delete c; return EL_ERR_HIP; }
    // fp32 copies of the three biases the segment form needs (b^K enters its statistics, Eq. 7)
    struct { float **dst; const void *src; int n; } vecs[] = {
        {&c->w.bk32, bk, c->hd}, {&c->w.bv32, bv, c->hd}, {&c->w.bo32, bo, cfg->d_model},
    };
    for (auto &v : vecs) {
        if (hipMalloc((void **)v.dst, (size_t)v.n * sizeof(float)) != hipSuccess) { free_weights(c); delete c; return EL_ERR_ALLOC; }
        if (launch_vec_f32(cfg->dtype, v.src, *v.dst, v.n, s) != hipSuccess) { free_weights(c); delete c; return EL_ERR_HIP; }
    }
    c->use_mfma_gemm = (c->use_mfma_core && gemm_mfma_supported(cfg->dtype, cfg->d_model, cfg->d_k)) ? 1 : 0;
    if (c->use_mfma_gemm) {
        // transposed copies so that every MFMA operand is contiguous along k; everything after a1 runs
        // in fp16, so bf16 weights of a2, a6, a7 are converted once here
        struct { void **dst; const void *src; int rows, cols; bool to_f16; } tr[] = {
            {&c->w.WqT, c->w.Wq, cfg->d_model, c->hd, false}, {&c->w.WvT, c->w.Wv, cfg->d_model, c->hd, true},
            {&c->w.WoT, c->w.Wo, c->hd, cfg->d_model, true},  {&c->w.WkH, c->w.Wk, 0, 0, true},
        };
        const size_t nel = (size_t)cfg->d_model * c->hd;
        for (auto &t : tr) {
            if (hipMalloc(t.dst, wbytes) != hipSuccess) { free_weights(c); delete c; return EL_ERR_ALLOC; }
            hipError_t e = t.rows ? launch_transpose16(t.src, *t.dst, t.rows, t.cols, s)
                                  : hipMemcpyAsync(*t.dst, t.src, wbytes, hipMemcpyDeviceToDevice, s);
            if (e == hipSuccess && t.to_f16 && cfg->dtype == EL_BF16) e = launch_bf16_to_f16(*t.dst, *t.dst, nel, s);
            if (e != hipSuccess) { free_weights(c); delete c; return EL_ERR_HIP; }
        }
    }

    *out_ctx = c;
    return EL_OK;
}

size_t el_attn_workspace_bytes(const el_attn_ctx *ctx) { return ctx ? ctx->ws_need : 0; }

el_status el_attn_bind_workspace(el_attn_ctx *ctx, void *dev_ptr, size_t bytes)
{
    if (!ctx || !dev_ptr) return EL_ERR_INVALID_ARG;
    if (((uintptr_t)dev_ptr & 255u) != 0) return EL_ERR_INVALID_ARG;
    if (bytes < ctx->ws_need) return EL_ERR_WORKSPACE;
    ctx->ws_base = dev_ptr;
    ctx->ws_bytes = bytes;
    return EL_OK;
}

el_status el_attn_set_splits(el_attn_ctx *ctx, int32_t splits)
{
    if (!ctx || splits < 0 || splits > kMaxParts) return EL_ERR_INVALID_ARG;
    ctx->splits_override = splits;
    return EL_OK;
}

el_status el_attn_set_row_groups(el_attn_ctx *ctx, int32_t row_groups)
{
    if (!ctx || (row_groups != 0 && row_groups != 1 && row_groups != 2)) return EL_ERR_INVALID_ARG;
    ctx->nrg_override = row_groups;
    return EL_OK;
}

el_status el_attn_plan_preview(int32_t B, int32_t beam, int32_t heads, int32_t d_model, int32_t n,
                               int32_t compute_units, int32_t *row_groups, int32_t *spans)
{
    if (!row_groups || !spans) return EL_ERR_INVALID_ARG;
    if (B < 1 || beam < 1 || heads < 1 || n < 1 || compute_units < 1) return EL_ERR_INVALID_ARG;
    if (!core_mfma_supported(EL_BF16, d_model)) return EL_ERR_UNSUPPORTED;
    Problem p;
    std::memset(&p, 0, sizeof(p));
    p.B = B; p.beam = beam; p.n = n; p.heads = heads; p.d_m = d_model; p.R = heads * beam;
    const CorePlan pl = plan_core_mfma(p, 0, 0, compute_units, B * kMaxParts);
    *row_groups = pl.nrg;
    *spans = pl.G;
    return EL_OK;
}

el_status el_attn_check_step_operands(const el_attn_config *cfg, int32_t mfma, const void *H, int64_t H_batch_stride,
                                      const int32_t *lengths, const void *queries, const void *out,
                                      int32_t B, int32_t beam, int32_t n)
{
    if (!cfg || !valid_dtype(cfg->dtype) || !valid_dtype(cfg->out_dtype) || cfg->d_model < 1) return EL_ERR_INVALID_ARG;
    if (mfma && !core_mfma_supported(cfg->dtype, cfg->d_model)) return EL_ERR_UNSUPPORTED;
    el_status st = check_queries(*cfg, mfma != 0, queries, B, beam);
    if (st != EL_OK) return st;
    if ((st = check_out(*cfg, mfma != 0, out)) != EL_OK) return st;
    return check_hidden(*cfg, mfma != 0, H, H_batch_stride, lengths, n);
}

int32_t el_attn_uses_mfma(const el_attn_ctx *ctx)
{
    return (ctx && ctx->use_mfma_core && !(ctx->cfg.flags & EL_FLAG_FORCE_GENERIC)) ? 1 : 0;
}

el_status el_attn_expand_query(el_attn_ctx *ctx, const void *queries, float *elq_out,
                               int32_t B, int32_t beam, void *stream)
{
    el_status st = check_step_args(ctx, queries, B, beam);
    if (st != EL_OK) return st;
    if (!elq_out) return EL_ERR_INVALID_ARG;
    if (!ctx->ws_base) return EL_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    forget_foreign_errors();
    const Workspace ws = carve(ctx);
    const Problem p = make_problem(ctx, nullptr, 0, nullptr, queries, nullptr, B, beam, 1);
    if (launch_qproj_generic(ctx, p, ws, s) != hipSuccess) return EL_ERR_HIP;
    if (launch_elq_generic(ctx, p, ws.Qp, elq_out, s) != hipSuccess) return EL_ERR_HIP;
    return EL_OK;
}

el_status el_attn_decode_step(el_attn_ctx *ctx, const void *H, int64_t H_batch_stride,
                              const int32_t *lengths, const void *queries, void *out,
                              int32_t B, int32_t beam, int32_t n, void *stream)
{
    el_status st = check_step_args(ctx, queries, B, beam);
    if (st != EL_OK) return st;
    if ((st = check_out(ctx->cfg, el_attn_uses_mfma(ctx) != 0, out)) != EL_OK) return st;
    if ((st = check_keys(ctx, H, H_batch_stride, lengths, n)) != EL_OK) return st;

    hipStream_t s = (hipStream_t)stream;
    forget_foreign_errors();
    const Workspace ws = carve(ctx);
    const Problem p = make_problem(ctx, H, H_batch_stride, lengths, queries, out, B, beam, n);
    StepFormats fmt;
    if ((st = run_a1_to_a6(ctx, p, ws, s, &fmt)) != EL_OK) return st;
    return run_a7(ctx, p, ws, ctx->w.c_out, s);
}

el_status el_attn_decode_step_static(el_attn_ctx *ctx, const void *H, int64_t H_batch_stride,
                                     const int32_t *lengths, const void *queries, void *out,
                                     int32_t B, int32_t beam, int32_t n, void *stream)
{
    el_status st = check_step_args(ctx, queries, B, beam);
    if (st != EL_OK) return st;
    if ((st = check_out(ctx->cfg, el_attn_uses_mfma(ctx) != 0, out)) != EL_OK) return st;
    if ((st = check_hidden(ctx->cfg, el_attn_uses_mfma(ctx) != 0, H, H_batch_stride, lengths, n)) != EL_OK) return st;
    // the workspace of THIS call's batch and beam count must fit the static array
    const WsLayout L = ws_layout_for(ctx, B, beam);
    if (L.total > kStaticScratchBytes) return EL_ERR_WORKSPACE;
    void *base = static_scratch_of(ctx->device);
    if (!base) return EL_ERR_HIP;

    hipStream_t s = (hipStream_t)stream;
    forget_foreign_errors();
    const Workspace ws = carve_from(base, L);
    const Problem p = make_problem(ctx, H, H_batch_stride, lengths, queries, out, B, beam, n);
    StepFormats fmt;
    if ((st = run_a1_to_a6(ctx, p, ws, s, &fmt)) != EL_OK) return st;
    return run_a7(ctx, p, ws, ctx->w.c_out, s);
}

el_status el_attn_decode_segment(el_attn_ctx *ctx, const void *H, int64_t H_batch_stride,
                                 const int32_t *lengths, const void *queries,
                                 float *seg_A, float *seg_lse,
                                 int32_t B, int32_t beam, int32_t n, void *stream)
{
    el_status st = check_step_args(ctx, queries, B, beam);
    if (st != EL_OK) return st;
    if (!seg_A || !seg_lse) return EL_ERR_INVALID_ARG;
    if (!aligned_to(seg_A, sizeof(float)) || !aligned_to(seg_lse, sizeof(float))) return EL_ERR_INVALID_ARG;
    if ((st = check_keys(ctx, H, H_batch_stride, lengths, n)) != EL_OK) return st;

    hipStream_t s = (hipStream_t)stream;
    forget_foreign_errors();
    const Workspace ws = carve(ctx);
    const Problem p = make_problem(ctx, H, H_batch_stride, lengths, queries, nullptr, B, beam, n);
    StepFormats fmt;
    if ((st = run_a1_to_a6(ctx, p, ws, s, &fmt)) != EL_OK) return st;
    SegFinishArgs f;
    f.A = ws.A; f.Qp = ws.Qp; f.ML = ws.ML; f.bk32 = ctx->w.bk32; f.bv32 = ctx->w.bv32;
    f.seg_A = seg_A; f.seg_lse = seg_lse;
    f.beam = beam; f.heads = p.heads; f.d_k = p.d_k; f.hd = p.hd; f.pm = fmt.pm; f.Rstride = fmt.Rstride;
    f.ml_to_nat = fmt.ml_to_nat; f.c_to_nat = fmt.c_to_nat;
    if (launch_seg_finish(f, fmt.a_f16, fmt.qp_f16, B * beam, s) != hipSuccess) return EL_ERR_HIP;
    return EL_OK;
}

el_status el_attn_merge_segments(el_attn_ctx *ctx, int32_t nseg, const float *const *seg_A,
                                 const float *const *seg_lse, void *out,
                                 int32_t B, int32_t beam, void *stream)
{
    if (!ctx || !seg_A || !seg_lse || !out) return EL_ERR_INVALID_ARG;
    if (nseg < 1 || nseg > kMaxSegments) return EL_ERR_INVALID_ARG;
    if (!aligned_to(out, (el_attn_uses_mfma(ctx) && ctx->use_mfma_gemm) ? 16 : dtype_size(ctx->cfg.out_dtype))) return EL_ERR_INVALID_ARG;
    if (B < 1 || beam < 1 || B > ctx->cfg.max_batch || beam > ctx->cfg.max_beam) return EL_ERR_INVALID_ARG;
    for (int i = 0; i < nseg; ++i)
        if (!seg_A[i] || !seg_lse[i] || !aligned_to(seg_A[i], sizeof(float)) || !aligned_to(seg_lse[i], sizeof(float))) return EL_ERR_INVALID_ARG;
    if (!ctx->ws_base) return EL_ERR_WORKSPACE;

    hipStream_t s = (hipStream_t)stream;
    forget_foreign_errors();
    const Workspace ws = carve(ctx);
    const Problem p = make_problem(ctx, nullptr, 0, nullptr, nullptr, out, B, beam, 1);
    const bool f16_path = el_attn_uses_mfma(ctx) && ctx->use_mfma_gemm;
    SegMergeArgs m;
    for (int i = 0; i < kMaxSegments; ++i) {
        m.A[i] = i < nseg ? seg_A[i] : nullptr;
        m.lse[i] = i < nseg ? seg_lse[i] : nullptr;
    }
    m.A_out = ws.A; m.nseg = nseg; m.heads = p.heads; m.d_k = p.d_k; m.hd = p.hd;
    if (launch_seg_merge(m, f16_path, B * beam, s) != hipSuccess) return EL_ERR_HIP;
    return run_a7(ctx, p, ws, ctx->w.bo32, s);   // b^V is already inside every segment's A
}

int32_t el_attn_max_segments(void) { return kMaxSegments; }

static void free_events(el_attn_ctx *ctx)
{
    if (ctx->ev) {
        for (int i = 0; i < 2 * ctx->ev_cap; ++i)
            if (ctx->ev[i]) (void)hipEventDestroy(ctx->ev[i]);
        std::free(ctx->ev);
    }
    ctx->ev = nullptr;
    ctx->ev_cap = ctx->ev_used = 0;
}

el_status el_attn_core_timing_enable(el_attn_ctx *ctx, int32_t max_steps)
{
    if (!ctx || max_steps < 0 || max_steps > (1 << 20)) return EL_ERR_INVALID_ARG;
    free_events(ctx);
    if (max_steps == 0) return EL_OK;
    ctx->ev = (hipEvent_t *)std::calloc((size_t)2 * max_steps, sizeof(hipEvent_t));
    if (!ctx->ev) return EL_ERR_ALLOC;
    ctx->ev_cap = max_steps;
    for (int i = 0; i < 2 * max_steps; ++i)
        if (hipEventCreate(&ctx->ev[i]) != hipSuccess) { free_events(ctx); return EL_ERR_HIP; }
    return EL_OK;
}

el_status el_attn_core_timing_read(el_attn_ctx *ctx, float *ms_out, int32_t capacity, int32_t *count)
{
    if (!ctx || !ms_out || !count || capacity < 0) return EL_ERR_INVALID_ARG;
    *count = 0;
    const int n = ctx->ev_used < capacity ? ctx->ev_used : capacity;
    for (int i = 0; i < n; ++i) {
        if (hipEventSynchronize(ctx->ev[2 * i + 1]) != hipSuccess) return EL_ERR_HIP;
        if (hipEventElapsedTime(&ms_out[i], ctx->ev[2 * i], ctx->ev[2 * i + 1]) != hipSuccess) return EL_ERR_HIP;
    }
    *count = n;
    ctx->ev_used = 0;
    return EL_OK;
}

el_status el_attn_destroy(el_attn_ctx *ctx)
{
    if (!ctx) return EL_ERR_INVALID_ARG;
    free_events(ctx);
    free_weights(ctx);
    delete ctx;
    return EL_OK;
}

} // extern "C"
