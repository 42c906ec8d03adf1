/*
 * el_attn.h -- C ABI of the EL-attention incremental decode step for MI355X (gfx950).
 *
 * What the library computes.  For every batch element b (one matrix of hidden
 * states H_b with a valid prefix of lengths[b] positions) and every beam j (one
 * query vector), the multi-head attention output of appendix B, Eq. 6,
 *
 *     out[b,j] = sum_i softmax( Q_i K_i^T / sqrt(d_k) ) V_i W_i^O  (+ b^O),
 *     Q_i = q W_i^Q + b_i^Q,  K_i = H_b W_i^K + b_i^K,  V_i = H_b W_i^V + b_i^V,
 *
 * evaluated in the EL-attention order of Eq. 5 / Eq. 9: the query is expanded per
 * head to model width, EL-Q_i = Q_i (W_i^K)^T, scored directly against the
 * unprojected H_b, the probabilities are applied to H_b, and the result goes
 * through W_i^V and W_i^O (the seven steps of the EL "encoder_decoder_attention"
 * routine of appendix A, Algorithm 3).  No per-head key or value is ever built.
 * The key bias only adds a per-row constant to the scores and cancels in the
 * softmax; the value bias contributes sum_i b_i^V W_i^O because probabilities sum
 * to one (remark closing appendix B); the library uses both facts.
 *
 * Conventions
 *   - Every tensor pointer is a DEVICE pointer owned by the caller.  The library
 *     never frees caller memory and keeps no reference to H, lengths, queries or
 *     out after a call returns.  Weights are copied at prepare time.
 *   - Row-major everywhere.  Head i owns columns [i*d_k, (i+1)*d_k) of W^Q, W^K,
 *     W^V and rows [i*d_k, (i+1)*d_k) of W^O (the concatenation form noted under
 *     Eq. 2).  Weights are used as x . W (Eq. 2: W_i^{Q,K,V} in R^{d_m x d_k}).
 *   - Calls are asynchronous on the HIP stream passed in (`stream` is a
 *     hipStream_t cast to void*; NULL is the default stream).  Nothing
 *     synchronises.  el_attn_decode_step never allocates.
 *   - Errors are return codes.  Argument errors are found before any HIP call is
 *     made, so they can be exercised on a host without a GPU.
 *   - One GPU, one context per attention layer.  A context may be used from one
 *     stream at a time (its workspace is shared by its calls).
 */
#ifndef EL_ATTN_H
#define EL_ATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct el_attn_ctx el_attn_ctx; /* opaque, owned by the library */

typedef enum {
    EL_OK = 0,
    EL_ERR_INVALID_ARG = 1, /* null pointer, non-positive size, size beyond the prepared maxima */
    EL_ERR_UNSUPPORTED = 2, /* a shape or dtype no kernel covers (e.g. heads*d_k != d_model)     */
    EL_ERR_ALLOC = 3,       /* device or host allocation failed in prepare                       */
    EL_ERR_HIP = 4,         /* a HIP runtime call failed (no device, launch error)               */
    EL_ERR_WORKSPACE = 5    /* decode_step without a bound workspace, or one too small           */
} el_status;

typedef enum { EL_F32 = 0, EL_F16 = 1, EL_BF16 = 2 } el_dtype;

/* flags */
#define EL_FLAG_FORCE_GENERIC 1u /* run the plain fp32-arithmetic kernels even where an MFMA path exists */

typedef struct {
    int32_t heads;     /* h                                                         */
    int32_t d_model;   /* d_m                                                       */
    int32_t d_k;       /* per-head width; heads*d_k must equal d_model              */
    int32_t dtype;     /* el_dtype: storage type of H, queries, weights and biases  */
    int32_t out_dtype; /* el_dtype of `out`: EL_F32 or the same as `dtype`          */
    int32_t max_batch; /* largest B a decode_step call will pass                    */
    int32_t max_beam;  /* largest beam                                              */
    int32_t max_n;     /* largest padded key length n                               */
    uint32_t flags;    /* EL_FLAG_*                                                 */
} el_attn_config;

/*
 * Step a0 (once per attention layer, off the per-step path): take the layer's
 * projection weights, keep private packed copies, and fold the biases as the
 * closing remark of appendix B allows: c_out = b^O + sum_i b_i^V W_i^O (Eq. 8/9)
 * is computed here.  b^K cancels inside one softmax (Eq. 7) and the decode step
 * never reads it; only the segment form below, whose statistics are compared
 * across key sets, keeps it.
 *
 *   Wq, Wk, Wv  [d_model, heads*d_k]   device, `dtype`
 *   Wo          [heads*d_k, d_model]   device, `dtype`
 *   bq, bk, bv  [heads*d_k] or NULL    device, `dtype`
 *   bo          [d_model]   or NULL    device, `dtype`
 *
 * The copies are enqueued on `stream`; the caller may release its weights once
 * the stream has passed this point.  On success *out_ctx owns device memory
 * until el_attn_destroy.  Errors: INVALID_ARG (null cfg/weights/out_ctx, sizes
 * < 1), UNSUPPORTED (heads*d_k != d_model, unknown dtype, out_dtype neither
 * EL_F32 nor dtype), ALLOC, HIP.
 */
el_status el_attn_prepare(const el_attn_config *cfg,
                          const void *Wq, const void *bq,
                          const void *Wk, const void *bk,
                          const void *Wv, const void *bv,
                          const void *Wo, const void *bo,
                          void *stream, el_attn_ctx **out_ctx);

/*
 * Scratch memory one decode step needs at the prepared maxima (expanded
 * queries, split partials, projected rows).  The caller allocates at least
 * this many bytes of device memory, 256-byte aligned, and binds it; the
 * library neither frees it nor touches it outside decode_step /
 * expand_query.  Its contents need not be initialised.
 */
size_t el_attn_workspace_bytes(const el_attn_ctx *ctx);
el_status el_attn_bind_workspace(el_attn_ctx *ctx, void *dev_ptr, size_t bytes);

/*
 * One incremental decode step (steps a1..a7 of Algorithm 3's attention routine):
 *
 *   a1  Qp    = queries . W^Q + b^Q                              (per beam row)
 *   a2  EL-Q  = Qp_i . (W_i^K)^T / sqrt(d_k)   -> [B, heads*beam, d_model]   (Eq. 5)
 *   a3  S     = EL-Q . H_b^T   over t < lengths[b]                           (Eq. 9)
 *   a4  P     = softmax_t(S)   (fp32)                                        (Eq. 1)
 *   a5  X     = P . H_b                                  -> [B, heads*beam, d_model]
 *   a6  A     = X_i . W_i^V                              -> [B*beam, heads*d_k] (Eq. 5/8)
 *   a7  out   = A . W^O + c_out                          -> [B, beam, d_model]  (Eq. 2)
 *
 *   H        [B, n, d_model], row stride d_model, batch stride H_batch_stride
 *            ELEMENTS (>= n*d_model); device, `dtype`.  Rows t >= lengths[b] are
 *            never read; they may hold anything, NaN included.
 *   lengths  [B] int32 device, each in [1, n]; NULL means every row has length n.
 *            Values are not validated on the device; a value outside [1, n] is
 *            undefined behaviour of the caller.
 *   queries  [B, beam, d_model] contiguous, device, `dtype`.
 *   out      [B, beam, d_model] contiguous, device, `out_dtype`.
 *
 * Self-attention over a per-beam history is the same call with B := B*beam and
 * beam := 1 (section 3.1.1: the state is the previous layer's output, appended
 * by the caller before the call).
 *
 * Alignment: where el_attn_uses_mfma(ctx) is 1 the kernels move operands in
 * 16-byte pieces, so H, queries and out must be 16-byte aligned and
 * H_batch_stride * sizeof(element) a multiple of 16 (d_model is 512, 768 or
 * 1024 there, so rows are); on the generic path element alignment suffices.
 * lengths must be 4-byte aligned.  A violation is INVALID_ARG, found on the host
 * before any device work.  el_attn_decode_segment and el_attn_merge_segments
 * apply the same rules to their operands (their fp32 buffers: 4 bytes).
 *
 * Errors: INVALID_ARG (null ctx/H/queries/out; B, beam or n < 1 or beyond the
 * prepared maxima; H_batch_stride < n*d_model; misaligned operands),
 * WORKSPACE, HIP (launch failure).
 */
el_status el_attn_decode_step(el_attn_ctx *ctx,
                              const void *H, int64_t H_batch_stride,
                              const int32_t *lengths,
                              const void *queries,
                              void *out,
                              int32_t B, int32_t beam, int32_t n,
                              void *stream);

/*
 * Segment form of the step, for decoder-only models (section 3.2: EL-attention
 * over the part of the history every beam shares and ordinary attention over
 * each beam's own continuation, joined under ONE softmax).  A segment is one key
 * set scored by the same queries; el_attn_decode_segment runs a1..a6 on it and
 * returns, instead of the output row, what a joint softmax over several segments
 * needs, per query row m = b*beam + j and head i:
 *
 *   seg_A     [B*beam, heads*d_k]  float32, device: the segment's own head output
 *             sum_t p_t (H_t W_i^V + b_i^V) with p the softmax INSIDE the segment
 *             (Eq. 8 before W^O);
 *   seg_lse   [B*beam, heads]      float32, device: log sum_t exp(s_t) with
 *             s_t = Q_i (H_t W_i^K + b_i^K)^T / sqrt(d_k)  in natural-log units.
 *             The key-bias term of Eq. 7 is constant within a segment but is part
 *             of s, so this value is directly comparable with the log-sum-exp of
 *             any ordinary attention over projected keys (a per-beam cache a caller
 *             keeps for the generated suffix, or another segment of this library).
 *
 * el_attn_merge_segments joins 1..el_attn_max_segments() segments of the same
 * query rows and finishes the step:
 *
 *   w_s = exp(lse_s) / sum_s' exp(lse_s')   (evaluated relative to max_s lse_s),
 *   A = sum_s w_s seg_A_s,   out = A . W^O + b^O                 (Eq. 2)
 *
 * which equals multi-head attention over the union of the segments' keys.  The
 * segments may come from calls with different (B, beam) factorizations of the
 * same B*beam rows: a shared prefix as (B, beam) and a per-beam suffix as
 * (B*beam, 1) (section 3.1.1; the context must then have been prepared with
 * max_batch >= B*beam).  A segment whose lse is -inf is ignored.  seg_A and
 * seg_lse passed to merge are HOST arrays of nseg device pointers, read during
 * the call only.  Other arguments as for el_attn_decode_step.  Both calls use the
 * bound workspace and never allocate.
 *
 * Errors: as el_attn_decode_step, plus INVALID_ARG for null outputs, nseg outside
 * [1, el_attn_max_segments()] or a null segment pointer.
 */
el_status el_attn_decode_segment(el_attn_ctx *ctx,
                                 const void *H, int64_t H_batch_stride,
                                 const int32_t *lengths,
                                 const void *queries,
                                 float *seg_A, float *seg_lse,
                                 int32_t B, int32_t beam, int32_t n,
                                 void *stream);
el_status el_attn_merge_segments(el_attn_ctx *ctx, int32_t nseg,
                                 const float *const *seg_A,
                                 const float *const *seg_lse,
                                 void *out,
                                 int32_t B, int32_t beam,
                                 void *stream);
int32_t el_attn_max_segments(void);

/*
 * Diagnostic export of steps a1+a2 alone (Eq. 5, EL-Q_i = (Q W_i^Q + b_i^Q)(W_i^K)^T,
 * already divided by sqrt(d_k)):  elq_out [B, heads*beam, d_model] float32, device,
 * row r = i*beam + j holds head i of beam j.  Uses the bound workspace.
 */
el_status el_attn_expand_query(el_attn_ctx *ctx, const void *queries, float *elq_out,
                               int32_t B, int32_t beam, void *stream);

/*
 * Tuning knob, never semantics: about how many pieces per batch element the attention core
 * cuts the keys into (the MFMA core cuts the list of all valid 16-row tiles of a batch into
 * B x splits equal spans, one workgroup each per block of rows; the generic core cuts every
 * element into `splits` key ranges; partial results are merged with the log-sum-exp rule).
 * 0 restores the automatic choice.  Must not exceed el_attn_max_splits().
 */
el_status el_attn_set_splits(el_attn_ctx *ctx, int32_t splits);
int32_t el_attn_max_splits(void);

/*
 * Second tuning knob, never semantics: how many 16-row groups of expanded queries one
 * workgroup of the MFMA attention core owns (1 or 2; 0 restores the automatic choice, which
 * is 2 wherever the shape has more than 16 rows).  The row blocks of one span stream the
 * same H tiles (served by the shared L2 after the first touch).
 */
el_status el_attn_set_row_groups(el_attn_ctx *ctx, int32_t row_groups);

/*
 * What the automatic choice would be for a shape on a device with `compute_units` compute units (host
 * arithmetic only, no device needed): rows per workgroup in groups of 16 (*row_groups) and the number of
 * equal spans the list of valid tiles is cut into (*spans; workgroups = spans x row blocks) by the MFMA
 * attention core.  Errors: INVALID_ARG (null outputs, sizes < 1), UNSUPPORTED (d_model other than 512, 768 or
 * 1024: no MFMA core).
 */
el_status el_attn_plan_preview(int32_t B, int32_t beam, int32_t heads, int32_t d_model, int32_t n,
                               int32_t compute_units, int32_t *row_groups, int32_t *spans);

/*
 * el_attn_decode_step for callers that cannot allocate and have no workspace to bind: code running
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same operands, same
 * result and same checks as el_attn_decode_step, but the intermediates of the step live in a fixed array
 * of EL_ATTN_STATIC_SCRATCH_BYTES (32 MiB) that is part of the library's device code: every GPU the
 * library is used on holds one copy until the process ends, and no workspace needs to be bound.  The
 * call allocates nothing and only launches kernels.
 *
 * Limit: the intermediates of THIS call (about 41 bytes x B x R64 x d_model, R64 = heads * beam rounded
 * up to a multiple of 64) must fit the array; otherwise WORKSPACE is returned and nothing is launched
 * (at d_model = 1024, 16 heads, beam 4: B up to 12).  All calls on one GPU share that GPU's array,
 * whatever their context or stream: calls that overlap in time on one GPU race.  Nothing in the array
 * has to survive from call to call or start at zero.  The array's address on a device is resolved when
 * a context is prepared on that device.
 * Errors: as el_attn_decode_step; WORKSPACE as above; HIP if the array's address was not resolved.
 */
#define EL_ATTN_STATIC_SCRATCH_BYTES ((size_t)32 << 20)
el_status el_attn_decode_step_static(el_attn_ctx *ctx,
                                     const void *H, int64_t H_batch_stride, const int32_t *lengths,
                                     const void *queries, void *out,
                                     int32_t B, int32_t beam, int32_t n, void *stream);

/*
 * The operand checks of el_attn_decode_step (shapes against the configured maxima, strides, and the
 * alignment rules stated there) as host arithmetic on a configuration alone: no context, no device, no
 * pointer is dereferenced.  `mfma` says which path's rules apply (what el_attn_uses_mfma would return
 * for a context prepared from `cfg`).  Returns EL_OK, INVALID_ARG as decode_step would, or UNSUPPORTED
 * if `mfma` is nonzero for a (dtype, d_model) the MFMA kernels do not cover.  For callers that want to
 * validate buffers when they allocate them rather than on the first step.
 */
el_status el_attn_check_step_operands(const el_attn_config *cfg, int32_t mfma,
                                      const void *H, int64_t H_batch_stride, const int32_t *lengths,
                                      const void *queries, const void *out,
                                      int32_t B, int32_t beam, int32_t n);

/* 1 if decode_step on this context runs the MFMA kernels, 0 if the generic fp32 ones. */
int32_t el_attn_uses_mfma(const el_attn_ctx *ctx);

/*
 * Measurement aid for callers that cannot see inside a step (the benchmark): once enabled
 * with room for `max_steps` steps, every decode_step brackets its attention-core kernel
 * (steps a3-a5) with a pair of HIP events on the stream it was given (the MFMA core's launch
 * carries the pair itself, so it reads that dispatch's own begin and end).  read() waits for the
 * recorded events, writes the elapsed milliseconds of each step's core kernel to ms_out
 * (at most `capacity`), stores the number written in *count and forgets them.  Steps beyond
 * max_steps are not bracketed.  max_steps = 0 disables timing and releases the events.
 * Errors: INVALID_ARG (null ctx/ms_out/count, negative sizes), ALLOC, HIP.
 */
el_status el_attn_core_timing_enable(el_attn_ctx *ctx, int32_t max_steps);
el_status el_attn_core_timing_read(el_attn_ctx *ctx, float *ms_out, int32_t capacity, int32_t *count);

/*
 * State maintenance between decode steps (section 3.1.1 and the "reorder" cost the paper's
 * Algorithm 3 leaves to the caller): the state of EL-attention is the hidden states themselves,
 * so keeping it in step with the search is a gather of whole batch elements,
 *
 *     H_dst[i, 0:len, :] = H_src[index[i], 0:len, :],   len = lengths_src[index[i]],
 *     lengths_dst[i]     = len                                     for i < B_dst.
 *
 * With index = the batch elements that are still running it drops finished sentences
 * (encoder-decoder attention: one H per sentence, shared by its beams); with index = the parent
 * beam of every surviving beam it re-orders per-beam histories after a beam-search step
 * (self-attention, B := B*beam).  Only the valid prefix is read and written: rows at or beyond
 * len keep whatever H_dst held.
 *
 *   H_src     [B_src, n, d_model], row stride d_model, batch stride src_batch_stride ELEMENTS, device
 *   H_dst     [B_dst, n, d_model], batch stride dst_batch_stride ELEMENTS, device; must not overlap H_src
 *   lengths_src [B_src] int32 device or NULL (every element has length n)
 *   lengths_dst [B_dst] int32 device or NULL (not written)
 *   index     [B_dst] int32 device; an entry outside [0, B_src) leaves its destination untouched
 *             (and its lengths_dst entry at 0)
 *   dtype     element type of H (EL_F32, EL_F16, EL_BF16); d_model * element size must be a multiple of 16 bytes
 *
 * Asynchronous on `stream`, allocates nothing, needs no context.
 * Errors: INVALID_ARG (null H_src/H_dst/index, sizes < 1, strides < n*d_model, bad dtype, row bytes
 * not a multiple of 16, H pointers not 16-byte aligned), HIP (launch failure).
 */
el_status el_attn_gather_batch(el_dtype dtype, int32_t d_model,
                               const void *H_src, int64_t src_batch_stride, const int32_t *lengths_src, int32_t B_src,
                               void *H_dst, int64_t dst_batch_stride, int32_t *lengths_dst, int32_t B_dst,
                               const int32_t *index, int32_t n, void *stream);

/*
 * Diagnostic pass over the inputs of a decode step: what the step assumes and, living in device
 * memory, does not verify on its hot path.  One read of the valid rows of H (rows at or beyond a
 * length are not read; a length outside [0, n] is clamped for reading) fills
 *
 *   report[0]  lengths outside [1, n]          (section 3.1: a softmax over no position is undefined)
 *   report[1]  elements that are NaN or +-Inf
 *   report[2]  finite elements with |v| > 65504: the 16-bit MFMA path converts bf16 operands to
 *              fp16, which saturates beyond that magnitude (fp16 storage cannot hold such values)
 *   report[3]  elements examined = sum_b min(max(len_b, 0), n) * d_model
 *
 *   report   [4] uint64, DEVICE memory, 8-byte aligned; cleared and filled on `stream`.
 *   H, lengths, strides, dtype as for el_attn_gather_batch (16-byte alignment rules included).
 *
 * Context-free, asynchronous, allocates nothing.  Errors: INVALID_ARG (null H/report, unknown
 * dtype, sizes < 1, B > 65535, stride < n*d_model, alignment), HIP.
 */
el_status el_attn_check_inputs(el_dtype dtype, int32_t d_model,
                               const void *H, int64_t H_batch_stride, const int32_t *lengths,
                               int32_t B, int32_t n, uint64_t *report, void *stream);

/* Release the context and its packed weights (not the workspace, which the caller owns). */
el_status el_attn_destroy(el_attn_ctx *ctx);

const char *el_attn_status_string(el_status s);

/* Library version as major*10000 + minor*100 + patch. */
int32_t el_attn_version(void);

#ifdef __cplusplus
}
#endif
#endif /* EL_ATTN_H */
