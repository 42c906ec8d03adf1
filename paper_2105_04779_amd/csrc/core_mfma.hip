// Planning and launch of the MFMA attention core (steps a3-a5 of the EL-attention decode step; the
// kernel itself is in core_stream.hip), plus the two small fp32-FMA kernels that stand in for the MFMA
// projections around it when the head size is not 64: the query expansion as a high + low pair of
// 16-bit planes (in the fragment order the core loads) and the log-sum-exp merge of the pieces.
#include <cmath>
#include <cstdlib>
#include "el_internal.h"

namespace el {

// a2 for the MFMA core: EL-Q pre-multiplied by log2(e) (Qp already carries 1/sqrt(d_k)), as a high and a
// low plane in the storage type.
template <typename T, bool BF16>
__global__ void k_elq_planes(const float *__restrict__ Qp, const T *__restrict__ Wk, uint16_t *__restrict__ planes,
                             int beam, int d_m, int d_k, int hd, int R, int Rs)
{
    const int d = blockIdx.x * 256 + threadIdx.x;
    const int r = blockIdx.y, b = blockIdx.z;
    if (d >= d_m) return;
    const int i = r / beam, j = r % beam;   // Qp carries 1/sqrt(d_k) only on this path
    const float *qp = Qp + ((size_t)b * beam + j) * hd + (size_t)i * d_k;
    const T *wk = Wk + (size_t)d * hd + (size_t)i * d_k;
    float acc = 0.f;
    for (int c = 0; c < d_k; ++c) acc = fmaf(qp[c], to_f32(wk[c]), acc);
    acc *= 1.4426950408889634f;
    split16<BF16>(acc, planes[elq_frag_index(b, r, d, 0, Rs, d_m)], planes[elq_frag_index(b, r, d, 1, Rs, d_m)]);
}

// Log-sum-exp merge of normalised fp16 pieces (reference maxima in log2 units):
// X = sum_p (w_p l_p) Xhat_p / sum_p (w_p l_p),  w_p = 2^(m_p - M).
__global__ void k_merge_exp2(const f16_t *__restrict__ Xp, const float *__restrict__ ML, float *__restrict__ Xn,
                             int d_m, int R, int Rs, const PieceMap pm)
{
    const int d = blockIdx.x * 256 + threadIdx.x;
    const int r = blockIdx.y, b = blockIdx.z;
    if (d >= d_m) return;
    int slot0, np;
    piece_range(pm, b, slot0, np);
    float M = -INFINITY;
    for (int p = 0; p < np; ++p) {
        const size_t rowi = ((size_t)slot0 + p) * Rs + r;
        if (ML[rowi * 2 + 1] > 0.f) M = fmaxf(M, ML[rowi * 2]);
    }
    float num = 0.f, den = 0.f;
    for (int p = 0; p < np; ++p) {
        const size_t rowi = ((size_t)slot0 + p) * Rs + r;
        const float mp = ML[rowi * 2], lp = ML[rowi * 2 + 1];
        if (lp > 0.f) {
            const float wgt = exp2f(mp - M) * lp;
            num = fmaf(wgt, (float)Xp[rowi * d_m + d], num);
            den += wgt;
        }
    }
    Xn[((size_t)b * R + r) * d_m + d] = num / den;
}


// ---------------------------------------------------------------------------------------------
bool core_mfma_supported(int dtype, int d_m)
{
    return (dtype == EL_F16 || dtype == EL_BF16) && (d_m == 512 || d_m == 768 || d_m == 1024);
}

// How the work is cut.  A workgroup takes 16 or 32 of the R = heads x beams rows that share one H (the
// row blocks of one span read the same tiles, the second one from L2) and one span of the list of all
// valid 16-row tiles.  Lengths live on the device, so the host fixes only the number of spans G: one
// workgroup per compute unit when the longest possible list gives every span at least kMinSpan tiles,
// fewer otherwise (but not fewer than one span per batch element); the kernel derives the span length from the actual lengths.  The floor on the span
// length keeps every element within kMaxParts pieces.  Batches beyond kScanMax elements are not cut as
// one list: one workgroup per (element, row block), scheduled by the hardware.
constexpr int kMinSpan = 8;
// What moving on to the next batch element costs a workgroup, in tiles of streaming time: the expanded queries of
// the new element (128 KB for 32 rows) and the write-out of the finished piece.  Spans that cross an element hold
// that many tiles fewer, so that all workgroups finish together (measured on 64 ragged inputs of 512-1024 rows:
// workgroups with a crossing ended 5-6 us after the others).
constexpr int kBoundaryCost = 4;

CorePlan plan_core_mfma(const Problem &p, int splits_override, int nrg_override, int num_cus, int max_slots)
{
    CorePlan pl;
    pl.nrg = p.R <= 16 ? 1 : 2;
    if (nrg_override == 1) pl.nrg = 1;
    pl.nblocks = (p.R + 16 * pl.nrg - 1) / (16 * pl.nrg);
    pl.Rs = pl.nblocks * 16 * pl.nrg;
    const int tiles = (p.n + 15) / 16;
    pl.flat = p.B <= kScanMax && max_slots - p.B >= 1 ? 1 : 0;
    if (!pl.flat) {
        pl.G = p.B; pl.lfloor = tiles; pl.kcost = 0; pl.parts = 1; pl.slots = p.B;
        return pl;
    }
    long G;
    if (splits_override > 0) {
        G = (long)p.B * splits_override;                   // about that many pieces per element
    } else {
        const long by_cu = num_cus / pl.nblocks > 0 ? num_cus / pl.nblocks : 1;
        long by_len = (long)p.B * tiles / kMinSpan > 0 ? (long)p.B * tiles / kMinSpan : 1;
        // short inputs: a span per batch element rather than spans of kMinSpan tiles that each cross into a second
        // element and fetch its expanded queries as well (B = 64, n = 64: 16 instead of 23 us)
        const long per_elem = p.B < by_cu ? p.B : by_cu;
        if (by_len < per_elem) by_len = per_elem;
        G = by_cu < by_len ? by_cu : by_len;
    }
    if (G > max_slots - p.B) G = max_slots - p.B;
    if (G < 1) G = 1;
    pl.G = (int)G;
    pl.lfloor = (tiles + kMaxParts - 2) / (kMaxParts - 1);
    pl.kcost = kBoundaryCost;
    pl.parts = kMaxParts;
    pl.slots = pl.G + p.B;
    return pl;
}

PieceMap piece_map(const CorePlan &pl, const Workspace &ws, int B)
{
    PieceMap m;
    m.E = pl.flat ? ws.E : nullptr;
    m.parts = 1; m.G = pl.G; m.lfloor = pl.lfloor; m.B = B; m.kcost = pl.kcost;
    return m;
}

hipError_t launch_elq_f16(const el_attn_ctx *ctx, const Problem &p, const Workspace &ws, const CorePlan &pl,
                          hipStream_t s)
{
    const dim3 grid((p.d_m + 255) / 256, p.R, p.B), block(256);
    uint16_t *planes = (uint16_t *)ws.ELQ;
    if (p.dtype == EL_F16)
        hipLaunchKernelGGL((k_elq_planes<f16_t, false>), grid, block, 0, s, (const float *)ws.Qp, (const f16_t *)ctx->w.Wk,
                           planes, p.beam, p.d_m, p.d_k, p.hd, p.R, pl.Rs);
    else
        hipLaunchKernelGGL((k_elq_planes<bf16_t, true>), grid, block, 0, s, (const float *)ws.Qp, (const bf16_t *)ctx->w.Wk,
                           planes, p.beam, p.d_m, p.d_k, p.hd, p.R, pl.Rs);
    return hipGetLastError();
}

hipError_t launch_core_mfma(const el_attn_ctx *, const Problem &p, const Workspace &ws, const CorePlan &pl,
                            hipStream_t s, hipEvent_t ev0, hipEvent_t ev1)
{
    StreamArgs a;
    a.H = p.H; a.h_stride = p.H_batch_stride; a.lengths = p.lengths;
    a.elq = (const uint16_t *)ws.ELQ;
    a.Xp = (f16_t *)ws.Xp; a.ML = ws.ML; a.E = pl.flat ? ws.E : nullptr;
    a.n = p.n; a.B = p.B; a.R = p.R; a.Rs = pl.Rs; a.nblocks = pl.nblocks;
    a.flat = pl.flat; a.G = pl.G; a.lfloor = pl.lfloor; a.kcost = pl.kcost;
    // H is read once per step; when a batch of it is larger than the 256 MB memory-side cache, keeping its lines
    // out of the caches leaves them to the data that is re-read and raises the streaming rate (measured, core
    // kernel: 1 GB of per-beam histories 216 -> 184 us; 640 MB shared by two row blocks 149 -> 144 us).  Below
    // that it costs: the second row block of a span then misses what the first one fetched (128 MB: 42.7 -> 44.6 us).
    a.stream_hint = (double)p.B * p.n * p.d_m * 2.0 >= 256.0 * 1024 * 1024 ? 1 : 0;
    return launch_core_stream(a, p.d_m, p.dtype == EL_BF16, pl.nrg, s, ev0, ev1);
}

hipError_t launch_merge_exp2(const el_attn_ctx *, const Problem &p, const Workspace &ws, const CorePlan &pl,
                             hipStream_t s)
{
    hipLaunchKernelGGL(k_merge_exp2, dim3((p.d_m + 255) / 256, p.R, p.B), dim3(256), 0, s,
                       (const f16_t *)ws.Xp, (const float *)ws.ML, ws.Xn, p.d_m, p.R, pl.Rs, piece_map(pl, ws, p.B));
    return hipGetLastError();
}

} // namespace el
