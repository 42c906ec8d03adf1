// Planning and launch of the MFMA attention core (steps a3-a5 of the EL-attention decode step; the
// kernel itself is in core_ds.hip), plus the two small fp32-FMA kernels that stand in for the MFMA
// projections around it when the head size is not 64: the query expansion in fp16 and the
// log-sum-exp merge of the key-range partials.
#include <cmath>
#include <cstdlib>
#include "el_internal.h"

namespace el {

// a2 for the MFMA core: EL-Q in fp16, pre-multiplied by log2(e) (Qp already carries 1/sqrt(d_k)),
// rows padded with zeros up to Rs.
template <typename T>
__global__ void k_elq_f16(const float *__restrict__ Qp, const T *__restrict__ Wk, f16_t *__restrict__ elq,
                          int beam, int d_m, int d_k, int hd, int R, int Rs)
{
    const int d = blockIdx.x * 256 + threadIdx.x;
    const int r = blockIdx.y, b = blockIdx.z;
    if (d >= d_m) return;
    float acc = 0.f;
    if (r < R) {
        const int i = r / beam, j = r % beam;   // Qp carries 1/sqrt(d_k) only on this path
        const float *qp = Qp + ((size_t)b * beam + j) * hd + (size_t)i * d_k;
        const T *wk = Wk + (size_t)d * hd + (size_t)i * d_k;
        for (int c = 0; c < d_k; ++c) acc = fmaf(qp[c], to_f32(wk[c]), acc);
        acc *= 1.4426950408889634f;
    }
    elq[((size_t)b * Rs + r) * d_m + d] = (f16_t)acc;
}

// Log-sum-exp merge of normalised fp16 partials (reference maxima in log2 units):
// X = sum_p (w_p l_p) Xhat_p / sum_p (w_p l_p),  w_p = 2^(m_p - M).
__global__ void k_merge_exp2(const f16_t *__restrict__ Xp, const float *__restrict__ ML, float *__restrict__ Xn,
                             int d_m, int R, int Rs, int parts)
{
    const int d = blockIdx.x * 256 + threadIdx.x;
    const int r = blockIdx.y, b = blockIdx.z;
    if (d >= d_m) return;
    float M = -INFINITY;
    for (int p = 0; p < parts; ++p) {
        const size_t rowi = ((size_t)b * parts + p) * Rs + r;
        if (ML[rowi * 2 + 1] > 0.f) M = fmaxf(M, ML[rowi * 2]);
    }
    float num = 0.f, den = 0.f;
    for (int p = 0; p < parts; ++p) {
        const size_t rowi = ((size_t)b * parts + p) * Rs + r;
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
    return (dtype == EL_F16 || dtype == EL_BF16) && (d_m == 512 || d_m == 1024);
}

// How the work is cut.  A workgroup takes 16, 32 or 64 of the R = heads x beams rows that share one H
// (row groups of 16) and one of S key ranges; one workgroup runs per compute unit at a time.  Fewer rows per
// workgroup mean more workgroups without any partial results, but H is pulled from L2 once per row block;
// more key ranges mean more partial results to write and to merge.  Lengths live on the device, so the plan
// is made for the longest possible input.  It minimises a cost model fitted to measurements on MI355X
// (d_m = 1024, microseconds; tile terms scale with d_m):
//     rounds * (F + ceil(tiles / S) * t_tile) + S * t_merge ,        rounds = ceil(workgroups / CUs)
//     F       = 14.5 + 0.7 S | 11.5 + 0.3 S | 10.5 + 0.15 S          set-up, expanded-query fetch, write-out
//     t_tile  = max(compute 1.28 | 1.10 | 1.05,                      for 64 | 32 | 16 rows
//                   1.40 * distinct tiles in flight / 256,           HBM: 256 tiles of 32 KB per 1.4 us (ragged batches)
//                   1.05 * workgroups in flight / 256)               L2 -> compute units
//     t_merge = 1.1 per 8.4 MB of partial rows (B * rows * d_m fp16)
CorePlan plan_core_mfma(const Problem &p, int splits_override, int nrg_override, int num_cus)
{
    int nrg_max = p.R <= 16 ? 1 : (p.R <= 32 ? 2 : 4);
    const double wide = p.d_m / 1024.0;
    const double tiles = (p.n + 15) / 16;
    double best = 0.0;
    CorePlan pl;
    pl.nrg = 0;
    for (int nrg = nrg_max; nrg >= 1; nrg >>= 1) {
        if (nrg_override > 0 && nrg != (nrg_override < nrg_max ? nrg_override : nrg_max)) continue;
        const int nblocks = (p.R + 16 * nrg - 1) / (16 * nrg);
        const int Rs = nblocks * 16 * nrg;
        const double groups = (double)p.B * nblocks;
        const double f0 = nrg == 4 ? 14.5 : (nrg == 2 ? 11.5 : 10.5), f1 = nrg == 4 ? 0.7 : (nrg == 2 ? 0.3 : 0.15);
        const double t_c = (nrg == 4 ? 1.28 : (nrg == 2 ? 1.10 : 1.05)) * wide;
        const double t_merge = 1.1 * ((double)p.B * Rs * p.d_m) / (64.0 * 64.0 * 1024.0);
        for (int c = 1; c <= kMaxParts; ++c) {
            if (splits_override > 0 && c != splits_override) continue;
            if (splits_override <= 0 && c > 1 && tiles / c < 4.0) break;   // shorter ranges are not worth a workgroup
            const double wgs = groups * c;
            const double rounds = ceil(wgs / num_cus);
            const double active = wgs < num_cus ? wgs : num_cus;
            double t_tile = t_c;
            t_tile = fmax(t_tile, 1.40 * wide * (active / nblocks) / 256.0);
            t_tile = fmax(t_tile, 1.05 * wide * active / 256.0);
            const double t = rounds * ((f0 + f1 * c) * (0.5 + 0.5 * wide) + ceil(tiles / c) * t_tile) + c * t_merge;
            if (pl.nrg == 0 || t < best) {
                best = t;
                pl.nrg = nrg; pl.nblocks = nblocks; pl.Rs = Rs; pl.S = c;
            }
        }
    }
    if (pl.nrg == 0) {   // an override outside what the shape allows: fall back to the widest block, no cut
        pl.nrg = nrg_max; pl.nblocks = (p.R + 16 * nrg_max - 1) / (16 * nrg_max); pl.Rs = pl.nblocks * 16 * nrg_max; pl.S = 1;
    }
    pl.parts = pl.S;
    return pl;
}

hipError_t launch_elq_f16(const el_attn_ctx *ctx, const Problem &p, const Workspace &ws, const CorePlan &pl,
                          hipStream_t s)
{
    const dim3 grid((p.d_m + 255) / 256, pl.Rs, p.B), block(256);
    if (p.dtype == EL_F16)
        hipLaunchKernelGGL((k_elq_f16<f16_t>), grid, block, 0, s, (const float *)ws.Qp, (const f16_t *)ctx->w.Wk,
                           (f16_t *)ws.ELQ, p.beam, p.d_m, p.d_k, p.hd, p.R, pl.Rs);
    else
        hipLaunchKernelGGL((k_elq_f16<bf16_t>), grid, block, 0, s, (const float *)ws.Qp, (const bf16_t *)ctx->w.Wk,
                           (f16_t *)ws.ELQ, p.beam, p.d_m, p.d_k, p.hd, p.R, pl.Rs);
    return hipGetLastError();
}

hipError_t launch_core_mfma(const el_attn_ctx *, const Problem &p, const Workspace &ws, const CorePlan &pl,
                            hipStream_t s, hipEvent_t ev0, hipEvent_t ev1)
{
    CoreArgs a;
    a.H = p.H; a.h_stride = p.H_batch_stride; a.lengths = p.lengths;
    a.elq = (const f16_t *)ws.ELQ; a.Xp = (f16_t *)ws.Xp; a.ML = ws.ML;
    a.n = p.n; a.B = p.B; a.R = p.R; a.Rs = pl.Rs; a.S = pl.S; a.nblocks = pl.nblocks;
    // H is read once per step; when a batch of it is large against the 256 MB memory-side cache, keeping its
    // lines out of the caches leaves them to the data that is re-read and raises the streaming rate (measured:
    // 5.3 -> 6.2 TB/s on 1 GB of per-beam histories; 0.5 us per step at 128 MB; slower on a 25 MB batch)
    a.stream_hint = (double)p.B * p.n * p.d_m * 2.0 >= 128.0 * 1024 * 1024 ? 1 : 0;
    const bool bf = p.dtype == EL_BF16;
    return launch_core_ds(a, p.d_m, bf, pl.nrg, s, ev0, ev1);
}

hipError_t launch_merge_exp2(const el_attn_ctx *, const Problem &p, const Workspace &ws, const CorePlan &pl,
                             hipStream_t s)
{
    hipLaunchKernelGGL(k_merge_exp2, dim3((p.d_m + 255) / 256, p.R, p.B), dim3(256), 0, s,
                       (const f16_t *)ws.Xp, (const float *)ws.ML, ws.Xn, p.d_m, p.R, pl.Rs, pl.parts);
    return hipGetLastError();
}

} // namespace el
