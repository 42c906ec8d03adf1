// MFMA attention core for gfx950: steps a3-a5 of the EL-attention decode step (Algorithm 3's two
// products over the hidden states and the softmax between them; Eq. 9 with K = V = H).
//
// One workgroup (4 wavefronts, one per SIMD) owns a contiguous range of 32-row tiles of one
// batch element's H and up to 64 expanded-query rows.  Every H tile is pulled from HBM once,
// straight into LDS (global_load_lds, no registers in between), converted there to fp16 when the
// storage type is bf16, and then used twice from LDS:
//
//   S^T = H_tile . ELQ^T      v_mfma_f32_16x16x32_f16, A = H rows (ds_read_b128), B = ELQ (registers)
//   X^T += H_tile^T . P^T     same instruction, A = H columns (ds_read_b64_tr_b16 transposing
//                             reads), B = P (the score accumulators, exponentiated in place)
//
// Working on the transposes puts the query row in lane%16 for both products, so the softmax
// statistics, the probabilities and the output accumulators of a row all live in the same lanes
// and P never moves between lanes.  Scores arrive pre-multiplied by log2(e)/sqrt(d_k), so the
// softmax is exp2 of a difference; max and sum are kept per row in fp32, the running reference
// maximum is only advanced (and the accumulators rescaled) when it would grow by more than 2^10.
//
// Each wavefront keeps its 16 rows of ELQ (fp16) and its 16 x d_m fp32 accumulators in registers
// for the whole range.  With fewer than 64 rows the spare wavefronts take alternate tiles and
// produce partial results of their own; all partials (key-range splits and wavefront parities)
// are combined afterwards by the log-sum-exp merge.
#include <cstdlib>
#include "el_internal.h"

namespace el {

typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef _Float16 h2 __attribute__((ext_vector_type(2)));
typedef short s4 __attribute__((ext_vector_type(4)));
typedef float f4 __attribute__((ext_vector_type(4)));
typedef unsigned int u4 __attribute__((ext_vector_type(4)));
#define EL_LDS(T) __attribute__((address_space(3))) T
#define EL_GLOBAL(T) __attribute__((address_space(1))) T

constexpr int kTileRows = 32;
constexpr float kRescaleStep = 10.0f; // log2 units: probabilities stay below 2^10


__device__ __forceinline__ unsigned bf16x2_to_f16x2(unsigned x)
{
    const float lo = __uint_as_float(x << 16);
    const float hi = __uint_as_float(x & 0xffff0000u);
    return __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_pkrtz(lo, hi));
}

#ifdef EL_CORE_PROF
#define EL_PROF_DECL unsigned long long prof_t = clock64(), prof_acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
#define EL_PROF(i) { const unsigned long long now = clock64(); prof_acc[i] += now - prof_t; prof_t = now; }
#else
#define EL_PROF_DECL
#define EL_PROF(i)
#endif

template <int DM, bool BF16, int NRG>
__global__ void __launch_bounds__(256)
k_core_mfma(const CoreArgs a)
{
    constexpr int ROWB = DM * 2;                  // bytes per tile row (2-byte elements)
    constexpr int TILE_BYTES = kTileRows * ROWB;
    constexpr int PIECES_PER_ROW = ROWB / 1024;   // 1 KB LDS-DMA pieces per row (1 or 2)
    constexpr int CHUNKS_PER_THREAD = TILE_BYTES / 16 / 256;
    constexpr int KCH = DM / 32;                  // k-chunks of the score product
    constexpr int DB = DM / 16;                   // 16-column blocks of the output
    constexpr int TS = 4 / NRG;                   // wavefronts sharing a row group (tile parities)
    static_assert(ROWB % 1024 == 0 && PIECES_PER_ROW <= 2, "rows are fetched as one or two 1 KB pieces");

    // Two tile buffers.  A tile lands raw (storage dtype) in swizzled order, is converted to fp16 in
    // place when the storage type is bf16, and is then read by the MFMA phases.
    __shared__ __attribute__((aligned(1024))) char T[2 * TILE_BYTES];

    const int tid = threadIdx.x, l = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r16 = l & 15, g = l >> 4;

    // workgroup -> (batch element, key split, row block); workgroups that share an H range differ
    // by multiples of 8 so they are dispatched to the same XCD (same L2).
    const int id = blockIdx.x;
    const int oct = id / (8 * a.nblocks), rem = id % (8 * a.nblocks);
    const int rb = rem >> 3, group = oct * 8 + (rem & 7);
    if (group >= a.B * a.S) return;
    const int b = group / a.S, s = group % a.S;

    const int rg = w % NRG, tsel = w / NRG;
    const int row = rb * (16 * NRG) + 16 * rg + r16;   // expanded-query row of this lane

    int len = a.lengths ? a.lengths[b] : a.n;
    len = min(max(len, 1), a.n);
    const int NT = (len + kTileRows - 1) / kTileRows;
    const int k0 = (int)(((int64_t)NT * s) / a.S), k1 = (int)(((int64_t)NT * (s + 1)) / a.S);
    const int nloc = k1 - k0;

    const int parts = a.S * TS, part = s * TS + tsel;
    float *ml_out = a.ML + (((size_t)b * parts + part) * a.Rs + row) * 2;

    const char *Hb = (const char *)a.H + (size_t)b * a.h_stride * 2;

    // ---- ELQ rows of this wavefront: B operand of the score product ------------------------
    h8 elq[KCH];
    {
        // pad rows (row >= R) are never written by the expansion step: they read as zero here
        const f16_t *src = a.elq + ((size_t)b * a.Rs + row) * DM + 8 * g;
        const h8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
        for (int c = 0; c < KCH; ++c) elq[c] = row < a.R ? *(const h8 *)(src + 32 * c) : zero;
    }

    f4 X[DB];
#pragma unroll
    for (int i = 0; i < DB; ++i) X[i] = f4{0.f, 0.f, 0.f, 0.f};
    float m_ref = -INFINITY, l_sum = 0.f;

    // ---- per-lane LDS offsets inside a tile buffer -----------------------------------------
    const EL_LDS(char) *Tl = (const EL_LDS(char) *)T;
    const unsigned t_lds = (unsigned)(uintptr_t)Tl;
    int a_base[4]; // score product: row r16 (+16), chunk 4c+g
    {
        const int fx = row_swizzle(r16), cx = fx >> 2, gx = g ^ (fx & 3);
#pragma unroll
        for (int ci = 0; ci < 4; ++ci) a_base[ci] = r16 * ROWB + ((ci ^ cx) << 6) + (gx << 4);
    }
    int b_base[8]; // weighted sum: lane i=4k+q of block g reads row 4g+k (+16), columns 16db+4q..+3
    {
        const int k = r16 >> 2, q = r16 & 3, t_lo = 4 * g + k, ft = row_swizzle(t_lo);
#pragma unroll
        for (int di = 0; di < 8; ++di)
            b_base[di] = t_lo * ROWB + ((((2 * di) + (q >> 1)) ^ ft) << 4) + (q & 1) * 8;
    }

    // Fetch rows [i_begin, i_end) of this wavefront's share (rows 8w..8w+7) of tile kt into the buffer at
    // byte offset `buf`.  Lane i of a piece lands at physical chunk i and therefore fetches logical
    // chunk i ^ swizzle(row), so the tile arrives already in the bank-friendly order the MFMA phases
    // read (a permutation inside one 256-byte span: the global access stays fully coalesced).
    // Rows at or beyond len are not read.
    auto issue_dma_rows = [&](int kt, unsigned buf, int i_begin, int i_end) {
        const char *sbase = Hb + ((size_t)kt * kTileRows + 8 * w) * ROWB;
        const int rows_valid = len - (kt * kTileRows + 8 * w);      // wave-uniform
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            if (i < i_begin || i >= i_end) continue;
            const int f = (i << 1) | (w & 1);                        // row_swizzle(8w + i)
            const unsigned voff = (unsigned)(((l ^ f) << 4) + i * ROWB);
            const unsigned dst = t_lds + buf + (8 * w + i) * ROWB;
            if (i < rows_valid) {
                if (PIECES_PER_ROW == 2) dma_row_2k(dst, voff, sbase);
                else dma_piece(dst, voff, sbase);
            }
        }
    };
    auto issue_dma = [&](int kt, unsigned buf) { issue_dma_rows(kt, buf, 0, 8); };

    // Storage dtype -> fp16 in place (bf16 only) for tile kt_conv in `cbuf`, zero-fill of its rows at or
    // beyond len (ragged last tile: their bytes were never fetched and must not reach the MFMAs as
    // garbage), interleaved with the fetch requests of tile kt_dma into `dbuf`: the requests stall at
    // issue when the memory pipeline is busy, and that time is spent waiting for LDS data anyway.
    auto stage = [&](bool do_conv, int kt_conv, unsigned cbuf, bool do_dma, int kt_dma, unsigned dbuf) {
        const bool full = (kt_conv + 1) * kTileRows <= len;
        if (!do_conv || (!BF16 && full)) {
            if (do_dma) issue_dma(kt_dma, dbuf);
            return;
        }
        constexpr int NB = CHUNKS_PER_THREAD / 4;     // batches of four 16-byte chunks per thread
        constexpr int RPB = 8 / NB;                   // fetch rows issued per batch
        char *base = T + cbuf + tid * 16;
        u4 v[2][4];
#pragma unroll
        for (int e = 0; e < 4; ++e) v[0][e] = *(const u4 *)(base + e * 4096);
#pragma unroll
        for (int bi = 0; bi < NB; ++bi) {
            if (bi + 1 < NB) {
#pragma unroll
                for (int e = 0; e < 4; ++e) v[(bi + 1) & 1][e] = *(const u4 *)(base + (4 * (bi + 1) + e) * 4096);
            }
            if (do_dma) issue_dma_rows(kt_dma, dbuf, bi * RPB, (bi + 1) * RPB);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                u4 x = v[bi & 1][e];
                if (BF16) {
                    x.x = bf16x2_to_f16x2(x.x); x.y = bf16x2_to_f16x2(x.y);
                    x.z = bf16x2_to_f16x2(x.z); x.w = bf16x2_to_f16x2(x.w);
                }
                if (!full) {
                    const int trow = ((4 * bi + e) * 4096 + tid * 16) / ROWB;
                    if (kt_conv * kTileRows + trow >= len) x = u4{0u, 0u, 0u, 0u};
                }
                *(u4 *)(base + (4 * bi + e) * 4096) = x;
            }
        }
    };

    EL_PROF_DECL
    if (nloc > 0) {
        issue_dma(k0, 0);
        if (nloc > 1) issue_dma(k0 + 1, TILE_BYTES);
        // tile k0 must have landed; the fetches of tile k0+1 (issued later, completing in order) may still fly
        // (only when that tile is full, so that this wavefront issued exactly 8 rows of it)
        if (nloc > 1 && (k0 + 2) * kTileRows <= len) asm volatile("s_waitcnt vmcnt(%0)" :: "n"(8 * PIECES_PER_ROW) : "memory");
        else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        stage(true, k0, 0, false, 0, 0);
        __syncthreads();
    }
    // The compiler does not see the LDS-DMA requests; it does see the ELQ loads above, and would place
    // their wait (which also drains every later fetch) in front of the first MFMA of EVERY iteration.
    // Consuming the registers here, on every path into the loop, moves that wait out of it.
#pragma unroll
    for (int c = 0; c < KCH; ++c) asm volatile("" :: "v"(elq[c]));
    EL_PROF(0)

    for (int kk = 0; kk < nloc; ++kk) {
        const int kt = k0 + kk;
        const unsigned cur = (kk & 1) * TILE_BYTES, nxt = TILE_BYTES - cur;
        const EL_LDS(char) *Fl = Tl + cur;

        if (TS == 1 || (kk % TS) == tsel) {
        // ---- scores: S^T[t, r] for the 32 rows of the tile --------------------------------
        // Software-pipelined by hand in groups of two k-chunks: the LDS reads of the next group are
        // issued before the MFMAs of this one; the scheduling barriers keep the compiler from
        // hoisting every read to the top (which would spill the accumulators).
        f4 s0a = {0.f, 0.f, 0.f, 0.f}, s0b = s0a, s1a = s0a, s1b = s0a;
        {
            h8 hb[2][4];
            auto load_grp = [&](int cp, h8 *dst) {   // k-chunks 2cp, 2cp+1 for both 16-row halves
#pragma unroll
                for (int e = 0; e < 2; ++e) {
                    const int cidx = 2 * cp + e;
                    dst[e] = *(const EL_LDS(h8) *)(Fl + a_base[cidx & 3] + (cidx >> 2) * 256);
                    dst[2 + e] = *(const EL_LDS(h8) *)(Fl + a_base[cidx & 3] + (cidx >> 2) * 256 + 16 * ROWB);
                }
            };
            load_grp(0, hb[0]);
#pragma unroll
            for (int cp = 0; cp < KCH / 2; ++cp) {
                if (cp + 1 < KCH / 2) load_grp(cp + 1, hb[(cp + 1) & 1]);
                __builtin_amdgcn_sched_barrier(0);
                const h8 *hc = hb[cp & 1];
                s0a = __builtin_amdgcn_mfma_f32_16x16x32_f16(hc[0], elq[2 * cp + 0], s0a, 0, 0, 0);
                s1a = __builtin_amdgcn_mfma_f32_16x16x32_f16(hc[2], elq[2 * cp + 0], s1a, 0, 0, 0);
                s0b = __builtin_amdgcn_mfma_f32_16x16x32_f16(hc[1], elq[2 * cp + 1], s0b, 0, 0, 0);
                s1b = __builtin_amdgcn_mfma_f32_16x16x32_f16(hc[3], elq[2 * cp + 1], s1b, 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        EL_PROF(5)
        float sc[8];
#pragma unroll
        for (int j = 0; j < 4; ++j) { sc[j] = s0a[j] + s0b[j]; sc[4 + j] = s1a[j] + s1b[j]; }
        if ((kt + 1) * kTileRows > len) {   // last, ragged tile: positions at or beyond len do not exist
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int t = kt * kTileRows + 16 * (j >> 2) + 4 * g + (j & 3);
                if (t >= len) sc[j] = -INFINITY;
            }
        }

        // ---- softmax bookkeeping (row = lane%16; its 32 scores sit in 4 lanes x 8 registers) ----
        float mx = fmaxf(fmaxf(fmaxf(sc[0], sc[1]), fmaxf(sc[2], sc[3])),
                         fmaxf(fmaxf(sc[4], sc[5]), fmaxf(sc[6], sc[7])));
        mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        const bool grow = mx > m_ref + kRescaleStep;   // also true on the first tile (m_ref = -inf)
        if (__any(grow)) {
            const float alpha = grow ? __builtin_amdgcn_exp2f(m_ref - mx) : 1.0f;
            if (grow) m_ref = mx;
            l_sum *= alpha;
#pragma unroll
            for (int i = 0; i < DB; ++i) {
                // one accumulator tuple at a time through arch VGPRs; the empty asm statements pin
                // the register classes so the allocator does not move the whole array at once
                f4 t = X[i];
                asm volatile("" : "+v"(t));
                t[0] *= alpha; t[1] *= alpha; t[2] *= alpha; t[3] *= alpha;
                asm volatile("" : "+a"(t));
                X[i] = t;
            }
        }
        float pr[8];
        float psum = 0.f;
#pragma unroll
        for (int j = 0; j < 8; ++j) { pr[j] = __builtin_amdgcn_exp2f(sc[j] - m_ref); psum += pr[j]; }
        l_sum += psum;
        h8 P;   // round-to-nearest-even: an unbiased P keeps sum(P) and the weighted sum consistent
        {
            typedef float f2 __attribute__((ext_vector_type(2)));
            const h2 p01 = __builtin_convertvector(f2{pr[0], pr[1]}, h2), p23 = __builtin_convertvector(f2{pr[2], pr[3]}, h2);
            const h2 p45 = __builtin_convertvector(f2{pr[4], pr[5]}, h2), p67 = __builtin_convertvector(f2{pr[6], pr[7]}, h2);
            P = h8{p01[0], p01[1], p23[0], p23[1], p45[0], p45[1], p67[0], p67[1]};
        }
        EL_PROF(6)

        // ---- weighted sum: X^T[d, r] += sum_t H[t, d] P[r, t] ----------------------------------
        // Same hand pipelining, in groups of four 16-column blocks (8 transposing reads each).
        {
            typedef short s8 __attribute__((ext_vector_type(8)));
            s4 tb[2][8];
            auto load_grp = [&](int dq, s4 *dst) {    // 16-column blocks 4dq .. 4dq+3
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int db = 4 * dq + e;
                    dst[2 * e] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((EL_LDS(s4) *)(Fl + b_base[db & 7] + (db >> 3) * 256));
                    dst[2 * e + 1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((EL_LDS(s4) *)(Fl + b_base[db & 7] + (db >> 3) * 256 + 16 * ROWB));
                }
            };
            load_grp(0, tb[0]);
#pragma unroll
            for (int dq = 0; dq < DB / 4; ++dq) {
                if (dq + 1 < DB / 4) load_grp(dq + 1, tb[(dq + 1) & 1]);
                __builtin_amdgcn_sched_barrier(0);
                const s4 *tc = tb[dq & 1];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const s4 lo = tc[2 * e], hi = tc[2 * e + 1];
                    const h8 A = __builtin_bit_cast(h8, s8{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]});
                    X[4 * dq + e] = __builtin_amdgcn_mfma_f32_16x16x32_f16(A, P, X[4 * dq + e], 0, 0, 0);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        EL_PROF(7)
        }

        // Tile kt+1 was requested a whole period ago: drain this wavefront's share, then meet the others.
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();            // every wave is done reading `cur`; tile kt+1 has landed in `nxt`
        EL_PROF(1)
        // tile kt+2 is requested into `cur` (it flies during this conversion and the next tile's MFMAs)
        // while tile kt+1 is converted in `nxt`
        stage(kk + 1 < nloc, kt + 1, nxt, kk + 2 < nloc, kt + 2, cur);
        EL_PROF(2)
        __syncthreads();            // `nxt` is ready for the MFMA phases
        EL_PROF(3)
    }

    // ---- partial result of this wavefront -----------------------------------------------------
    l_sum += __shfl_xor(l_sum, 16, 64);
    l_sum += __shfl_xor(l_sum, 32, 64);
#ifdef EL_CORE_PROF
    if (blockIdx.x == 0 && threadIdx.x == 0 && a.prof) {
        for (int i = 0; i < 8; ++i) a.prof[i] = prof_acc[i];
        a.prof[8] = (unsigned long long)nloc;
    }
#endif
    if (row < a.R && g == 0) { ml_out[0] = m_ref; ml_out[1] = l_sum; }

    // The partial goes out normalised by its own sum, in fp16 (|x| <= max|H|; 2^-12 relative rounding,
    // far inside the error budget) and through LDS so that every global store instruction writes
    // 1 KB of one row: the partials are the largest write stream of the step.
    __syncthreads();                                   // all wavefronts are done with the tile buffers
    const bool had_tiles = TS == 1 ? nloc > 0 : nloc > tsel;
    if (had_tiles) {
        typedef float f2 __attribute__((ext_vector_type(2)));
        typedef _Float16 h4 __attribute__((ext_vector_type(4)));
        const float inv = 1.0f / l_sum;
        char *E = T + w * (16 * ROWB);                 // this wavefront's 16 x DM fp16 staging area
        // 8-byte units of a row are XOR-swizzled with the row number to spread the banks
#pragma unroll
        for (int db = 0; db < DB; ++db) {
            const f4 x = X[db];
            const h2 lo = __builtin_convertvector(f2{x[0] * inv, x[1] * inv}, h2);
            const h2 hi = __builtin_convertvector(f2{x[2] * inv, x[3] * inv}, h2);
            *(h4 *)(E + r16 * ROWB + (((4 * db + g) ^ r16) << 3)) = h4{lo[0], lo[1], hi[0], hi[1]};
        }
        const int row0 = rb * (16 * NRG) + 16 * rg;
        f16_t *x_out = a.Xp + (((size_t)b * parts + part) * a.Rs + row0) * DM;
#pragma unroll
        for (int rr = 0; rr < 16; ++rr) {
#pragma unroll
            for (int hf = 0; hf < DM / 512; ++hf) {
                if (row0 + rr >= a.R) continue;
                const int u0 = hf * 128 + 2 * l;
                const h4 v0 = *(const h4 *)(E + rr * ROWB + ((u0 ^ rr) << 3));
                const h4 v1 = *(const h4 *)(E + rr * ROWB + (((u0 + 1) ^ rr) << 3));
                *(h8 *)(x_out + (size_t)rr * DM + hf * 512 + 8 * l) = h8{v0[0], v0[1], v0[2], v0[3], v1[0], v1[1], v1[2], v1[3]};
            }
        }
    }
}

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

#ifdef EL_CORE_PROF
static unsigned long long *g_core_prof = nullptr;
extern "C" void el_attn_debug_set_prof(unsigned long long *p) { g_core_prof = p; }
#endif

// ---------------------------------------------------------------------------------------------
bool core_mfma_supported(int dtype, int d_m)
{
    return (dtype == EL_F16 || dtype == EL_BF16) && (d_m == 512 || d_m == 1024);
}

// Two attention-core kernels exist.  The column-split kernel (core_ds.hip) reads every tile byte from
// LDS only twice and has no per-wavefront partials, which wins when few rows share one H (greedy
// decoding, per-beam histories: 16 or 32 rows).  With 64 rows per H the row-split kernel below, with
// its larger tiles and fewer synchronisation points per byte, is still the faster one as measured.
// ELATTN_CORE=rows|cols forces one of them (tuning only).
static bool row_split_core(int R)
{
    static const char *force = getenv("ELATTN_CORE");
    if (force && force[0] == 'r') return true;
    if (force && force[0] == 'c') return false;
    return R > 32;
}

CorePlan plan_core_mfma(const Problem &p, int splits_override, int nrg_override)
{
    CorePlan pl;
    if (p.R <= 16) pl.nrg = 1;
    else if (p.R <= 32) pl.nrg = 2;
    else pl.nrg = 4;
    if (nrg_override > 0 && nrg_override < pl.nrg) pl.nrg = nrg_override;
    pl.nblocks = (p.R + 16 * pl.nrg - 1) / (16 * pl.nrg);
    pl.Rs = pl.nblocks * 16 * pl.nrg;
    const int ts = row_split_core(p.R) ? 4 / pl.nrg : 1;   // the column-split kernel has no per-wavefront partials
    const int max_s = kMaxParts / ts;
    int S = splits_override;
    if (S <= 0) {
        const long groups = (long)p.B * pl.nblocks;
        S = groups >= 256 ? 1 : (int)((256 + groups - 1) / groups);
        const int by_len = p.n / 64 > 0 ? p.n / 64 : 1;
        if (S > by_len) S = by_len;
    }
    if (S > max_s) S = max_s;
    if (S < 1) S = 1;
    pl.S = S;
    pl.parts = S * ts;
    return pl;
}

template <int DM, bool BF16>
static hipError_t launch_core_t(const CoreArgs &a, int nrg, hipStream_t s)
{
    const int groups = a.B * a.S;
    const dim3 grid(((groups + 7) / 8) * 8 * a.nblocks), block(256);
    switch (nrg) {
    case 1: hipLaunchKernelGGL((k_core_mfma<DM, BF16, 1>), grid, block, 0, s, a); break;
    case 2: hipLaunchKernelGGL((k_core_mfma<DM, BF16, 2>), grid, block, 0, s, a); break;
    default: hipLaunchKernelGGL((k_core_mfma<DM, BF16, 4>), grid, block, 0, s, a); break;
    }
    return hipGetLastError();
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
                            hipStream_t s)
{
    CoreArgs a;
    a.H = p.H; a.h_stride = p.H_batch_stride; a.lengths = p.lengths;
    a.elq = (const f16_t *)ws.ELQ; a.Xp = (f16_t *)ws.Xp; a.ML = ws.ML;
    a.n = p.n; a.B = p.B; a.R = p.R; a.Rs = pl.Rs; a.S = pl.S; a.nblocks = pl.nblocks;
#ifdef EL_CORE_PROF
    a.prof = g_core_prof;
#endif
    const bool bf = p.dtype == EL_BF16;
    if (!row_split_core(p.R)) return launch_core_ds(a, p.d_m, bf, pl.nrg, s);
    if (p.d_m == 1024) return bf ? launch_core_t<1024, true>(a, pl.nrg, s) : launch_core_t<1024, false>(a, pl.nrg, s);
    if (p.d_m == 512) return bf ? launch_core_t<512, true>(a, pl.nrg, s) : launch_core_t<512, false>(a, pl.nrg, s);
    return hipErrorInvalidValue;
}

hipError_t launch_merge_exp2(const el_attn_ctx *, const Problem &p, const Workspace &ws, const CorePlan &pl,
                             hipStream_t s)
{
    hipLaunchKernelGGL(k_merge_exp2, dim3((p.d_m + 255) / 256, p.R, p.B), dim3(256), 0, s,
                       (const f16_t *)ws.Xp, (const float *)ws.ML, ws.Xn, p.d_m, p.R, pl.Rs, pl.parts);
    return hipGetLastError();
}

} // namespace el
