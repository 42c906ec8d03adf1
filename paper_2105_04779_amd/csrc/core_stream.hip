// MFMA attention core for gfx950, steps a3-a5 of the EL-attention decode step (Algorithm 3's two
// products over the hidden states and the softmax between them; Eq. 9 with K = V = H).
//
// The valid 16-row tiles of all batch elements form one list (element 0's tiles, then element 1's,
// ...).  The list is cut into G equal spans; a workgroup walks one span for one block of 16 or 32
// expanded-query rows, so every compute unit streams the same number of bytes whatever the lengths
// are.  Where a span crosses from one batch element to the next the workgroup closes a PIECE: it
// writes that element's partial result (normalised by its own sum, with the softmax statistics) to
// slot `span + element` and goes on with the next element without draining its pipeline; a6 merges
// an element's pieces by the log-sum-exp rule.  An element that lies inside one span has one piece
// and needs no merge.
//
// On this hardware an LDS instruction holds its wavefront for about as long as an MFMA does (~32
// clocks), and a wavefront issues in order, so the work of a tile is spread over eight wavefronts,
// two per SIMD, with two roles of about equal issue time:
//
//   score wavefronts (0..3)   own a quarter of the model dimension for all rows of the workgroup.
//       S^T[t, r] partial over those columns: 16x16x32 MFMA in the STORAGE type, A = H rows (one
//       ds_read_b128 feeds the MFMAs of both row groups and both planes), B = the wavefront's slice of
//       EL-Q held in registers as a high + low pair of 16-bit values, so a score keeps ~16 mantissa
//       bits however peaked the softmax is, and bf16 H enters the MFMA as it is.  The four partials
//       meet in LDS; one step later each score wavefront sums them for a quarter of the rows and does
//       the softmax bookkeeping in fp32 (running reference maximum, advanced only when it would grow
//       by more than 2^10), then publishes P (fp16, or a high + low bf16 pair), the rescale factors
//       and, where a piece ends, 1/sum.
//   sum wavefronts (4..7)     own a quarter of the model dimension: X^T[d, r] += H^T[d, t] P^T[t, r],
//       32x32x16 MFMA, A = H columns through the transposing LDS read (ds_read_b64_tr_b16), B = P from
//       LDS, fp32 accumulators.  They also request the tiles: each 1 KB piece of a tile row goes
//       straight from HBM into one of four LDS tile slots (global_load_lds), across piece boundaries
//       as well.  Lane i of a 1 KB piece fetches chunk i ^ swizzle(row), which keeps both operand read
//       patterns spread over all banks.
//
// One barrier per tile.  In step i the scores of tile i, the softmax of tile i-1 and the weighted sum
// of tile i-2 run side by side; the sum wavefronts take tile i's column fragments into registers in
// the same step, so a slot is read in one step only: one tile is resident, three are in flight.
// Scores arrive pre-multiplied by log2(e)/sqrt(d_k), so the softmax is an exp2 of a difference.
#include <type_traits>
#include <hip/hip_ext.h>
#include "el_internal.h"

namespace el {

typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef _Float16 h4 __attribute__((ext_vector_type(4)));
typedef _Float16 h2 __attribute__((ext_vector_type(2)));
typedef __bf16 b8 __attribute__((ext_vector_type(8)));
typedef short s4 __attribute__((ext_vector_type(4)));
typedef short s8 __attribute__((ext_vector_type(8)));
typedef float f2 __attribute__((ext_vector_type(2)));
typedef float f4 __attribute__((ext_vector_type(4)));
typedef float f16v __attribute__((ext_vector_type(16)));
typedef unsigned int u4 __attribute__((ext_vector_type(4)));
typedef unsigned int u2 __attribute__((ext_vector_type(2)));
#define EL_LDS(T) __attribute__((address_space(3))) T

namespace {

constexpr int kTile = 16;                 // rows of H per tile
constexpr float kRescaleStep = 10.0f;     // log2 units: probabilities stay below 2^10
constexpr float kMasked = -1.0e30f;       // score of a position that does not exist: finite, exp2 of it is 0

// chunk swizzle of a 16-row tile: the two bit pairs of the row number swapped.  A bijection on
// four bits (row-wise b128 reads of 16 rows hit 16 different chunk positions) whose upper pair
// runs over all four values inside {8g + k} and {8g + 4 + k}, k = 0..3 (the row sets one
// transposing read touches), so those reads use every bank exactly twice.
__device__ __forceinline__ int tile_swizzle(int row) { return ((row & 3) << 2) | ((row >> 2) & 3); }

// butterfly over the four lanes of a quad on the VALU (DPP quad_perm), no LDS round trip
__device__ __forceinline__ float quad_xor1(float v) { return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0xB1, 0xF, 0xF, true)); }
__device__ __forceinline__ float dpp_half_mirror(float v) { return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x141, 0xF, 0xF, true)); }   // lane i <-> 7 - i of each 8
__device__ __forceinline__ float dpp_row_mirror(float v) { return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x140, 0xF, 0xF, true)); }    // lane i <-> 15 - i of each 16
__device__ __forceinline__ float quad_xor2(float v) { return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x4E, 0xF, 0xF, true)); }

template <bool BF16> struct Mma;
template <> struct Mma<false> {
    static __device__ __forceinline__ f4 s16(u4 a, u4 b, f4 c) { return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(h8, a), __builtin_bit_cast(h8, b), c, 0, 0, 0); }
    static __device__ __forceinline__ f16v s32(u4 a, u4 b, f16v c) { return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(h8, a), __builtin_bit_cast(h8, b), c, 0, 0, 0); }
};
template <> struct Mma<true> {
    static __device__ __forceinline__ f4 s16(u4 a, u4 b, f4 c) { return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(b8, a), __builtin_bit_cast(b8, b), c, 0, 0, 0); }
    static __device__ __forceinline__ f16v s32(u4 a, u4 b, f16v c) { return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(b8, a), __builtin_bit_cast(b8, b), c, 0, 0, 0); }
};

__device__ __forceinline__ int wave_sum(int v)
{
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o, 64);
    return __builtin_amdgcn_readfirstlane(v);
}

} // namespace

template <int DM, bool BF16, int RG, bool NT>
__global__ void __launch_bounds__(512)
k_core_stream(const StreamArgs a)
{
    constexpr int ROWB = DM * 2;                    // bytes per tile row (2-byte elements)
    constexpr int SLOT = kTile * ROWB;              // one tile
    constexpr int NSLOT = 4;
    constexpr int PIECES = ROWB / 1024;             // 1 KB LDS-DMA pieces per row (rows of 1 or 2 KB)
    constexpr bool LIN = ROWB % 1024 != 0;          // rows of 1.5 KB: a wavefront's four rows are fetched as one 6 KB block
    constexpr int NI = 4 * ROWB / 1024;             // fetch instructions per sum wavefront per tile (four rows)
    constexpr int CPR = ROWB / 16;                  // 16-byte chunks per row
    constexpr int CHK = DM / 128;                   // 32-column chunks of one score wavefront (a quarter of the columns)
    constexpr int DS = DM / 4;                      // columns per sum wavefront
    constexpr int MB = DS / 32;                     // 32-column blocks of the output per sum wavefront
    constexpr int NP = BF16 ? 2 : 1;                // 16-bit planes of P
    constexpr int ROWS = 16 * RG;                   // expanded-query rows of this workgroup
    constexpr int SXP = ROWS * 16;                  // floats of one part of one exchange buffer [row][position]
    constexpr int SXB = 4 * SXP;                    // one exchange buffer (four column parts)
    constexpr int TPL = RG;                         // positions per softmax lane
    constexpr int LPR = 16 / TPL;                   // softmax lanes per row
    constexpr int RPW = 64 / LPR;                   // rows whose softmax one score wavefront does (= ROWS / 4)
    static_assert(DM == 512 || DM == 768 || DM == 1024, "d_m is 512, 768 or 1024");
    static_assert(LIN ? NI == DM / 128 : true, "one block fetch per 32-column block of a sum wavefront");
    static_assert(RG == 1 || RG == 2, "row groups per workgroup");

    __shared__ __attribute__((aligned(1024))) char T[NSLOT * SLOT];
    __shared__ __attribute__((aligned(16))) float Sx[2 * SXB];                // partial scores [tile parity][part][row][position]
    __shared__ __attribute__((aligned(16))) uint16_t Px[2 * NP * 32 * 16];    // probabilities [tile parity][plane][row][position]
    __shared__ float Ax[2 * 32];                                              // per-row rescale factor [tile parity][row]
    __shared__ float Linv[2 * 32];                                            // per-row 1/sum of a piece [parity of its last tile][row]
    __shared__ __attribute__((aligned(1024))) char Dz[ROWB];                  // where fetches of rows that do not exist land
    __shared__ int Lt[kScanMax];                                              // clamped lengths of all batch elements (flattened cut)

    const int tid = threadIdx.x, l = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r16 = l & 15, g = l >> 4, r32 = l & 31, kg = l >> 5;

    // workgroup -> (span, row block).  Workgroup ids that differ by a multiple of 8 run on the same XCD (same L2);
    // the row blocks of one span, which read the same tiles, and neighbouring spans, which share expanded queries,
    // get consecutive places on one XCD.
    const int nwg = a.G * a.nblocks;
    const int per_xcd = (nwg + 7) >> 3;
    const int place = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (place >= nwg) return;
    const int span = place / a.nblocks, rb = place % a.nblocks;   // (the piece slots are span + element: see PieceMap)
    const int row0 = rb * ROWS;                      // first expanded-query row of this workgroup

    auto clamp_len = [&](int v) { return min(max(v, 1), a.n); };

    // ---- where this span starts: element b0, tile kt0 of it, nspan tiles in all ----
    int b0, kt0, nspan, len0;
    if (a.flat) {
        // Tiles on the cost axis (see PieceMap): element b starts at E[b] + kcost * b with a gap of kcost units, then
        // its tiles.  This span is [c0, c1) of that axis.
        for (int i = tid; i < a.B; i += 512) Lt[i] = clamp_len(a.lengths ? a.lengths[i] : a.n);
        __syncthreads();
        int part = 0;
        for (int i = l; i < a.B; i += 64) part += (Lt[i] + kTile - 1) / kTile;
        const int total = wave_sum(part);
        const int cspan = flat_cspan(total, a.B, a.G, a.lfloor, a.kcost);
        const int c0 = span * cspan, c1 = min(c0 + cspan, total + a.kcost * a.B);
        const bool writer = place == 0 && w == 0 && a.E != nullptr;       // one wavefront publishes the prefix for a6
        if (writer && l == 0) a.E[0] = 0;
        // tiles_before(c): tiles at coordinates below c; for c0 also the element and tile the span starts at
        b0 = -1; kt0 = 0;
        int t_lo = 0, t_hi = -1, run = 0;                                 // run: tiles of the chunks already scanned
        for (int c = 0; c * 64 < a.B; ++c) {
            const int i = c * 64 + l;
            const int mine = i < a.B ? (Lt[i] + kTile - 1) / kTile : 0;
            int inc = mine;
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                const int up = __shfl_up(inc, o, 64);
                if (l >= o) inc += up;
            }
            inc += run;                                                   // tiles of elements 0..i
            if (writer && i < a.B) a.E[i + 1] = inc;
            const int cend = inc + a.kcost * (i + 1);                    // one past the last coordinate of element i
            // the first element that ends beyond c0 holds the span's first tile (or the gap before its tiles)
            const int n0 = __builtin_popcountll(__ballot(i < a.B && cend <= c0));
            if (b0 < 0 && n0 < 64 && c * 64 + n0 < a.B) {
                b0 = c * 64 + n0;
                const int tiles_b = __shfl(mine, n0, 64), end_b = __shfl(cend, n0, 64);
                kt0 = max(c0 - (end_b - tiles_b), 0);                     // coordinate of its tile 0 is end_b - tiles_b
                t_lo = __shfl(inc, n0, 64) - tiles_b + kt0;
            }
            const int n1 = __builtin_popcountll(__ballot(i < a.B && cend <= c1));
            if (t_hi < 0 && n1 < 64 && c * 64 + n1 < a.B) {
                const int tiles_b = __shfl(mine, n1, 64), end_b = __shfl(cend, n1, 64);
                t_hi = __shfl(inc, n1, 64) - tiles_b + max(c1 - (end_b - tiles_b), 0);
            }
            run = __shfl(inc, 63, 64);
        }
        if (t_hi < 0) t_hi = total;                                      // c1 is the end of the axis
        b0 = __builtin_amdgcn_readfirstlane(b0);
        kt0 = __builtin_amdgcn_readfirstlane(kt0);
        nspan = __builtin_amdgcn_readfirstlane(t_hi - t_lo);
        if (nspan <= 0 || b0 < 0) return;            // the axis is shorter than G spans of the floor length, or the span is all gap
        len0 = __builtin_amdgcn_readfirstlane(Lt[b0]);
    } else {
        b0 = span; kt0 = 0;
        len0 = __builtin_amdgcn_readfirstlane(clamp_len(a.lengths ? a.lengths[b0] : a.n));
        nspan = (len0 + kTile - 1) / kTile;
    }
    // length of an element the span moves on to (only the flattened cut crosses elements)
    auto next_len = [&](int b) -> int { return __builtin_amdgcn_readfirstlane(a.flat && b < a.B ? Lt[b] : kTile); };
    // a cursor over the span's tiles: element, tile of it, the element's length
    struct Cursor {
        int b, kt, len;
        __device__ __forceinline__ int rows() const { return len - kt * kTile; }          // valid rows from this tile on
        __device__ __forceinline__ bool elem_last() const { return rows() <= kTile; }
    };
    auto advance = [&](Cursor &c) {
        if (c.elem_last()) { ++c.b; c.kt = 0; c.len = next_len(c.b); } else ++c.kt;
    };

    const EL_LDS(char) *Tl = (const EL_LDS(char) *)T;
    const unsigned t_lds = (unsigned)(uintptr_t)Tl;
    const unsigned dz_lds = (unsigned)(uintptr_t)(const EL_LDS(char) *)Dz;

    // before the first barrier: no probabilities yet (the sum wavefronts multiply by them from step 0 on)
    if (tid < 2 * 32) Ax[tid] = 1.0f;
    for (int i = tid; i < 2 * NP * 32 * 16; i += 512) Px[i] = 0;

    // The pipeline over the span's tiles at list positions 0 .. nspan-1, one barrier per step i = 0 .. nspan+1;
    // pieces follow each other without a gap:
    //   score wavefronts   (i < nspan) partial scores of tile i into exchange buffer i&1; on an element's last tile
    //                      each chunk of EL-Q is replaced, once its MFMAs are issued, by the next element's;
    //                      (1 <= i <= nspan) softmax of tile i-1 from exchange buffer (i-1)&1 into P buffer (i-1)&1.
    //   sum wavefronts     request tile i+3 (its slot was read last in step i-1); weighted sum of tile i-2 from the
    //                      column fragments held in register set i&1 and P buffer i&1 (all zero while i < 2), each
    //                      fragment replaced, once consumed, by the one of tile i (i < nspan); where tile i-2
    //                      ends a piece, the piece is written out and the accumulators start afresh.
    const int nsteps = nspan + 2;
    if (w < 4) {
        // =========================== score wavefront ===========================
        const int part = w;
        int a_base[CHK];                                 // row r16, 16-byte chunk 4 (part CHK + c) + g of the row
        {
            const int fx = tile_swizzle(r16);
#pragma unroll
            for (int c = 0; c < CHK; ++c) a_base[c] = r16 * ROWB + (((4 * (part * CHK + c) + g) ^ fx) << 4);
        }
        // this wavefront's slice of EL-Q (all rows of the workgroup; high and low planes): B operand of the scores
        // (fragment order: chunk c of row group rg lies 2 KB after chunk c - 1, its low plane 1 KB after the high
        // one, so one 64-bit base per batch element and compile-time offsets address everything)
        u4 elq[CHK][RG][2];
        const unsigned elq_lane = (unsigned)(elq_frag_index(0, row0 + r16, 32 * (part * CHK) + 8 * g, 0, a.Rs, DM) * 2);   // bytes
        const size_t elq_elem = (size_t)a.Rs * DM * 4;                     // bytes of one batch element (two planes)
        constexpr int kRgStep = (DM / 32) * 2048;                           // bytes between row groups
        // pad rows (>= R) are never written by a2: their lanes keep the zeros they start with (a lane always holds
        // the same rows, so loads under this predicate never touch them)
        bool row_ok[RG];
#pragma unroll
        for (int rg = 0; rg < RG; ++rg) row_ok[rg] = row0 + 16 * rg + r16 < a.R;
#pragma unroll
        for (int c = 0; c < CHK; ++c)
#pragma unroll
            for (int rg = 0; rg < RG; ++rg) elq[c][rg][0] = elq[c][rg][1] = u4{0u, 0u, 0u, 0u};
        const char *elq_src = nullptr;                                     // this lane's first fragment of the element being loaded
        auto elq_begin = [&](int b) { elq_src = (const char *)a.elq + (size_t)b * elq_elem + elq_lane; };
        auto load_elq_chunk = [&](int c) {
#pragma unroll
            for (int rg = 0; rg < RG; ++rg) {
                if (row_ok[rg]) {
                    elq[c][rg][0] = *(const u4 *)(elq_src + rg * kRgStep + c * 2048);
                    elq[c][rg][1] = *(const u4 *)(elq_src + rg * kRgStep + c * 2048 + 1024);
                }
            }
        };
        // exchange buffer: row stride 16 floats, 16-byte chunk c of row r at chunk position c ^ ((r >> 2) & 3)
        int sx_put[RG];
#pragma unroll
        for (int rg = 0; rg < RG; ++rg) sx_put[rg] = part * SXP + (16 * rg + r16) * 16 + ((g ^ (r16 >> 2)) << 2);
        // Softmax bookkeeping: this wavefront does rows part RPW .. part RPW + RPW - 1 of the workgroup; lane =
        // LPR row + q holds positions TPL q .. TPL q + TPL - 1 of its row, so a row's statistics stay inside
        // LPR neighbouring lanes (DPP).  Branch-free: a row whose maximum does not grow gets the factor exp2(0) = 1.
        // It is cut into eight small stages that ride between the MFMAs of the next tile's scores: a stage is a few
        // instructions, which issue while the matrix unit works; done in one piece, the chain of LDS round trips
        // and dependent vector instructions would be waited for in full, every tile.
        const int srow = part * RPW + l / LPR, t0 = TPL * (l % LPR);
        const int sx_get = srow * 16 + (((t0 >> 2) ^ ((srow >> 2) & 3)) << 2) + (t0 & 3);
        float m_ref = -INFINITY, l_sum = 0.f;
        float sq[4][TPL], sv[TPL], pr[TPL], mx = 0.f, alpha = 1.f;
        constexpr int NST = 8;
        auto sm_stage = [&](int k, int pos, int lim) {
            const float *sp = Sx + (pos & 1) * SXB + sx_get;
            uint16_t *dst = Px + ((pos & 1) * NP * 32 + srow) * 16 + t0;
            switch (k) {
            case 0:
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    if (TPL == 2) { const f2 o = *(const f2 *)(sp + q * SXP); sq[q][0] = o[0]; sq[q][TPL - 1] = o[1]; }
                    else sq[q][0] = sp[q * SXP];
                }
                break;
            case 1:
#pragma unroll
                for (int j = 0; j < TPL; ++j) {
                    const float t = (sq[0][j] + sq[1][j]) + (sq[2][j] + sq[3][j]);
                    sv[j] = t0 + j < lim ? t : kMasked;                   // positions at or beyond the length do not exist
                }
                mx = sv[0];
                if (TPL == 2) mx = fmaxf(mx, sv[TPL - 1]);
                break;
            case 2: mx = fmaxf(mx, quad_xor1(mx)); mx = fmaxf(mx, quad_xor2(mx)); break;
            case 3: mx = fmaxf(mx, dpp_half_mirror(mx)); if (LPR == 16) mx = fmaxf(mx, dpp_row_mirror(mx)); break;
            case 4: {
                // the reference maximum only advances when it would grow by more than the rescale step; a piece's
                // first tile sets it (nothing is accumulated yet, so the factor 1 spares the pass over X)
                const float m_new = mx > m_ref + kRescaleStep ? mx : m_ref;
                alpha = m_ref == -INFINITY ? 1.0f : __builtin_amdgcn_exp2f(m_ref - m_new);
                m_ref = m_new;
                l_sum *= alpha;
                break;
            }
            case 5:
#pragma unroll
                for (int j = 0; j < TPL; ++j) { pr[j] = __builtin_amdgcn_exp2f(sv[j] - m_ref); l_sum += pr[j]; }
                break;
            case 6:
                if (BF16) {
                    // p = high + low, both bf16 by truncation
                    unsigned ph[TPL], plo[TPL];
#pragma unroll
                    for (int j = 0; j < TPL; ++j) {
                        ph[j] = __float_as_uint(pr[j]) & 0xffff0000u;
                        plo[j] = __float_as_uint(pr[j] - __uint_as_float(ph[j]));
                    }
                    if (TPL == 2) {
                        *(unsigned *)dst = (ph[0] >> 16) | ph[TPL - 1];
                        *(unsigned *)(dst + (NP - 1) * 32 * 16) = (plo[0] >> 16) | (plo[TPL - 1] & 0xffff0000u);
                    } else {
                        *dst = (uint16_t)(ph[0] >> 16);
                        *(dst + (NP - 1) * 32 * 16) = (uint16_t)(plo[0] >> 16);
                    }
                } else {
                    if (TPL == 2) *(h2 *)dst = __builtin_convertvector(f2{pr[0], pr[TPL - 1]}, h2);
                    else *(f16_t *)dst = (f16_t)pr[0];
                }
                break;
            default:
                if (l % LPR == 0) Ax[(pos & 1) * 32 + srow] = alpha;
                break;
            }
        };
        // where the tile at list position pos ends a piece: 1/sum for the sum wavefronts, the statistics for a6,
        // and a fresh start
        auto sm_close = [&](int pos, int b) {
            float l_tot = l_sum;
            l_tot += quad_xor1(l_tot);
            l_tot += quad_xor2(l_tot);
            l_tot += dpp_half_mirror(l_tot);
            if (LPR == 16) l_tot += dpp_row_mirror(l_tot);
            if (l % LPR == 0) {
                Linv[(pos & 1) * 32 + srow] = l_tot > 0.f ? 1.0f / l_tot : 0.f;
                if (row0 + srow < a.R) {
                    float *ml_out = a.ML + ((size_t)(a.flat ? span + b : b) * a.Rs + row0 + srow) * 2;
                    ml_out[0] = m_ref; ml_out[1] = l_tot;
                }
            }
            m_ref = -INFINITY; l_sum = 0.f;
        };
        // partial scores of the tile at list position pos over this wavefront's columns; the softmax of the tile
        // before it (whose `lim` first rows exist) rides between the MFMAs.  The fragment reads run PF chunks
        // ahead of the MFMAs that use them; 2 RG independent chains of MFMAs.  There is one copy of this code
        // per RELOAD value and no more: further copies that redefine the EL-Q registers make the compiler spill
        // them.  The span's first tile therefore runs the stages too, on no positions (lim = 0): finite
        // probabilities that meet zero fragments, and statistics that are reset afterwards.
        auto scores = [&](int pos, auto reload_tag, int nb, int lim) {
            constexpr bool RELOAD = decltype(reload_tag)::value;
            const EL_LDS(char) *F = Tl + (pos & 3) * SLOT;
            constexpr int PF = CHK < 4 ? CHK : 4;
            if (RELOAD) elq_begin(nb);
            u4 hb[CHK];
#pragma unroll
            for (int c = 0; c < PF; ++c) hb[c] = *(const EL_LDS(u4) *)(F + a_base[c]);
            f4 sc[RG][2];
#pragma unroll
            for (int rg = 0; rg < RG; ++rg) sc[rg][0] = sc[rg][1] = f4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int c = 0; c < CHK; ++c) {
                __builtin_amdgcn_sched_barrier(0);
                if (c + PF < CHK) hb[c + PF] = *(const EL_LDS(u4) *)(F + a_base[c + PF]);
#pragma unroll
                for (int pl = 0; pl < 2; ++pl) {
#pragma unroll
                    for (int rg = 0; rg < RG; ++rg) sc[rg][pl] = Mma<BF16>::s16(hb[c], elq[c][rg][pl], sc[rg][pl]);
#pragma unroll
                    for (int k = 0; k < NST; ++k)
                        if ((k * 2 * CHK) / NST == 2 * c + pl) sm_stage(k, pos - 1, lim);
                    __builtin_amdgcn_sched_barrier(0);
                }
                if (RELOAD) load_elq_chunk(c);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int rg = 0; rg < RG; ++rg)
                *(f4 *)(Sx + (pos & 1) * SXB + sx_put[rg]) = f4{sc[rg][0][0] + sc[rg][1][0], sc[rg][0][1] + sc[rg][1][1],
                                                                 sc[rg][0][2] + sc[rg][1][2], sc[rg][0][3] + sc[rg][1][3]};
        };

        elq_begin(b0);
#pragma unroll
        for (int c = 0; c < CHK; ++c) load_elq_chunk(c);
        Cursor cs{b0, kt0, len0}, cq{b0, kt0, len0};                  // tile whose scores / whose softmax comes next
        __syncthreads();                                              // the first tile has landed
        for (int i = 0; i < nsteps; ++i) {
            const bool sm = i >= 1 && i <= nspan;                         // the softmax of tile i - 1 belongs to this step
            const int lim = cq.rows();
            if (i < nspan) {
                const bool reload = cs.elem_last() && i + 1 < nspan;
                if (reload) scores(i, std::true_type{}, cs.b + 1, sm ? lim : 0);
                else scores(i, std::false_type{}, 0, sm ? lim : 0);
                if (!sm) { m_ref = -INFINITY; l_sum = 0.f; }
                advance(cs);
            } else if (sm) {
#pragma unroll
                for (int k = 0; k < NST; ++k) sm_stage(k, i - 1, lim);
            }
            if (sm) {
                if (cq.elem_last() || i == nspan) sm_close(i - 1, cq.b);
                advance(cq);
            }
            __syncthreads();
        }
    } else {
        // =========================== sum wavefront ===========================
        const int v = w - 4;
        // fetch cursor: the tile that is requested next (three list positions ahead of the scores)
        Cursor cf{b0, kt0, len0};
        int f_pos = 0;
        // A sum wavefront fetches rows 4v..4v+3 of every tile, always with the same number of instructions: a
        // row that does not exist (at or beyond the element's length, or past the span) is replaced by a fetch
        // of the first row of H into a dump area, and, if the tile will be used, zeros are written in its place
        // (the slot is free when its fetch is requested).  The fetch counter then advances by exactly NI per tile.
        // Everything a request needs is prepared once per tile (f_src, f_dst, f_rows), so that a request is a
        // compare, two selects and the instruction itself.
        auto dma1k = [&](unsigned dst, unsigned voff, const char *sbase) {
            if (NT) dma_piece_nt(dst, voff, sbase); else dma_piece(dst, voff, sbase);
        };
        auto dma = [&](unsigned dst, unsigned voff, const char *sbase) {
            if (PIECES == 2) { if (NT) dma_row_2k_nt(dst, voff, sbase); else dma_row_2k(dst, voff, sbase); }
            else { if (NT) dma_piece_nt(dst, voff, sbase); else dma_piece(dst, voff, sbase); }
        };
        const unsigned lx = (unsigned)((l ^ v) << 4);                   // lane's chunk position before the row's part of the swizzle
        const char *f_src;                                               // row 4v of the tile to request
        unsigned f_dst;                                                  // where that row goes in LDS
        int f_rows;                                                      // rows 4v.. of that tile that exist (<= 0: none)
        int f_valid = 0;                                                 // block fetch: valid rows of the whole tile (0: no tile)
        auto fetch_setup = [&]() {
            const bool live = f_pos < nspan;
            f_rows = live ? cf.rows() - 4 * v : 0;
            f_valid = live ? min(cf.rows(), kTile) : 0;
            // (block fetch: f_src is row 0 of the tile, the lane offsets carry the row)
            f_src = (const char *)a.H + ((size_t)min(cf.b, a.B - 1) * a.h_stride * 2 + ((size_t)cf.kt * kTile + (LIN ? 0 : 4 * v)) * ROWB);
            f_dst = t_lds + (f_pos & 3) * SLOT + 4 * v * ROWB;
        };
        // Block fetch (rows of 1.5 KB).  The four rows of a wavefront are 6 KB of contiguous memory and of contiguous
        // LDS: six 1 KB requests, lane l of request j landing at chunk position p = 64 j + l of the block, i.e. row
        // r = p / CPR, position q = p % CPR, where it must find chunk q ^ swizzle(row) of that row.  A row that does
        // not exist is replaced by the tile's last valid row (never by memory past the length): its scores are
        // masked and its probabilities are exactly zero, so a finite stand-in contributes nothing.
        unsigned lin_off[LIN ? NI : 1];
        if (LIN) {
#pragma unroll
            for (int j = 0; j < NI; ++j) {
                const int pz = 64 * j + l, r = pz / CPR, q = pz - r * CPR;
                lin_off[j] = (unsigned)((4 * v + r) * ROWB + ((q ^ tile_swizzle(4 * v + r)) << 4));
            }
        }
        auto fetch_lin = [&](int j) {
            if (f_valid <= 0) dma1k(dz_lds, (unsigned)(l << 4), (const char *)a.H);
            else if (f_valid >= kTile) dma1k(f_dst + 1024 * j, lin_off[LIN ? j : 0], f_src);
            else {
                const int pz = 64 * j + l, r = pz / CPR, q = pz - r * CPR;
                const int rs = min(4 * v + r, f_valid - 1);
                dma1k(f_dst + 1024 * j, (unsigned)(rs * ROWB + ((q ^ tile_swizzle(4 * v + r)) << 4)), f_src);
            }
        };
        // the request of one tile, row by row, so that the weighted sum can spread the four requests over its MFMAs
        // (a request holds its wavefront up while the address unit is busy with the other wavefronts' requests)
        auto fetch_row = [&](int i) {
            const bool ok = i < f_rows;                                    // wave-uniform
            const unsigned voff = (lx ^ (unsigned)(i << 6)) + (ok ? i * ROWB : 0);     // tile_swizzle(4v + i) = 4i + v
            dma(ok ? f_dst + i * ROWB : dz_lds, voff, ok ? f_src : (const char *)a.H);
            if (!ok && f_pos < nspan) {
#pragma unroll
                for (int j = 0; j < PIECES; ++j) *(u4 *)(T + (f_pos & 3) * SLOT + (4 * v + i) * ROWB + j * 1024 + l * 16) = u4{0u, 0u, 0u, 0u};
            }
        };
        auto fetch_advance = [&]() {
            if (f_pos < nspan) advance(cf);
            ++f_pos;
            fetch_setup();
        };
        auto fetch_next = [&]() {
            if (LIN) {
#pragma unroll
                for (int j = 0; j < NI; ++j) fetch_lin(j);
            } else {
#pragma unroll
                for (int i = 0; i < 4; ++i) fetch_row(i);
            }
            fetch_advance();
        };
        // wait until this wavefront's requests of a tile have landed while those of the two tiles after it are
        // still in flight (requests return in order; stores of a piece that were issued meanwhile are waited
        // for as well, which is more than needed but never less)
        auto wait_tile = [&]() { asm volatile("s_waitcnt vmcnt(%0)" :: "n"(2 * NI) : "memory"); };

        int b_lo[4], b_hi[4];   // lane i = 4k+q of 16-lane block (dh, kg) reads row 8kg+k (+4), columns 32mb+16dh+4q..+3
        {
            const int dh = g & 1, k = r16 >> 2, q = r16 & 3;
            const int t_lo = 8 * kg + k, t_hi = t_lo + 4;
            const int f_lo = tile_swizzle(t_lo), f_hi = tile_swizzle(t_hi);
#pragma unroll
            for (int mi = 0; mi < 4; ++mi) {
                const int cl = (DS * 2 / 16) * v + 4 * mi + 2 * dh + (q >> 1);
                b_lo[mi] = t_lo * ROWB + ((cl ^ f_lo) << 4) + (q & 1) * 8;
                b_hi[mi] = t_hi * ROWB + ((cl ^ f_hi) << 4) + (q & 1) * 8;
            }
        }
        f16v X[MB];
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int i = 0; i < 16; ++i) X[mb][i] = 0.f;
        s4 tb[2][MB][2];                                 // column fragments of two tiles in flight between scores and sum
#pragma unroll
        for (int s = 0; s < 2; ++s)
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) tb[s][mb][0] = tb[s][mb][1] = s4{0, 0, 0, 0};
        const bool active = r32 < ROWS;
        const int rowc = active ? r32 : 0;

        // Step i of the sum role, register set SET = i & 1: X^T[d, r] += sum_t H[t, d] P[r, t] for tile i - 2 (whose
        // fragments the set holds; P and the factors from buffer i & 1), each fragment replaced, once consumed,
        // by the one of tile i (past the span's end: by whatever the slot holds, which is never used), and the
        // requests of position i + 3 spread over the MFMAs.
        auto step = [&](auto set_tag, int i, auto &&bookkeeping) {
            constexpr int SET = decltype(set_tag)::value;
            const EL_LDS(char) *F = Tl + (i & 3) * SLOT;
            u4 P[NP];
#pragma unroll
            for (int pl = 0; pl < NP; ++pl) P[pl] = *(const u4 *)(Px + ((SET * NP + pl) * 32 + r32) * 16 + 8 * kg);
            const float al = Ax[SET * 32 + r32];
            bookkeeping();                                                // scalar work while the reads are on their way
            if (__any(al != 1.0f)) {
#pragma unroll
                for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                    for (int k = 0; k < 16; ++k) X[mb][k] *= al;
            }
            // An LDS read holds its wavefront for about as long as one of these MFMAs runs, so they alternate: the
            // MFMAs of block mb (both planes, the second accumulating on the first), each followed by one of the
            // two reads that refill the fragment of block mb - 1, whose MFMAs have been issued by then.
#pragma unroll
            for (int mb = 0; mb <= MB; ++mb) {
                __builtin_amdgcn_sched_barrier(0);
                u4 hfrag = u4{0u, 0u, 0u, 0u};
                if (mb < MB) {
                    const s4 lo = tb[SET][mb][0], hi = tb[SET][mb][1];
                    hfrag = __builtin_bit_cast(u4, s8{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]});
                    X[mb] = Mma<BF16>::s32(hfrag, P[0], X[mb]);
                }
                __builtin_amdgcn_sched_barrier(0);
                if (mb > 0) tb[SET][mb - 1][0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((EL_LDS(s4) *)(F + b_lo[(mb - 1) & 3] + ((mb - 1) >> 2) * 256));
                __builtin_amdgcn_sched_barrier(0);
                if (mb < MB && NP == 2) X[mb] = Mma<BF16>::s32(hfrag, P[NP - 1], X[mb]);
                __builtin_amdgcn_sched_barrier(0);
                if (mb > 0) tb[SET][mb - 1][1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((EL_LDS(s4) *)(F + b_hi[(mb - 1) & 3] + ((mb - 1) >> 2) * 256));
                if (LIN) { if (mb < NI) fetch_lin(mb); }
                else if (mb < MB && mb % (MB / 4 > 0 ? MB / 4 : 1) == (MB / 4 > 0 ? MB / 4 : 1) - 1) fetch_row(mb / (MB / 4 > 0 ? MB / 4 : 1));
            }
            fetch_advance();
            __builtin_amdgcn_sched_barrier(0);
        };
        // close the piece whose last tile sat at list position pos: X normalised by its own sum, straight from the
        // accumulators (a lane holds four consecutive columns of one row: 8-byte stores, two lanes side by side),
        // and a fresh start for the next piece
        auto close_piece = [&](int pos, int b) {
            const size_t slot = (size_t)(a.flat ? span + b : b);
            const float inv = Linv[(pos & 1) * 32 + rowc];
            // A lane holds columns 8 q4 + 4 kg .. + 3 of every 32-column block of its row.  The two lanes of a row
            // trade neighbouring groups (v_permlane32_swap), so that each holds eight consecutive columns and a
            // store instruction writes 32 contiguous bytes of each row instead of two pieces of 8.
            const bool keep = active && row0 + r32 < a.R;
            f16_t *x_out = a.Xp + (slot * a.Rs + row0 + rowc) * DM + DS * v + 8 * kg;
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int qp = 0; qp < 2; ++qp) {
                    unsigned ga[2], gb[2];                                   // groups q4 = 2 qp and 2 qp + 1, two fp16 pairs each
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        ga[h] = __builtin_bit_cast(unsigned, __builtin_convertvector(f2{X[mb][8 * qp + 2 * h] * inv, X[mb][8 * qp + 2 * h + 1] * inv}, h2));
                        gb[h] = __builtin_bit_cast(unsigned, __builtin_convertvector(f2{X[mb][8 * qp + 4 + 2 * h] * inv, X[mb][8 * qp + 4 + 2 * h + 1] * inv}, h2));
                        const auto sw = __builtin_amdgcn_permlane32_swap(ga[h], gb[h], false, false);
                        ga[h] = sw[0]; gb[h] = sw[1];
                    }
                    if (keep) *(u4 *)(x_out + 32 * mb + 16 * qp) = u4{ga[0], ga[1], gb[0], gb[1]};
                }
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int k = 0; k < 16; ++k) X[mb][k] = 0.f;
        };

        fetch_setup();
        fetch_next();
        fetch_next();
        fetch_next();
        wait_tile();
        __syncthreads();                                              // the first tile has landed
        Cursor cp{b0, kt0, len0};                                     // the tile whose weighted sum comes next
        auto one_step = [&](auto set_tag, int i) {
            bool closes = false;
            int close_b = 0;
            step(set_tag, i, [&]() {
                if (i >= 2) {
                    closes = cp.elem_last() || i - 2 == nspan - 1;
                    close_b = cp.b;
                    advance(cp);
                }
            });
            if (closes) close_piece(i - 2, close_b);
            wait_tile();
            __syncthreads();
        };
        for (int i = 0; i < nsteps; i += 2) {
            one_step(std::integral_constant<int, 0>{}, i);
            if (i + 1 < nsteps) one_step(std::integral_constant<int, 1>{}, i + 1);
        }
        // the last requests went to the dump area; none may be in flight when the workgroup gives up its LDS
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }
}

// ---------------------------------------------------------------------------------------------
// With a pair of events the launch carries them itself (they then read the dispatch's own begin and end,
// without the command-processor time a separately recorded event adds on either side).
template <int DM, bool BF16, int RG, bool NT>
static void launch_one(const StreamArgs &a, dim3 grid, hipStream_t s, hipEvent_t ev0, hipEvent_t ev1)
{
    if (ev0 && ev1) hipExtLaunchKernelGGL((k_core_stream<DM, BF16, RG, NT>), grid, dim3(512), 0, s, ev0, ev1, 0, a);
    else hipLaunchKernelGGL((k_core_stream<DM, BF16, RG, NT>), grid, dim3(512), 0, s, a);
}

template <int DM, bool BF16>
static hipError_t launch_t(const StreamArgs &a, int rg, hipStream_t s, hipEvent_t ev0, hipEvent_t ev1)
{
    const dim3 grid(((a.G * a.nblocks + 7) / 8) * 8);
    const bool nt = a.stream_hint != 0;
    if (rg == 1) { if (nt) launch_one<DM, BF16, 1, true>(a, grid, s, ev0, ev1); else launch_one<DM, BF16, 1, false>(a, grid, s, ev0, ev1); }
    else { if (nt) launch_one<DM, BF16, 2, true>(a, grid, s, ev0, ev1); else launch_one<DM, BF16, 2, false>(a, grid, s, ev0, ev1); }
    return hipGetLastError();
}

hipError_t launch_core_stream(const StreamArgs &a, int d_m, bool bf16, int rg, hipStream_t s, hipEvent_t ev0, hipEvent_t ev1)
{
    if (a.flat && a.B > kScanMax) return hipErrorInvalidValue;
    if (d_m == 1024) return bf16 ? launch_t<1024, true>(a, rg, s, ev0, ev1) : launch_t<1024, false>(a, rg, s, ev0, ev1);
    if (d_m == 768) return bf16 ? launch_t<768, true>(a, rg, s, ev0, ev1) : launch_t<768, false>(a, rg, s, ev0, ev1);
    if (d_m == 512) return bf16 ? launch_t<512, true>(a, rg, s, ev0, ev1) : launch_t<512, false>(a, rg, s, ev0, ev1);
    return hipErrorInvalidValue;
}

} // namespace el
