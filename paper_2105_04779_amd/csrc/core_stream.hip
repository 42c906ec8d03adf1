// MFMA attention core for gfx950, steps a3-a5 of the EL-attention decode step (Algorithm 3's two
// products over the hidden states and the softmax between them; Eq. 9 with K = V = H).
//
// The valid 16-row tiles of all batch elements form one list (element 0's tiles, then element 1's,
// ...).  The list is cut into G equal spans; a workgroup walks one span for one block of 16 or 32
// expanded-query rows, so every compute unit streams the same number of bytes whatever the lengths
// are.  Where a span crosses from one batch element to the next the workgroup closes a PIECE: it
// writes that element's partial result (normalised by its own sum, with the softmax statistics) to
// slot `span + element` and starts the next element with fresh statistics; a6 merges an element's
// pieces by the log-sum-exp rule.  An element that lies inside one span has one piece and needs no
// merge.
//
// A workgroup is eight wavefronts, two per SIMD, with two roles, so that on every SIMD the LDS
// traffic and dependent chains of one role hide behind the MFMAs of the other:
//
//   score wavefronts (0..3)   own one 16-row group of expanded queries and 1/2 or 1/4 of the model
//       dimension.  S^T[t, r] partial over those columns: 16x16x32 MFMA in the STORAGE type, A = H rows
//       (ds_read_b128), B = the wavefront's slice of EL-Q held in registers as a high + low pair of
//       16-bit values (two MFMAs), so a score keeps ~16 mantissa bits however peaked the softmax
//       is, and bf16 H enters the MFMA as it is.  The partials of a row group meet in LDS; its first
//       wavefront sums them and does the softmax bookkeeping in fp32 (running reference maximum,
//       advanced only when it would grow by more than 2^10), then publishes P (fp16, or a high + low
//       bf16 pair) and the rescale factors.
//   sum wavefronts (4..7)     own a quarter of the model dimension: X^T[d, r] += H^T[d, t] P^T[t, r],
//       32x32x16 MFMA, A = H columns through the transposing LDS read (ds_read_b64_tr_b16), B = P from
//       LDS, fp32 accumulators.  They also request the tiles: each 1 KB piece of a tile row goes
//       straight from HBM into one of four LDS tile slots (global_load_lds; two tiles are outstanding
//       while two are in use), across piece boundaries as well.  Lane i of a 1 KB piece fetches chunk
//       i ^ swizzle(row), which keeps both operand read patterns spread over all banks.
//
// Scores and softmax of a tile run one tile ahead of its weighted sum; two barriers per tile.
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

// chunk swizzle of a 16-row tile: the two bit pairs of the row number swapped.  A bijection on
// four bits (row-wise b128 reads of 16 rows hit 16 different chunk positions) whose upper pair
// runs over all four values inside {8g + k} and {8g + 4 + k}, k = 0..3 (the row sets one
// transposing read touches), so those reads use every bank exactly twice.
__device__ __forceinline__ int tile_swizzle(int row) { return ((row & 3) << 2) | ((row >> 2) & 3); }

// butterfly over the four lanes of a quad on the VALU (DPP quad_perm), no LDS round trip
__device__ __forceinline__ float quad_xor1(float v) { return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0xB1, 0xF, 0xF, true)); }
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

template <int DM, bool BF16, int RG>
__global__ void __launch_bounds__(512)
k_core_stream(const StreamArgs a)
{
    constexpr int ROWB = DM * 2;                    // bytes per tile row (2-byte elements)
    constexpr int SLOT = kTile * ROWB;              // one tile
    constexpr int NSLOT = 4;
    constexpr int PIECES = ROWB / 1024;             // 1 KB LDS-DMA pieces per row
    constexpr int NI = 4 * PIECES;                  // fetch instructions per sum wavefront per tile (four rows)
    constexpr int PARTS = 4 / RG;                   // score wavefronts per row group (column parts)
    constexpr int CHK = DM / 32 / PARTS;            // 32-column chunks of one score wavefront
    constexpr int DS = DM / 4;                      // columns per sum wavefront
    constexpr int MB = DS / 32;                     // 32-column blocks of the output per sum wavefront
    constexpr int NP = BF16 ? 2 : 1;                // 16-bit planes of P
    static_assert(DM == 512 || DM == 1024, "d_m is 512 or 1024");
    static_assert(RG == 1 || RG == 2, "row groups per workgroup");

    __shared__ __attribute__((aligned(1024))) char T[NSLOT * SLOT];
    __shared__ __attribute__((aligned(16))) float Sx[2 * 4 * 64 * 4];         // partial scores [tile parity][score wave][slot][4]
    __shared__ __attribute__((aligned(16))) uint16_t Px[2 * NP * 32 * 16];    // probabilities [tile parity][plane][row][t]
    __shared__ float Ax[2 * 32];                                              // per-row rescale factor [tile parity][row]
    __shared__ float Linv[32];                                                // per-row 1/sum of the piece being closed
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
    const int span = place / a.nblocks, rb = place % a.nblocks;
    const int row0 = rb * (16 * RG);                 // first expanded-query row of this workgroup

    auto clamp_len = [&](int v) { return min(max(v, 1), a.n); };

    // ---- where this span starts: element b0, tile kt0 of it, nspan tiles in all ----
    int b0, kt0, nspan;
    if (a.flat) {
        for (int i = tid; i < a.B; i += 512) Lt[i] = clamp_len(a.lengths ? a.lengths[i] : a.n);
        __syncthreads();
        int part = 0;
        for (int i = l; i < a.B; i += 64) part += (Lt[i] + kTile - 1) / kTile;
        const int total = wave_sum(part);
        const int lspan = max((total + a.G - 1) / a.G, a.lfloor);
        const int s0 = span * lspan;
        nspan = min(lspan, total - s0);
        const bool writer = place == 0 && w == 0 && a.E != nullptr;       // one wavefront publishes the prefix for a6
        if (writer && l == 0) a.E[0] = 0;
        b0 = -1; kt0 = 0;
        int run = 0;
        for (int c = 0; c * 64 < a.B; ++c) {
            const int i = c * 64 + l;
            int inc = i < a.B ? (Lt[i] + kTile - 1) / kTile : 0;
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                const int up = __shfl_up(inc, o, 64);
                if (l >= o) inc += up;
            }
            inc += run;
            if (writer && i < a.B) a.E[i + 1] = inc;
            const int cnt = __builtin_popcountll(__ballot(i < a.B && inc <= s0));
            if (b0 < 0 && cnt < 64 && c * 64 + cnt < a.B) {
                b0 = c * 64 + cnt;
                kt0 = s0 - (cnt ? __shfl(inc, cnt - 1, 64) : run);
                if (!writer) break;
            }
            run = __shfl(inc, 63, 64);
        }
        b0 = __builtin_amdgcn_readfirstlane(b0);
        kt0 = __builtin_amdgcn_readfirstlane(kt0);
        if (nspan <= 0 || b0 < 0) return;            // the list is shorter than G spans of the floor length
    } else {
        b0 = span; kt0 = 0;
        nspan = (clamp_len(a.lengths ? a.lengths[b0] : a.n) + kTile - 1) / kTile;
    }
    auto elem_len = [&](int b) -> int {
        int v;
        if (a.flat) v = b < a.B ? Lt[b] : kTile;
        else v = clamp_len(a.lengths ? a.lengths[min(b, a.B - 1)] : a.n);
        return __builtin_amdgcn_readfirstlane(v);
    };

    const EL_LDS(char) *Tl = (const EL_LDS(char) *)T;
    const unsigned t_lds = (unsigned)(uintptr_t)Tl;
    const unsigned dz_lds = (unsigned)(uintptr_t)(const EL_LDS(char) *)Dz;

    if (tid < 2 * 32) Ax[tid] = 1.0f;
    for (int i = tid; i < 2 * NP * 32 * 16; i += 512) Px[i] = 0;

    // partial scores of lane (row r16, position group g) go to exchange slot 4 r16 + (g ^ (r16 >> 2)): both the
    // b128 writes and the owner's b128 reads (lane = 4 row + group) then touch 16 different chunks per 16 lanes
    const int sx_put = (4 * r16 + (g ^ (r16 >> 2))) * 4;
    const int sr = l >> 2, sq = l & 3;                                    // softmax lane = 4 * row + position group
    const int sx_get = (4 * sr + (sq ^ (sr >> 2))) * 4;

    // The pipeline of a piece whose tiles sit at list positions j .. j+npc-1, one barrier per step i = 0 .. npc+1:
    //   score wavefronts   scores of tile j+i (i < npc) into exchange buffer (j+i)&1, and, between those MFMAs,
    //                      the softmax of tile j+i-1 (1 <= i <= npc) from the other buffer into P buffer (j+i-1)&1;
    //   sum wavefronts     request tile j+i+2 (i < npc); weighted sum of tile j+i-2 (2 <= i) from the column
    //                      fragments they hold in registers and P buffer (j+i-2)&1, each fragment replaced, as soon
    //                      as it is consumed, by the one of tile j+i-1 (1 <= i <= npc) read from its slot.
    // So a tile's slot is read in two consecutive steps (scores, then column fragments) and is free afterwards:
    // two tiles are resident and two in flight.  Both roles run npc + 2 barriers per piece.
    if (w < 4) {
        // =========================== score wavefront ===========================
        const int rg = w / PARTS, part = w % PARTS;
        const bool owner = part == 0;
        int a_base[CHK];                                 // row r16, 16-byte chunk 4 (part CHK + c) + g of the row
        {
            const int fx = tile_swizzle(r16);
#pragma unroll
            for (int c = 0; c < CHK; ++c) a_base[c] = r16 * ROWB + (((4 * (part * CHK + c) + g) ^ fx) << 4);
        }
        // this wavefront's slice of EL-Q (high and low planes): B operand of the score product
        u4 elq[CHK][2];
        auto load_elq = [&](int b) {
            const int row = row0 + 16 * rg + r16;
            const size_t off = ((size_t)b * a.Rs + row) * DM + 32 * (part * CHK) + 8 * g;
#pragma unroll
            for (int c = 0; c < CHK; ++c) {
                elq[c][0] = elq[c][1] = u4{0u, 0u, 0u, 0u};               // pad rows (>= R) are never written by a2
                if (row < a.R) {
                    elq[c][0] = *(const u4 *)(a.elq_hi + off + 32 * c);
                    elq[c][1] = *(const u4 *)(a.elq_lo + off + 32 * c);
                }
            }
        };
        // Softmax bookkeeping of this row group for one tile (owner only), cut into twelve small stages that ride
        // between the MFMAs of the next tile's scores (a stage is a few vector instructions: they issue while the
        // matrix unit works, a longer run of them would hold the chain of MFMAs up).  Lane = 4 * row + q holds
        // positions 4q..4q+3 of its row, so a row's statistics stay inside a quad.  Branch-free: a row whose
        // maximum does not grow gets the factor exp2(0) = 1.
        float m_ref = -INFINITY, l_sum = 0.f;
        f4 st[PARTS];
        float sv[4], pr[4], alpha = 1.f, mx = 0.f;
        unsigned ph[4], plo[4];
        int sm_lim = 0;
        auto sm_load = [&](int pos) {
#pragma unroll
            for (int p = 0; p < PARTS; ++p) st[p] = *(const f4 *)(Sx + (pos & 1) * 1024 + (rg * PARTS + p) * 256 + sx_get);
        };
        auto sm_sum = [&](int j) {                                    // sum of the partials of position 4q + j
            float v = st[0][j];
#pragma unroll
            for (int p = 1; p < PARTS; ++p) v += st[p][j];
            sv[j] = j < sm_lim ? v : -INFINITY;                         // positions at or beyond the length do not exist
        };
        auto sm_prob = [&](int j) { pr[j] = __builtin_amdgcn_exp2f(sv[j] - m_ref); l_sum += pr[j]; };
        auto sm_split = [&](int j) {                                  // p = high + low, both bf16 by truncation
            ph[j] = __float_as_uint(pr[j]) & 0xffff0000u;
            plo[j] = __float_as_uint(pr[j] - __uint_as_float(ph[j]));
        };
        auto sm_stage = [&](int k, int pos) {
            const int buf = pos & 1;
            uint16_t *dst = Px + buf * (NP * 32 * 16) + (16 * rg + sr) * 16 + 4 * sq;
            switch (k) {
            case 0: sm_sum(0); sm_sum(1); break;
            case 1: sm_sum(2); sm_sum(3); break;
            case 2: mx = fmaxf(fmaxf(sv[0], sv[1]), fmaxf(sv[2], sv[3])); mx = fmaxf(mx, quad_xor1(mx)); break;
            case 3: mx = fmaxf(mx, quad_xor2(mx)); break;
            case 4: {
                const float m_new = mx > m_ref + kRescaleStep ? mx : m_ref;    // also on a piece's first tile (m_ref = -inf)
                // first tile: nothing accumulated yet, so no rescale (the factor 1 spares the pass over X)
                alpha = m_ref == -INFINITY ? 1.0f : __builtin_amdgcn_exp2f(m_ref - m_new);
                m_ref = m_new;
                l_sum *= alpha;
                break;
            }
            case 5: sm_prob(0); sm_prob(1); break;
            case 6: sm_prob(2); sm_prob(3); break;
            case 7: if (BF16) { sm_split(0); sm_split(1); } break;
            case 8: if (BF16) { sm_split(2); sm_split(3); } break;
            case 9:
                if (BF16) *(u2 *)dst = u2{(ph[0] >> 16) | ph[1], (ph[2] >> 16) | ph[3]};
                else {
                    const h2 p01 = __builtin_convertvector(f2{pr[0], pr[1]}, h2), p23 = __builtin_convertvector(f2{pr[2], pr[3]}, h2);
                    *(h4 *)dst = h4{p01[0], p01[1], p23[0], p23[1]};
                }
                break;
            case 10:
                if (BF16) *(u2 *)(dst + 32 * 16) = u2{(plo[0] >> 16) | (plo[1] & 0xffff0000u), (plo[2] >> 16) | (plo[3] & 0xffff0000u)};
                break;
            default: Ax[buf * 32 + 16 * rg + sr] = alpha; break;      // the four lanes of a quad write the same value
            }
        };
        constexpr int NST = 12;
        // scores of the tile at list position pos over this wavefront's columns, left in LDS for the exchange;
        // with SM (owner only), the softmax of the tile before it rides between the MFMAs.  The fragment reads
        // run PF chunks ahead of the MFMAs that use them.
        auto scores = [&](int pos, auto sm_tag, int lim_rows) {
            constexpr bool SM = decltype(sm_tag)::value;
            const EL_LDS(char) *F = Tl + (pos & 3) * SLOT;
            constexpr int PF = CHK < 4 ? CHK : 4;
            if (SM) { sm_load(pos - 1); sm_lim = lim_rows - 4 * sq; }
            u4 hb[CHK];
#pragma unroll
            for (int c = 0; c < PF; ++c) hb[c] = *(const EL_LDS(u4) *)(F + a_base[c]);
            // two chains of MFMAs (high plane, low plane), so that no MFMA waits for the one issued just before it
            f4 sc = f4{0.f, 0.f, 0.f, 0.f}, sc2 = f4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int c = 0; c < CHK; ++c) {
                __builtin_amdgcn_sched_barrier(0);
                if (c + PF < CHK) hb[c + PF] = *(const EL_LDS(u4) *)(F + a_base[c + PF]);
                sc = Mma<BF16>::s16(hb[c], elq[c][0], sc);
                if (SM) {
#pragma unroll
                    for (int k = 0; k < NST; ++k)
                        if ((2 * k * CHK) / NST == 2 * c) sm_stage(k, pos - 1);
                    __builtin_amdgcn_sched_barrier(0);
                }
                sc2 = Mma<BF16>::s16(hb[c], elq[c][1], sc2);
                if (SM) {
#pragma unroll
                    for (int k = 0; k < NST; ++k)
                        if ((2 * k * CHK) / NST == 2 * c + 1) sm_stage(k, pos - 1);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
            *(f4 *)(Sx + (pos & 1) * 1024 + w * 256 + sx_put) = f4{sc[0] + sc2[0], sc[1] + sc2[1], sc[2] + sc2[2], sc[3] + sc2[3]};
        };

        load_elq(b0);
        int c_b = b0, c_kt = kt0, c_len = elem_len(b0);
        __syncthreads();                                              // the first two tiles have landed
        for (int j = 0;;) {
            const int ntile = (c_len + kTile - 1) / kTile;
            const int npc = min(ntile - c_kt, nspan - j);                // tiles of this piece
            const int rows0 = c_len - c_kt * kTile;                      // valid rows from the piece's first tile on
            scores(j, std::false_type{}, 0);
            __syncthreads();
            for (int i = 1; i < npc; ++i) {
                if (owner) scores(j + i, std::true_type{}, rows0 - (i - 1) * kTile);
                else scores(j + i, std::false_type{}, 0);
                __syncthreads();
            }
            j += npc;
            const bool more = j < nspan;
            // the next element's expanded queries are requested while this piece drains
            if (more) load_elq(c_b + 1);
            if (owner) {
                // the softmax of the piece's last tile, then this row group's statistics
                sm_load(j - 1); sm_lim = rows0 - (npc - 1) * kTile - 4 * sq;
#pragma unroll
                for (int k = 0; k < NST; ++k) sm_stage(k, j - 1);
                l_sum += quad_xor1(l_sum);
                l_sum += quad_xor2(l_sum);
                const int row = row0 + 16 * rg + sr;
                if (sq == 0) {
                    Linv[16 * rg + sr] = l_sum > 0.f ? 1.0f / l_sum : 0.f;
                    if (row < a.R) {
                        float *ml_out = a.ML + ((size_t)(a.flat ? span + c_b : c_b) * a.Rs + row) * 2;
                        ml_out[0] = m_ref; ml_out[1] = l_sum;
                    }
                }
            }
            m_ref = -INFINITY; l_sum = 0.f;
            __syncthreads();                                          // step npc: P of the last tile and 1/sum are in LDS
            __syncthreads();                                          // step npc+1: the sum wavefronts finish the piece
            if (!more) break;
            ++c_b; c_kt = 0; c_len = elem_len(c_b);
        }
    } else {
        // =========================== sum wavefront ===========================
        const int v = w - 4;
        const bool stream_hint = a.stream_hint != 0;
        // fetch cursor: the tile that is requested next (two list positions ahead of the scores)
        int f_b = b0, f_kt = kt0, f_len = elem_len(b0), f_pos = 0;
        const char *f_H = (const char *)a.H + (size_t)b0 * a.h_stride * 2;
        // A sum wavefront fetches rows 4v..4v+3 of every tile, always with the same number of instructions: a
        // row that does not exist (at or beyond the element's length, or past the span) is replaced by a fetch
        // of the first row of H into a dump area, and, if the tile will be used, zeros are written in its place
        // (the slot is free when its fetch is requested).  The fetch counter then advances by exactly NI per tile.
        auto dma = [&](unsigned dst, unsigned voff, const char *sbase) {
            if (PIECES == 2) { if (stream_hint) dma_row_2k_nt(dst, voff, sbase); else dma_row_2k(dst, voff, sbase); }
            else { if (stream_hint) dma_piece_nt(dst, voff, sbase); else dma_piece(dst, voff, sbase); }
        };
        unsigned voff4[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) voff4[i] = (unsigned)(((l ^ ((i << 2) | v)) << 4) + i * ROWB);    // tile_swizzle(4v + i)
        // the request of one tile, row by row, so that the weighted sum can spread the four requests over its MFMAs
        // (a request holds its wavefront up while the address unit is busy with the other wavefronts' requests)
        auto fetch_row = [&](int i) {
            const int slot = f_pos & 3;
            const bool live = f_pos < nspan;
            const int rows = live ? f_len - f_kt * kTile : 0;          // valid rows of this tile (may exceed 16)
            const int row = 4 * v + i;
            const bool ok = row < rows;                                    // wave-uniform
            const char *sbase = ok ? f_H + ((size_t)f_kt * kTile + 4 * v) * ROWB : (const char *)a.H - i * ROWB;
            const unsigned dst = ok ? t_lds + slot * SLOT + row * ROWB : dz_lds;
            dma(dst, voff4[i], sbase);
            if (live && !ok) {
#pragma unroll
                for (int j = 0; j < PIECES; ++j) *(u4 *)(T + slot * SLOT + row * ROWB + j * 1024 + l * 16) = u4{0u, 0u, 0u, 0u};
            }
        };
        auto fetch_advance = [&]() {
            const bool live = f_pos < nspan;
            ++f_pos;
            if (live) {
                if (++f_kt * kTile >= f_len) {
                    ++f_b; f_kt = 0;
                    f_len = elem_len(f_b);
                    f_H = (const char *)a.H + (size_t)min(f_b, a.B - 1) * a.h_stride * 2;
                }
            }
        };
        auto fetch_next = [&]() {
#pragma unroll
            for (int i = 0; i < 4; ++i) fetch_row(i);
            fetch_advance();
        };
        // wait until this wavefront's fetches of a tile have landed, given the tiles requested after it
        auto wait_own = [&](int later_tiles) {
            if (later_tiles >= 1) asm volatile("s_waitcnt vmcnt(%0)" :: "n"(NI) : "memory");
            else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        };
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
        s4 tb[MB][2];                                    // column fragments of the tile whose weighted sum comes next

        // One step of the sum role: X^T[d, r] += sum_t H[t, d] P[r, t] for the tile whose fragments are held
        // (do_pv; P and the factors from buffer pv_pos&1), each fragment replaced, once consumed, by the one of
        // the tile at list position ld_pos (do_ld).
        auto step = [&](bool do_pv, int pv_pos, bool do_ld, int ld_pos, bool do_fetch) {
            const EL_LDS(char) *F = Tl + (ld_pos & 3) * SLOT;
            u4 P[NP];
            float al = 1.f;
            if (do_pv) {
                const int buf = pv_pos & 1;
#pragma unroll
                for (int pl = 0; pl < NP; ++pl) P[pl] = *(const u4 *)(Px + (buf * NP + pl) * (32 * 16) + r32 * 16 + 8 * kg);
                al = Ax[buf * 32 + r32];
                if (__any(al != 1.0f)) {
#pragma unroll
                    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                        for (int i = 0; i < 16; ++i) X[mb][i] *= al;
                }
            }
            u4 hprev = u4{0u, 0u, 0u, 0u};
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) {
                __builtin_amdgcn_sched_barrier(0);
                if (do_pv) {
                    // plane 0 of this block, then plane 1 of the block before it: no MFMA waits for its predecessor
                    const s4 lo = tb[mb][0], hi = tb[mb][1];
                    const u4 hfrag = __builtin_bit_cast(u4, s8{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]});
                    X[mb] = Mma<BF16>::s32(hfrag, P[0], X[mb]);
                    if (NP == 2 && mb > 0) X[mb - 1] = Mma<BF16>::s32(hprev, P[1], X[mb - 1]);
                    hprev = hfrag;
                }
                if (do_ld) {
                    tb[mb][0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((EL_LDS(s4) *)(F + b_lo[mb & 3] + (mb >> 2) * 256));
                    tb[mb][1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((EL_LDS(s4) *)(F + b_hi[mb & 3] + (mb >> 2) * 256));
                }
                if (do_fetch && mb % (MB / 4) == MB / 4 - 1) fetch_row(mb / (MB / 4));
            }
            if (do_pv && NP == 2) X[MB - 1] = Mma<BF16>::s32(hprev, P[1], X[MB - 1]);
            if (do_fetch) fetch_advance();
            __builtin_amdgcn_sched_barrier(0);
        };
        // close a piece: X normalised by its own sum, straight from the accumulators (a lane holds four
        // consecutive columns of one row: 8-byte stores, two lanes side by side, four instructions fill 64 bytes
        // of each of 32 rows)
        auto store_piece = [&](int b) {
            const size_t slot = (size_t)(a.flat ? span + b : b);
            const float inv = r32 < 16 * RG ? Linv[r32] : 0.f;
            if (r32 < 16 * RG && row0 + r32 < a.R) {
                f16_t *x_out = a.Xp + (slot * a.Rs + row0 + r32) * DM + DS * v + 4 * kg;
#pragma unroll
                for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                    for (int q4 = 0; q4 < 4; ++q4) {
                        const h2 lo = __builtin_convertvector(f2{X[mb][4 * q4 + 0] * inv, X[mb][4 * q4 + 1] * inv}, h2);
                        const h2 hi = __builtin_convertvector(f2{X[mb][4 * q4 + 2] * inv, X[mb][4 * q4 + 3] * inv}, h2);
                        *(h4 *)(x_out + 32 * mb + 8 * q4) = h4{lo[0], lo[1], hi[0], hi[1]};
                    }
            }
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int i = 0; i < 16; ++i) X[mb][i] = 0.f;
        };

        fetch_next();
        fetch_next();
        int c_b = b0, c_kt = kt0, c_len = elem_len(b0);
        wait_own(0);
        __syncthreads();                                              // the first two tiles have landed
        for (int j = 0;;) {
            const int ntile = (c_len + kTile - 1) / kTile;
            const int npc = min(ntile - c_kt, nspan - j);
            for (int i = 0; i < npc; ++i) {
                // list position j + i + 2 is requested in every step
                if (i == 0) fetch_next();
                if (i == 1) step(false, 0, true, j, true);
                if (i >= 2) step(true, j + i - 2, true, j + i - 1, true);
                wait_own(1);
                __syncthreads();
            }
            j += npc;
            if (npc >= 2) step(true, j - 2, true, j - 1, false);      // step npc
            else step(false, 0, true, j - 1, false);
            __syncthreads();
            step(true, j - 1, false, 0, false);                       // step npc + 1
            store_piece(c_b);
            __syncthreads();
            if (j >= nspan) break;
            ++c_b; c_kt = 0; c_len = elem_len(c_b);
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }
}

// ---------------------------------------------------------------------------------------------
// With a pair of events the launch carries them itself (they then read the dispatch's own begin and end,
// without the command-processor time a separately recorded event adds on either side).
template <int DM, bool BF16, int RG>
static void launch_one(const StreamArgs &a, dim3 grid, hipStream_t s, hipEvent_t ev0, hipEvent_t ev1)
{
    if (ev0 && ev1) hipExtLaunchKernelGGL((k_core_stream<DM, BF16, RG>), grid, dim3(512), 0, s, ev0, ev1, 0, a);
    else hipLaunchKernelGGL((k_core_stream<DM, BF16, RG>), grid, dim3(512), 0, s, a);
}

template <int DM, bool BF16>
static hipError_t launch_t(const StreamArgs &a, int rg, hipStream_t s, hipEvent_t ev0, hipEvent_t ev1)
{
    const dim3 grid(((a.G * a.nblocks + 7) / 8) * 8);
    if (rg == 1) launch_one<DM, BF16, 1>(a, grid, s, ev0, ev1);
    else launch_one<DM, BF16, 2>(a, grid, s, ev0, ev1);
    return hipGetLastError();
}

hipError_t launch_core_stream(const StreamArgs &a, int d_m, bool bf16, int rg, hipStream_t s, hipEvent_t ev0, hipEvent_t ev1)
{
    if (a.flat && a.B > kScanMax) return hipErrorInvalidValue;
    if (d_m == 1024) return bf16 ? launch_t<1024, true>(a, rg, s, ev0, ev1) : launch_t<1024, false>(a, rg, s, ev0, ev1);
    if (d_m == 512) return bf16 ? launch_t<512, true>(a, rg, s, ev0, ev1) : launch_t<512, false>(a, rg, s, ev0, ev1);
    return hipErrorInvalidValue;
}

} // namespace el
