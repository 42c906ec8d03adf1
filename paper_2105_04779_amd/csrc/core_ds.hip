// MFMA attention core for gfx950, steps a3-a5 of the EL-attention decode step (Algorithm 3's two
// products over the hidden states and the softmax between them; Eq. 9 with K = V = H).
//
// One workgroup (4 wavefronts, one per SIMD) owns a contiguous range of 16-row tiles of one batch
// element's H and up to 64 expanded-query rows.  The four wavefronts split the MODEL dimension:
// wavefront w owns columns [w d_m/4, (w+1) d_m/4) of H for both products, so every byte of a tile
// is read from LDS exactly twice per workgroup (once per product), whatever the number of rows.
//
//   fetch      each 1 KB piece of a tile row goes straight from HBM into one of four LDS tile
//              slots (global_load_lds, no registers in flight; two tiles are outstanding while
//              two are in use).  Lane i of a piece fetches chunk i ^ swizzle(row): the tile
//              lands in the XOR-swizzled order that keeps both operand read patterns spread over
//              all banks.  bf16 fragments are converted to fp16 in registers after each LDS read,
//              behind the MFMAs, so a tile is never rewritten in LDS.
//   scores     S^T[t, r] partial over the wave's columns: v_mfma_f32_16x16x32_f16,
//              A = H rows (ds_read_b128), B = the wave's slice of ELQ (registers).
//   exchange   the four partial score tiles meet in LDS; wavefront g < RG sums them for row
//              group g and does that group's softmax bookkeeping in fp32 (running reference
//              maximum, advanced only when it would grow by more than 2^10; sum kept per lane),
//              then publishes P (fp16, round-to-nearest-even) and the rescale factors.
//   weighted   X^T[d, r] += H^T[d, t] P^T[t, r]: v_mfma_f32_32x32x16_f16, A = H columns through the
//   sum        transposing LDS read (ds_read_b64_tr_b16), B = P from LDS.  Each wavefront keeps
//              its d_m/4 x rows fp32 accumulators in AccVGPRs for the whole range.
//
// The scores and the softmax of a tile run one tile ahead of its weighted sum: the softmax's dependent
// chain rides between the MFMAs of the previous tile's weighted sum, and there are two barriers per tile.
//
// Scores arrive pre-multiplied by log2(e)/sqrt(d_k), so the softmax is an exp2 of a difference.
// The partial result (one per key-range split) leaves normalised by its own sum, in fp16, through
// LDS so that every global store instruction writes 1 KB of one row.
#include <type_traits>
#include <hip/hip_ext.h>
#include "el_internal.h"

namespace el {

typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef _Float16 h4 __attribute__((ext_vector_type(4)));
typedef _Float16 h2 __attribute__((ext_vector_type(2)));
typedef short s4 __attribute__((ext_vector_type(4)));
typedef short s8 __attribute__((ext_vector_type(8)));
typedef float f2 __attribute__((ext_vector_type(2)));
typedef float f4 __attribute__((ext_vector_type(4)));
typedef float f16v __attribute__((ext_vector_type(16)));
typedef unsigned int u4 __attribute__((ext_vector_type(4)));
#define EL_LDS(T) __attribute__((address_space(3))) T

constexpr int kTileRows16 = 16;
constexpr float kRescaleStep16 = 10.0f;   // log2 units: probabilities stay below 2^10

// chunk swizzle of a 16-row tile: the two bit pairs of the row number swapped.  A bijection on
// four bits (row-wise b128 reads of 16 rows hit 16 different chunk positions) whose upper pair
// runs over all four values inside {8g + k} and {8g + 4 + k}, k = 0..3 (the row sets one
// transposing read touches), so those reads use every bank exactly twice.
__device__ __forceinline__ int tile_swizzle(int row) { return ((row & 3) << 2) | ((row >> 2) & 3); }

__device__ __forceinline__ unsigned bf16x2_to_f16x2_ds(unsigned x)
{
    const float lo = __uint_as_float(x << 16);
    const float hi = __uint_as_float(x & 0xffff0000u);
    return __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_pkrtz(lo, hi));
}

// butterfly over the four lanes of a quad on the VALU (DPP quad_perm), no LDS round trip
__device__ __forceinline__ float quad_xor1(float v) { return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0xB1, 0xF, 0xF, true)); }
__device__ __forceinline__ float quad_xor2(float v) { return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x4E, 0xF, 0xF, true)); }

// eight bf16 values held in the bits of an fp16 fragment -> the same values in fp16
__device__ __forceinline__ h8 frag_bf16_to_f16(h8 v)
{
    u4 x = __builtin_bit_cast(u4, v);
    x.x = bf16x2_to_f16x2_ds(x.x); x.y = bf16x2_to_f16x2_ds(x.y);
    x.z = bf16x2_to_f16x2_ds(x.z); x.w = bf16x2_to_f16x2_ds(x.w);
    return __builtin_bit_cast(h8, x);
}


template <int DM, bool BF16, int RG>
__global__ void __launch_bounds__(256)
k_core_ds(const CoreArgs a)
{
    constexpr int ROWB = DM * 2;                    // bytes per tile row (2-byte elements)
    constexpr int SLOT = kTileRows16 * ROWB;        // one tile
    constexpr int NSLOT = 4;
    constexpr int PIECES = ROWB / 1024;             // 1 KB LDS-DMA pieces per row
    constexpr int NI = 4 * PIECES;                  // fetch instructions per wavefront per full tile
    constexpr int DS = DM / 4;                      // columns per wavefront
    constexpr int KC = DS / 32;                     // k-chunks of the score product
    constexpr int MB = DS / 32;                     // 32-column blocks of the output
    constexpr int NB = (RG + 1) / 2;                // 32-row blocks of expanded queries
    constexpr int CW16 = DS * 2;                    // byte offset step of a wavefront's column slice
    static_assert(ROWB % 1024 == 0 && KC >= 4 && KC % 4 == 0, "d_m must be a multiple of 512");
    static_assert(RG == 1 || RG == 2 || RG == 4, "row groups per workgroup");

    __shared__ __attribute__((aligned(1024))) char T[NSLOT * SLOT];
    __shared__ __attribute__((aligned(16))) float Sx[4 * RG * 64 * 4];   // partial scores [wave][rg][lane][4]
    __shared__ __attribute__((aligned(16))) f16_t Px[2 * NB * 32 * 16];  // probabilities [tile parity][row][t]
    __shared__ float Ax[2 * NB * 32];                                    // per-row rescale factor [tile parity][row]
    __shared__ float Linv[NB * 32];                                      // per-row 1/sum for the partial result
    __shared__ __attribute__((aligned(1024))) char Dz[ROWB];             // where fetches of rows that do not exist land

    const int tid = threadIdx.x, l = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r16 = l & 15, g = l >> 4, r32 = l & 31, kg = l >> 5;

    // workgroup -> (batch element, key split, row block); workgroups that share an H range differ
    // by multiples of 8 so they are dispatched to the same XCD (same L2).
    const int id = blockIdx.x;
    const int oct = id / (8 * a.nblocks), rem = id % (8 * a.nblocks);
    const int rb = rem >> 3, group = oct * 8 + (rem & 7);
    const int row0 = rb * (16 * RG);                 // first expanded-query row of this workgroup
    if (group >= a.B * a.S) return;
    const int b = group / a.S, s = group % a.S;
    int len = a.lengths ? a.lengths[b] : a.n;

    // ---- this wavefront's column slice of ELQ, all row groups: B operand of the score product ----
    // Requested first: the addresses need nothing but the workgroup's coordinates, so these loads are under
    // way while the element's length (a dependent load the tile requests have to wait for) is still coming.
    h8 elq[RG][KC];
#pragma unroll
    for (int rg = 0; rg < RG; ++rg) {
        const int row = row0 + 16 * rg + r16;
        // pad rows (row >= R) are never written by the expansion step: they read as zero here
        const f16_t *src = a.elq + ((size_t)b * a.Rs + row) * DM + DS * w + 8 * g;
        const h8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
        for (int c = 0; c < KC; ++c) elq[rg][c] = zero;
        if (row < a.R) {
#pragma unroll
            for (int c = 0; c < KC; ++c) elq[rg][c] = *(const h8 *)(src + 32 * c);
        }
    }

    len = min(max(len, 1), a.n);
    const int NT = (len + kTileRows16 - 1) / kTileRows16;
    const int k0 = (NT * s) / a.S, k1 = (NT * (s + 1)) / a.S;   // NT * S stays far below 2^31
    const int nloc = k1 - k0;
    const char *Hb = (const char *)a.H + (size_t)b * a.h_stride * 2;

    const EL_LDS(char) *Tl = (const EL_LDS(char) *)T;
    const unsigned t_lds = (unsigned)(uintptr_t)Tl;
    const unsigned dz_lds = (unsigned)(uintptr_t)(const EL_LDS(char) *)Dz;

    // A wavefront fetches rows 4w..4w+3 of every tile, always with the same number of instructions: a row
    // that does not exist (at or beyond len, or of a tile past this workgroup's range) is replaced by a
    // fetch of the element's first row into a dump area.  The fetch counter then advances by exactly NI
    // per tile, and the loop needs neither branches around the requests nor per-tile wait arithmetic.
    auto issue_dma_row = [&](int kt, int slot, int i, auto nt_tag) {
        constexpr bool NT = decltype(nt_tag)::value;
        const bool ok = kt < k1 && kt * kTileRows16 + 4 * w + i < len;               // wave-uniform
        const char *sbase = ok ? Hb + ((size_t)kt * kTileRows16 + 4 * w) * ROWB : Hb - i * ROWB;
        const int f = (i << 2) | w;                                                   // tile_swizzle(4w + i)
        const unsigned voff = (unsigned)(((l ^ f) << 4) + i * ROWB);
        const unsigned dst = ok ? t_lds + slot * SLOT + (4 * w + i) * ROWB : dz_lds;
        if (PIECES == 2) { if (NT) dma_row_2k_nt(dst, voff, sbase); else dma_row_2k(dst, voff, sbase); }
        else { if (NT) dma_piece_nt(dst, voff, sbase); else dma_piece(dst, voff, sbase); }
    };
    auto issue_dma_t = [&](int kt, int slot, auto nt_tag) {
        constexpr bool NT = decltype(nt_tag)::value;
        if (kt < k1 && (kt + 1) * kTileRows16 <= len) {
            // the common case, a whole tile inside the range: one source base and four destinations,
            // without the per-row selects below
            const char *sbase = Hb + ((size_t)kt * kTileRows16 + 4 * w) * ROWB;
            const unsigned dst0 = t_lds + slot * SLOT + (4 * w) * ROWB;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int f = (i << 2) | w;
                const unsigned voff = (unsigned)(((l ^ f) << 4) + i * ROWB);
                if (PIECES == 2) { if (NT) dma_row_2k_nt(dst0 + i * ROWB, voff, sbase); else dma_row_2k(dst0 + i * ROWB, voff, sbase); }
                else { if (NT) dma_piece_nt(dst0 + i * ROWB, voff, sbase); else dma_piece(dst0 + i * ROWB, voff, sbase); }
            }
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) issue_dma_row(kt, slot, i, nt_tag);
        }
    };
    // the cache hint is a launch-wide choice: both forms issue the same number of requests
    const bool stream_hint = a.stream_hint != 0;
    auto issue_dma = [&](int kt, int slot) {
        if (stream_hint) issue_dma_t(kt, slot, std::true_type{});
        else issue_dma_t(kt, slot, std::false_type{});
    };
    // wait until this wavefront's fetches of a tile have landed, given the tiles requested after it
    auto wait_own = [&](int later_tiles) {
        if (later_tiles >= 2) asm volatile("s_waitcnt vmcnt(%0)" :: "n"(2 * NI) : "memory");
        else if (later_tiles == 1) asm volatile("s_waitcnt vmcnt(%0)" :: "n"(NI) : "memory");
        else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    };
    // Rows at or beyond len were never fetched and must not reach the MFMAs as garbage: the wavefront that
    // owns such rows of the (last, ragged) tile kt writes zeros over them.
    auto zero_ragged = [&](int kt, int slot) {
        if ((kt + 1) * kTileRows16 <= len) return;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (kt * kTileRows16 + 4 * w + i < len) continue;
#pragma unroll
            for (int j = 0; j < PIECES; ++j)
                *(u4 *)(T + slot * SLOT + (4 * w + i) * ROWB + j * 1024 + l * 16) = u4{0u, 0u, 0u, 0u};
        }
    };

    // ---- prologue: request two tiles (right behind the ELQ loads), wait for everything ----
    if (nloc > 0) {
        issue_dma(k0, 0);
        issue_dma(k0 + 1, 1);
    }

    float m_ref = -INFINITY, l_sum = 0.f;           // meaningful in owner wavefronts (w < RG) only

    if (tid < 2 * NB * 32) Ax[tid] = 1.0f;
    if (tid < NB * 32) Linv[tid] = 0.f;
    for (int i = tid; i < 2 * NB * 32 * 16; i += 256) Px[i] = (f16_t)0.f;

    // ---- per-lane LDS offsets inside a tile slot ----
    int a_base[4];   // score product: row r16, chunk (slice) + 4c + g
    {
        const int fx = tile_swizzle(r16);
#pragma unroll
        for (int ci = 0; ci < 4; ++ci) a_base[ci] = r16 * ROWB + CW16 * w + (((4 * ci + g) ^ fx) << 4);
    }
    int b_lo[4], b_hi[4];   // weighted sum: lane i = 4k+q of 16-lane block (dh, kg) reads row 8kg+k (+4), columns 32mb+16dh+4q..+3
    {
        const int dh = g & 1, k = r16 >> 2, q = r16 & 3;
        const int t_lo = 8 * kg + k, t_hi = t_lo + 4;
        const int f_lo = tile_swizzle(t_lo), f_hi = tile_swizzle(t_hi);
#pragma unroll
        for (int mi = 0; mi < 4; ++mi) {
            const int cl = 4 * mi + 2 * dh + (q >> 1);
            b_lo[mi] = t_lo * ROWB + CW16 * w + ((cl ^ f_lo) << 4) + (q & 1) * 8;
            b_hi[mi] = t_hi * ROWB + CW16 * w + ((cl ^ f_hi) << 4) + (q & 1) * 8;
        }
    }

    f16v X[MB][NB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int i = 0; i < 16; ++i) X[mb][nb][i] = 0.f;
    // The compiler does not see the LDS-DMA requests; it does see the ELQ loads above, and would place
    // their wait (which also drains every later fetch) in front of the first MFMA of EVERY iteration.
    // Consuming the registers here, on every path into the loop, moves that wait out of it.
#pragma unroll
    for (int rg = 0; rg < RG; ++rg)
#pragma unroll
        for (int c = 0; c < KC; ++c) asm volatile("" :: "v"(elq[rg][c]));
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");                  // ELQ and, requested after it, both tiles
    if (nloc > 0) zero_ragged(k0, 0);
    __syncthreads();

    // ---- scores of tile kk (slot kk&3) over this wavefront's columns, left in LDS for the exchange.
    //      The fetch of tile kk+2 is requested between the fragment loads and the first MFMA (it fills
    //      the LDS latency); the conversion of each next fragment is issued behind an MFMA and runs
    //      while the matrix unit is busy. ----
    auto scores = [&](int kk) {
        const EL_LDS(char) *F = Tl + (kk & 3) * SLOT;
        u4 hb[KC];
#pragma unroll
        for (int c = 0; c < KC; ++c) hb[c] = *(const EL_LDS(u4) *)(F + a_base[c & 3] + (c >> 2) * 256);
        issue_dma(k0 + kk + 2, (kk + 2) & 3);
        f4 sc[RG];
#pragma unroll
        for (int rg = 0; rg < RG; ++rg) sc[rg] = f4{0.f, 0.f, 0.f, 0.f};
        constexpr int WPM = 4 / RG;                                    // words converted per MFMA
        u4 cur = hb[0];
        if (BF16) {
            cur.x = bf16x2_to_f16x2_ds(cur.x); cur.y = bf16x2_to_f16x2_ds(cur.y);
            cur.z = bf16x2_to_f16x2_ds(cur.z); cur.w = bf16x2_to_f16x2_ds(cur.w);
        }
#pragma unroll
        for (int c = 0; c < KC; ++c) {
            u4 nxt = hb[c + 1 < KC ? c + 1 : c];
#pragma unroll
            for (int rg = 0; rg < RG; ++rg) {
                __builtin_amdgcn_sched_barrier(0);
                sc[rg] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(h8, cur), elq[rg][c], sc[rg], 0, 0, 0);
                if (BF16 && c + 1 < KC) {
#pragma unroll
                    for (int e = 0; e < WPM; ++e) {
                        nxt[rg * WPM + e] = bf16x2_to_f16x2_ds(nxt[rg * WPM + e]);
                        asm volatile("" : "+v"(nxt[rg * WPM + e]));           // keeps the conversion behind this MFMA
                    }
                }
            }
            __builtin_amdgcn_sched_barrier(0);
            cur = nxt;
        }
#pragma unroll
        for (int rg = 0; rg < RG; ++rg) *(f4 *)(Sx + ((w * RG + rg) * 64 + l) * 4) = sc[rg];
    };

    // ---- softmax bookkeeping of row group w for one tile, cut into stages that the weighted sum of the
    //      previous tile interleaves with its MFMAs.  Lane = 4 * row + q holds positions 4q..4q+3 of its
    //      row, so a row's statistics stay inside a quad.  Everything is branch-free: a row whose maximum
    //      does not grow gets the factor exp2(0) = 1. ----
    const bool owner = RG == 4 || w < RG;
    const int sr = l >> 2, sq = l & 3;
    f4 st0, st1, st2, st3;
    float sv[4], pr[4], mx_l = 0.f, alpha = 1.f;
    auto sm_load = [&]() {
        if (!owner) return;
        const int src_lane = sr + 16 * sq;
        st0 = *(const f4 *)(Sx + ((0 * RG + w) * 64 + src_lane) * 4); st1 = *(const f4 *)(Sx + ((1 * RG + w) * 64 + src_lane) * 4);
        st2 = *(const f4 *)(Sx + ((2 * RG + w) * 64 + src_lane) * 4); st3 = *(const f4 *)(Sx + ((3 * RG + w) * 64 + src_lane) * 4);
    };
    auto sm_stage1 = [&](int kt) {                                    // sum of the four partials, local maximum
        if (!owner) return;
        const int lim = len - kt * kTileRows16 - 4 * sq;                // positions at or beyond len do not exist
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            sv[j] = (st0[j] + st1[j]) + (st2[j] + st3[j]);
            sv[j] = j < lim ? sv[j] : -INFINITY;
        }
        mx_l = fmaxf(fmaxf(sv[0], sv[1]), fmaxf(sv[2], sv[3]));
    };
    auto sm_stage2 = [&]() {                                          // row maximum, reference, rescale factor
        if (!owner) return;
        float mx = fmaxf(mx_l, quad_xor1(mx_l));
        mx = fmaxf(mx, quad_xor2(mx));
        const float m_new = mx > m_ref + kRescaleStep16 ? mx : m_ref;   // also on the first tile (m_ref = -inf)
        // first tile: nothing accumulated yet, so no rescale (the factor 1 spares the pass over X)
        alpha = m_ref == -INFINITY ? 1.0f : __builtin_amdgcn_exp2f(m_ref - m_new);
        m_ref = m_new;
    };
    auto sm_stage3 = [&]() {                                          // probabilities and running sum
        if (!owner) return;
        l_sum *= alpha;
#pragma unroll
        for (int j = 0; j < 4; ++j) { pr[j] = __builtin_amdgcn_exp2f(sv[j] - m_ref); l_sum += pr[j]; }
    };
    auto sm_stage4 = [&](int buf) {                                   // publish P (fp16, RNE) and the factors
        if (!owner) return;
        const h2 p01 = __builtin_convertvector(f2{pr[0], pr[1]}, h2), p23 = __builtin_convertvector(f2{pr[2], pr[3]}, h2);
        *(h4 *)(Px + buf * (NB * 32 * 16) + (16 * w + sr) * 16 + 4 * sq) = h4{p01[0], p01[1], p23[0], p23[1]};
        if (sq == 0) Ax[buf * (NB * 32) + 16 * w + sr] = alpha;
    };

    // ---- weighted sum of tile kk over this wavefront's columns: X^T[d, r] += sum_t H[t, d] P[r, t];
    //      with SM, the softmax stages of tile kk+1 ride between its MFMAs ----
    constexpr int PD = MB < 4 ? MB : 4;                               // transposing reads kept in flight (blocks)
    s4 tb[PD][2];
    h8 P[NB];
    float al[NB];
    auto pv_loads = [&](int kk) {                                     // operands that do not depend on the barrier
        const EL_LDS(char) *F = Tl + (kk & 3) * SLOT;
        const int buf = kk & 1;
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            P[nb] = *(const h8 *)(Px + buf * (NB * 32 * 16) + (32 * nb + r32) * 16 + 8 * kg);
            al[nb] = Ax[buf * (NB * 32) + 32 * nb + r32];
        }
#pragma unroll
        for (int mb = 0; mb < PD; ++mb) {
            tb[mb][0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((EL_LDS(s4) *)(F + b_lo[mb & 3] + (mb >> 2) * 256));
            tb[mb][1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((EL_LDS(s4) *)(F + b_hi[mb & 3] + (mb >> 2) * 256));
        }
    };
    auto pv = [&](int kk, auto sm_tag) {
        constexpr bool SM = decltype(sm_tag)::value;
        const EL_LDS(char) *F = Tl + (kk & 3) * SLOT;
        const int kt_next = k0 + kk + 1;
        if (SM) sm_load();
        bool resc = al[0] != 1.0f;
        if (NB > 1) resc = resc || al[NB - 1] != 1.0f;
        if (__any(resc)) {
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) {
                    // one accumulator tuple at a time through arch VGPRs; the empty asm statements pin
                    // the register classes so the allocator does not move the whole array at once
                    f16v t = X[mb][nb];
                    asm volatile("" : "+v"(t));
#pragma unroll
                    for (int i = 0; i < 16; ++i) t[i] *= al[nb];
                    asm volatile("" : "+a"(t));
                    X[mb][nb] = t;
                }
            }
        }
        constexpr int S0 = MB >= 8 ? 1 : 0;                            // block after which softmax stage 1 runs
        auto packed = [&](int mb) {
            const s4 lo = tb[mb % PD][0], hi = tb[mb % PD][1];
            return __builtin_bit_cast(u4, s8{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]});
        };
        constexpr int WPM = 4 / NB;                                    // words converted per MFMA
        u4 cur = packed(0);
        if (BF16) {
            cur.x = bf16x2_to_f16x2_ds(cur.x); cur.y = bf16x2_to_f16x2_ds(cur.y);
            cur.z = bf16x2_to_f16x2_ds(cur.z); cur.w = bf16x2_to_f16x2_ds(cur.w);
        }
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            u4 nxt = packed(mb + 1 < MB ? mb + 1 : mb);
            __builtin_amdgcn_sched_barrier(0);
            if (mb + PD < MB) {                                        // into the block `cur` came from
                tb[mb % PD][0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((EL_LDS(s4) *)(F + b_lo[(mb + PD) & 3] + ((mb + PD) >> 2) * 256));
                tb[mb % PD][1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((EL_LDS(s4) *)(F + b_hi[(mb + PD) & 3] + ((mb + PD) >> 2) * 256));
            }
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                __builtin_amdgcn_sched_barrier(0);
                X[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(h8, cur), P[nb], X[mb][nb], 0, 0, 0);
                if (BF16 && mb + 1 < MB) {
#pragma unroll
                    for (int e = 0; e < WPM; ++e) {
                        nxt[nb * WPM + e] = bf16x2_to_f16x2_ds(nxt[nb * WPM + e]);
                        asm volatile("" : "+v"(nxt[nb * WPM + e]));           // keeps the conversion behind this MFMA
                    }
                }
            }
            __builtin_amdgcn_sched_barrier(0);
            if (SM) {
                if (mb == S0) sm_stage1(kt_next);
                if (mb == S0 + 1) sm_stage2();
                if (mb == S0 + 2) sm_stage3();
                if (mb == S0 + 3) sm_stage4((kk + 1) & 1);
                __builtin_amdgcn_sched_barrier(0);
            }
            cur = nxt;
        }
    };

    // Tile j's scores and softmax run one tile ahead of its weighted sum.  What crosses the barriers:
    //   B1(j): the partial scores of tile j are in LDS;
    //   B2(j): P and the rescale factors of tile j are in LDS (buffer j&1; the weighted sum of tile j-1
    //          took its operands from the other buffer before B1(j)); every wavefront has left the
    //          weighted sum of tile j-1, so that tile's slot may be refilled (tile j+3 goes there, requested
    //          at the start of the scores of tile j+1), and has waited for its own rows of tile j+1.
    if (nloc > 0) {
        scores(0);
        __syncthreads();                                              // B1(0)
        sm_load(); sm_stage1(k0); sm_stage2(); sm_stage3(); sm_stage4(0);
        wait_own(1);
        if (nloc > 1) zero_ragged(k0 + 1, 1);
        __syncthreads();                                              // B2(0)
        for (int kk = 1; kk < nloc; ++kk) {
            scores(kk);
            pv_loads(kk - 1);
            __syncthreads();                                          // B1(kk)
            pv(kk - 1, std::true_type{});
            wait_own(1);
            if (kk + 1 < nloc) zero_ragged(k0 + kk + 1, (kk + 1) & 3);
            __syncthreads();                                          // B2(kk)
        }
        pv_loads(nloc - 1);
        pv(nloc - 1, std::false_type{});
    }

    // the last fetches went to the dump area; none may be in flight when the workgroup gives up its LDS
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");

    // ---- partial result: statistics from the owner wavefronts, X normalised by its own sum ----
    const int parts = a.S, part = s;
    if (w < RG) {
        l_sum += quad_xor1(l_sum);
        l_sum += quad_xor2(l_sum);
        const int sr = l >> 2, row = row0 + 16 * w + sr;
        if ((l & 3) == 0) {
            Linv[16 * w + sr] = l_sum > 0.f ? 1.0f / l_sum : 0.f;
            if (row < a.R) {
                float *ml_out = a.ML + (((size_t)b * parts + part) * a.Rs + row) * 2;
                ml_out[0] = m_ref; ml_out[1] = l_sum;
            }
        }
    }
    __syncthreads();
    if (nloc <= 0) return;                            // nothing accumulated: the merge skips sum == 0

    // stage [row][d] in fp16 over the tile slots (8-byte units XOR-swizzled by the row to spread the
    // banks), then every wavefront writes 16 rows, 1 KB per store instruction
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        const float inv = Linv[32 * nb + r32];
        const int srow = 32 * nb + r32;
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const f16v x = X[mb][nb];
                const h2 lo = __builtin_convertvector(f2{x[4 * q4 + 0] * inv, x[4 * q4 + 1] * inv}, h2);
                const h2 hi = __builtin_convertvector(f2{x[4 * q4 + 2] * inv, x[4 * q4 + 3] * inv}, h2);
                const int d = DS * w + 32 * mb + 8 * q4 + 4 * kg;        // four consecutive columns
                *(h4 *)(T + srow * ROWB + (((d >> 2) ^ (srow & 31)) << 3)) = h4{lo[0], lo[1], hi[0], hi[1]};
            }
        }
    }
    __syncthreads();
    f16_t *x_out = a.Xp + (((size_t)b * parts + part) * a.Rs + row0) * DM;
    constexpr int ROWS_PER_WAVE = NB * 32 / 4;
#pragma unroll
    for (int i = 0; i < ROWS_PER_WAVE; ++i) {
        const int srow = ROWS_PER_WAVE * w + i;
#pragma unroll
        for (int hf = 0; hf < DM / 512; ++hf) {
            if (srow >= 16 * RG || row0 + srow >= a.R) continue;
            const int u0 = hf * 128 + 2 * l;
            const h4 v0 = *(const h4 *)(T + srow * ROWB + ((u0 ^ (srow & 31)) << 3));
            const h4 v1 = *(const h4 *)(T + srow * ROWB + (((u0 + 1) ^ (srow & 31)) << 3));
            *(h8 *)(x_out + (size_t)srow * DM + hf * 512 + 8 * l) = h8{v0[0], v0[1], v0[2], v0[3], v1[0], v1[1], v1[2], v1[3]};
        }
    }
}

// ---------------------------------------------------------------------------------------------
// With a pair of events the launch carries them itself (they then read the dispatch's own begin and end,
// without the command-processor time a separately recorded event adds on either side).
template <int DM, bool BF16, int RG>
static void launch_ds_one(const CoreArgs &a, dim3 grid, hipStream_t s, hipEvent_t ev0, hipEvent_t ev1)
{
    if (ev0 && ev1) hipExtLaunchKernelGGL((k_core_ds<DM, BF16, RG>), grid, dim3(256), 0, s, ev0, ev1, 0, a);
    else hipLaunchKernelGGL((k_core_ds<DM, BF16, RG>), grid, dim3(256), 0, s, a);
}

template <int DM, bool BF16>
static hipError_t launch_ds_t(const CoreArgs &a, int rg, hipStream_t s, hipEvent_t ev0, hipEvent_t ev1)
{
    const int groups = a.B * a.S;
    const dim3 grid(((groups + 7) / 8) * 8 * a.nblocks);
    switch (rg) {
    case 1: launch_ds_one<DM, BF16, 1>(a, grid, s, ev0, ev1); break;
    case 2: launch_ds_one<DM, BF16, 2>(a, grid, s, ev0, ev1); break;
    default: launch_ds_one<DM, BF16, 4>(a, grid, s, ev0, ev1); break;
    }
    return hipGetLastError();
}

hipError_t launch_core_ds(const CoreArgs &a, int d_m, bool bf16, int rg, hipStream_t s, hipEvent_t ev0, hipEvent_t ev1)
{
    if (d_m == 1024) return bf16 ? launch_ds_t<1024, true>(a, rg, s, ev0, ev1) : launch_ds_t<1024, false>(a, rg, s, ev0, ev1);
    if (d_m == 512) return bf16 ? launch_ds_t<512, true>(a, rg, s, ev0, ev1) : launch_ds_t<512, false>(a, rg, s, ev0, ev1);
    return hipErrorInvalidValue;
}

} // namespace el
