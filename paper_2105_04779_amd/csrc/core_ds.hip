// MFMA attention core for gfx950, steps a3-a5 of the EL-attention decode step (Algorithm 3's two
// products over the hidden states and the softmax between them; Eq. 9 with K = V = H).
//
// One workgroup (4 wavefronts, one per SIMD) owns a contiguous range of 16-row tiles of one batch
// element's H and up to 64 expanded-query rows.  The four wavefronts split the MODEL dimension:
// wavefront w owns columns [w d_m/4, (w+1) d_m/4) of H for both products, so every byte of a tile
// is read from LDS exactly twice per workgroup (once per product), whatever the number of rows.
//
//   fetch      each 1 KB piece of a tile row goes straight from HBM into one of four LDS tile
//              slots (global_load_lds, no registers in flight; three tiles are outstanding while
//              one is being used).  Lane i of a piece fetches chunk i ^ swizzle(row): the tile
//              lands in the XOR-swizzled order that keeps both operand read patterns spread over
//              all banks.  A wavefront converts exactly the rows it fetched (bf16 -> fp16, in
//              place), so landing needs no cross-wave handshake; the conversion of tile k+1 is
//              interleaved with the score MFMAs of tile k.
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
// Scores arrive pre-multiplied by log2(e)/sqrt(d_k), so the softmax is an exp2 of a difference.
// The partial result (one per key-range split) leaves normalised by its own sum, in fp16, through
// LDS so that every global store instruction writes 1 KB of one row.
#include <type_traits>
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

#ifdef EL_CORE_PROF
#define EL_PROF_DECL unsigned long long prof_t = clock64(), prof_acc[12] = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#define EL_PROF(i) { const unsigned long long now = clock64(); prof_acc[i] += now - prof_t; prof_t = now; }
#else
#define EL_PROF_DECL
#define EL_PROF(i)
#endif

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
    constexpr int CH = 4 * ROWB / 1024;             // 16-byte chunks per lane in a wavefront's 4 rows
    constexpr int CW16 = DS * 2;                    // byte offset step of a wavefront's column slice
    static_assert(ROWB % 1024 == 0 && KC >= 4 && KC % 4 == 0, "d_m must be a multiple of 512");
    static_assert(RG == 1 || RG == 2 || RG == 4, "row groups per workgroup");

    __shared__ __attribute__((aligned(1024))) char T[NSLOT * SLOT];
    __shared__ __attribute__((aligned(16))) float Sx[4 * RG * 64 * 4];   // partial scores [wave][rg][lane][4]
    __shared__ __attribute__((aligned(16))) f16_t Px[NB * 32 * 16];      // probabilities [row][t]
    __shared__ float Ax[NB * 32];                                        // per-row rescale factor / final 1/sum
    __shared__ int Fx[4];                                                // per row group: some row rescales
    __shared__ __attribute__((aligned(1024))) char Dz[ROWB];             // where fetches of rows that do not exist land

    const int tid = threadIdx.x, l = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r16 = l & 15, g = l >> 4, r32 = l & 31, kg = l >> 5;

    // workgroup -> (batch element, key split, row block); workgroups that share an H range differ
    // by multiples of 8 so they are dispatched to the same XCD (same L2).
    const int id = blockIdx.x;
    const int oct = id / (8 * a.nblocks), rem = id % (8 * a.nblocks);
    const int rb = rem >> 3, group = oct * 8 + (rem & 7);
    if (group >= a.B * a.S) return;
    const int b = group / a.S, s = group % a.S;
    const int row0 = rb * (16 * RG);                 // first expanded-query row of this workgroup

    int len = a.lengths ? a.lengths[b] : a.n;
    len = min(max(len, 1), a.n);
    const int NT = (len + kTileRows16 - 1) / kTileRows16;
    const int k0 = (int)(((int64_t)NT * s) / a.S), k1 = (int)(((int64_t)NT * (s + 1)) / a.S);
    const int nloc = k1 - k0;
    const char *Hb = (const char *)a.H + (size_t)b * a.h_stride * 2;

    // ---- this wavefront's column slice of ELQ, all row groups: B operand of the score product ----
    h8 elq[RG][KC];
#pragma unroll
    for (int rg = 0; rg < RG; ++rg) {
        const int row = row0 + 16 * rg + r16;
        // pad rows (row >= R) are never written by the expansion step: they read as zero here
        const f16_t *src = a.elq + ((size_t)b * a.Rs + row) * DM + DS * w + 8 * g;
        const h8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
        for (int c = 0; c < KC; ++c) elq[rg][c] = row < a.R ? *(const h8 *)(src + 32 * c) : zero;
    }

    f16v X[MB][NB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int i = 0; i < 16; ++i) X[mb][nb][i] = 0.f;
    float m_ref = -INFINITY, l_sum = 0.f;           // meaningful in owner wavefronts (w < RG) only

    if (tid < NB * 32) Ax[tid] = 1.0f;
    for (int i = tid; i < NB * 32 * 16; i += 256) Px[i] = (f16_t)0.f;
    if (tid < 4) Fx[tid] = 0;

    // ---- per-lane LDS offsets inside a tile slot ----
    const EL_LDS(char) *Tl = (const EL_LDS(char) *)T;
    const unsigned t_lds = (unsigned)(uintptr_t)Tl;
    const unsigned dz_lds = (unsigned)(uintptr_t)(const EL_LDS(char) *)Dz;
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

    // A wavefront fetches rows 4w..4w+3 of every tile, always with the same number of instructions: a row
    // that does not exist (at or beyond len, or of a tile past this workgroup's range) is replaced by a
    // fetch of the element's first row into a dump area.  The fetch counter then advances by exactly NI
    // per tile, and the loop needs neither branches around the requests nor per-tile wait arithmetic.
    auto issue_dma_row = [&](int kt, int slot, int i) {
        const bool ok = kt < k1 && kt * kTileRows16 + 4 * w + i < len;               // wave-uniform
        const char *sbase = ok ? Hb + ((size_t)kt * kTileRows16 + 4 * w) * ROWB : Hb - i * ROWB;
        const int f = (i << 2) | w;                                                   // tile_swizzle(4w + i)
        const unsigned voff = (unsigned)(((l ^ f) << 4) + i * ROWB);
        const unsigned dst = ok ? t_lds + slot * SLOT + (4 * w + i) * ROWB : dz_lds;
        if (PIECES == 2) dma_row_2k(dst, voff, sbase);
        else dma_piece(dst, voff, sbase);
    };
    auto issue_dma = [&](int kt, int slot) {
#pragma unroll
        for (int i = 0; i < 4; ++i) issue_dma_row(kt, slot, i);
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
    // score-product fragments of one tile: row r16, this wavefront's columns (storage bits)
    u4 hb[KC];
    auto load_hb = [&](const EL_LDS(char) *F, int c) { hb[c] = *(const EL_LDS(u4) *)(F + a_base[c & 3] + (c >> 2) * 256); };

    EL_PROF_DECL
    // ---- prologue: request three tiles, wait for the first ----
    if (nloc > 0) {
        issue_dma(k0, 0);
        issue_dma(k0 + 1, 1);
        issue_dma(k0 + 2, 2);
        wait_own(2);
        zero_ragged(k0, 0);
    }
    // The compiler does not see the LDS-DMA requests; it does see the ELQ loads above, and would place
    // their wait (which also drains every later fetch) in front of the first MFMA of EVERY iteration.
    // Consuming the registers here, on every path into the loop, moves that wait out of it.
#pragma unroll
    for (int rg = 0; rg < RG; ++rg)
#pragma unroll
        for (int c = 0; c < KC; ++c) asm volatile("" :: "v"(elq[rg][c]));
    __syncthreads();
#pragma unroll
    for (int c = 0; c < KC; ++c) load_hb(Tl, c);
    EL_PROF(0)

    // Per tile: scores -> B1 -> softmax -> B2 -> weighted sum.  What crosses the barriers:
    //   B1(k): the partial scores of tile k are in LDS; every wavefront has left the weighted sum of tile
    //          k-1, so that tile's slot may be refilled (tile k+3 is requested into it after B2(k));
    //   B2(k): P, rescale factors and flags of tile k are in LDS; every wavefront has waited for its own
    //          rows of tile k+1, so tile k+1 may be read (its score fragments are requested during the
    //          weighted sum of tile k and arrive under those MFMAs).
    for (int kk = 0; kk < nloc; ++kk) {
        const int kt = k0 + kk;
        const int slot = kk & 3;
        const EL_LDS(char) *Fl = Tl + slot * SLOT;
        const EL_LDS(char) *Fn = Tl + ((kk + 1) & 3) * SLOT;
        const bool more = kk + 1 < nloc;
        EL_PROF(1)

        // ---- partial scores over this wavefront's columns.  One wavefront per SIMD: the conversion of
        //      the next fragment is issued behind each MFMA and runs while the matrix unit is busy ----
        f4 sc[RG];
#pragma unroll
        for (int rg = 0; rg < RG; ++rg) sc[rg] = f4{0.f, 0.f, 0.f, 0.f};
        {
            constexpr int WPM = 4 / RG;                                // words converted per MFMA
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
                            asm volatile("" : "+v"(nxt[rg * WPM + e]));       // keeps the conversion behind this MFMA
                        }
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
                cur = nxt;
            }
        }
#pragma unroll
        for (int rg = 0; rg < RG; ++rg) *(f4 *)(Sx + ((w * RG + rg) * 64 + l) * 4) = sc[rg];
        EL_PROF(2)
        __syncthreads();                                              // B1
        EL_PROF(3)

        // the first operand blocks of the weighted sum do not depend on the softmax: request them now
        constexpr int PD = MB < 4 ? MB : 4;                           // transposing reads kept in flight (blocks)
        s4 tb[PD][2];
        auto load_tb = [&](int mb) {
            tb[mb % PD][0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((EL_LDS(s4) *)(Fl + b_lo[mb & 3] + (mb >> 2) * 256));
            tb[mb % PD][1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((EL_LDS(s4) *)(Fl + b_hi[mb & 3] + (mb >> 2) * 256));
        };
#pragma unroll
        for (int mb = 0; mb < PD; ++mb) load_tb(mb);

        // ---- softmax bookkeeping of row group w (row = lane%16; its 16 scores sit in 4 lanes x 4 registers) ----
        if (w < RG) {
            // lane = 4 * row + q holds positions 4q..4q+3 of its row: the row's statistics stay inside a quad
            const int sr = l >> 2, sq = l & 3, src_lane = sr + 16 * sq;
            f4 t0 = *(const f4 *)(Sx + ((0 * RG + w) * 64 + src_lane) * 4), t1 = *(const f4 *)(Sx + ((1 * RG + w) * 64 + src_lane) * 4);
            f4 t2 = *(const f4 *)(Sx + ((2 * RG + w) * 64 + src_lane) * 4), t3 = *(const f4 *)(Sx + ((3 * RG + w) * 64 + src_lane) * 4);
            float sv[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) sv[j] = (t0[j] + t1[j]) + (t2[j] + t3[j]);
            if ((kt + 1) * kTileRows16 > len) {      // ragged last tile: positions at or beyond len do not exist
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (kt * kTileRows16 + 4 * sq + j >= len) sv[j] = -INFINITY;
            }
            float mx = fmaxf(fmaxf(sv[0], sv[1]), fmaxf(sv[2], sv[3]));
            mx = fmaxf(mx, quad_xor1(mx));
            mx = fmaxf(mx, quad_xor2(mx));
            const bool grow = mx > m_ref + kRescaleStep16;   // also true on the first tile (m_ref = -inf)
            const bool any_grow = __any(grow);
            float alpha = 1.0f;
            if (grow) { alpha = __builtin_amdgcn_exp2f(m_ref - mx); m_ref = mx; }
            l_sum *= alpha;
            float pr[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) { pr[j] = __builtin_amdgcn_exp2f(sv[j] - m_ref); l_sum += pr[j]; }
            const h2 p01 = __builtin_convertvector(f2{pr[0], pr[1]}, h2), p23 = __builtin_convertvector(f2{pr[2], pr[3]}, h2);
            *(h4 *)(Px + (16 * w + sr) * 16 + 4 * sq) = h4{p01[0], p01[1], p23[0], p23[1]};
            if (sq == 0) Ax[16 * w + sr] = alpha;
            if (l == 0) Fx[w] = any_grow ? 1 : 0;
        }
        // our rows of tile k+1 must have landed before B2 hands the tile over (tile k+2 may still fly)
        wait_own(1);
        if (more) zero_ragged(kt + 1, (kk + 1) & 3);
        EL_PROF(4)
        __syncthreads();                                              // B2
        EL_PROF(5)

        // ---- weighted sum over this wavefront's columns: X^T[d, r] += sum_t H[t, d] P[r, t] ----
        {
            int any = 0;
#pragma unroll
            for (int rg = 0; rg < RG; ++rg) any |= Fx[rg];
            h8 P[NB];
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) P[nb] = *(const h8 *)(Px + (32 * nb + r32) * 16 + 8 * kg);
            if (any) {
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
                    const float alpha = Ax[32 * nb + r32];
#pragma unroll
                    for (int mb = 0; mb < MB; ++mb) {
                        // one accumulator tuple at a time through arch VGPRs; the empty asm statements pin
                        // the register classes so the allocator does not move the whole array at once
                        f16v t = X[mb][nb];
                        asm volatile("" : "+v"(t));
#pragma unroll
                        for (int i = 0; i < 16; ++i) t[i] *= alpha;
                        asm volatile("" : "+a"(t));
                        X[mb][nb] = t;
                    }
                }
            }
            // One code path only: a second copy of this block makes the compiler reconcile two versions of
            // the accumulators where the paths meet, at the price of hundreds of spilled registers.
            constexpr int WPM = 4 / NB;                                // words converted per MFMA
            auto packed = [&](int mb) {
                const s4 lo = tb[mb % PD][0], hi = tb[mb % PD][1];
                return __builtin_bit_cast(u4, s8{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]});
            };
            u4 cur = packed(0);
            if (BF16) {
                cur.x = bf16x2_to_f16x2_ds(cur.x); cur.y = bf16x2_to_f16x2_ds(cur.y);
                cur.z = bf16x2_to_f16x2_ds(cur.z); cur.w = bf16x2_to_f16x2_ds(cur.w);
            }
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) {
                u4 nxt = packed(mb + 1 < MB ? mb + 1 : mb);
                __builtin_amdgcn_sched_barrier(0);
                if (mb + PD < MB) load_tb(mb + PD);                    // into the block `cur` came from
                // the fetch of tile k+3 goes into the slot tile k-1 left before B1
                if (mb < 4) issue_dma_row(kt + 3, (kk + 3) & 3, mb);
                // the score fragments of tile k+1, two per block over the second half of the blocks (after
                // the last tile they read a slot nobody uses)
                if (mb >= MB / 2) { load_hb(Fn, 2 * (mb - MB / 2)); load_hb(Fn, 2 * (mb - MB / 2) + 1); }
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
                    __builtin_amdgcn_sched_barrier(0);
                    X[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(h8, cur), P[nb], X[mb][nb], 0, 0, 0);
                    if (BF16 && mb + 1 < MB) {
#pragma unroll
                        for (int e = 0; e < WPM; ++e) {
                            nxt[nb * WPM + e] = bf16x2_to_f16x2_ds(nxt[nb * WPM + e]);
                            asm volatile("" : "+v"(nxt[nb * WPM + e]));       // keeps the conversion behind this MFMA
                        }
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
                cur = nxt;
            }
        }
        EL_PROF(6)
        EL_PROF(7)
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
            Ax[16 * w + sr] = l_sum > 0.f ? 1.0f / l_sum : 0.f;
            if (row < a.R) {
                float *ml_out = a.ML + (((size_t)b * parts + part) * a.Rs + row) * 2;
                ml_out[0] = m_ref; ml_out[1] = l_sum;
            }
        }
    }
    __syncthreads();
    EL_PROF(9)
    if (nloc <= 0) return;                            // nothing accumulated: the merge skips sum == 0

    // stage [row][d] in fp16 over the tile slots (8-byte units XOR-swizzled by the row to spread the
    // banks), then every wavefront writes 16 rows, 1 KB per store instruction
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        const float inv = Ax[32 * nb + r32];
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
    EL_PROF(10)
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
#ifdef EL_CORE_PROF
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    EL_PROF(11)
    if (blockIdx.x == 0 && threadIdx.x == 0 && a.prof) {
        for (int i = 0; i < 12; ++i) a.prof[i] = prof_acc[i];
        a.prof[12] = (unsigned long long)nloc;
    }
#endif
}

// ---------------------------------------------------------------------------------------------
template <int DM, bool BF16>
static hipError_t launch_ds_t(const CoreArgs &a, int rg, hipStream_t s)
{
    const int groups = a.B * a.S;
    const dim3 grid(((groups + 7) / 8) * 8 * a.nblocks), block(256);
    switch (rg) {
    case 1: hipLaunchKernelGGL((k_core_ds<DM, BF16, 1>), grid, block, 0, s, a); break;
    case 2: hipLaunchKernelGGL((k_core_ds<DM, BF16, 2>), grid, block, 0, s, a); break;
    default: hipLaunchKernelGGL((k_core_ds<DM, BF16, 4>), grid, block, 0, s, a); break;
    }
    return hipGetLastError();
}

hipError_t launch_core_ds(const CoreArgs &a, int d_m, bool bf16, int rg, hipStream_t s)
{
    if (d_m == 1024) return bf16 ? launch_ds_t<1024, true>(a, rg, s) : launch_ds_t<1024, false>(a, rg, s);
    if (d_m == 512) return bf16 ? launch_ds_t<512, true>(a, rg, s) : launch_ds_t<512, false>(a, rg, s);
    return hipErrorInvalidValue;
}

} // namespace el
