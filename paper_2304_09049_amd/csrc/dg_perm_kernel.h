// The tuned table kernel for gfx950: table rows live in registers and products are fetched with
// v_perm_b32, four per lane-instruction.
//
// How the 16-entry table (Sec. 3 "LUT-16") meets an 8-byte permute pool
//   v_perm_b32 picks each of its 4 result bytes out of an 8-byte pool {S0,S1}.  A table ROW
//   (the four products of one weight code with the four activation codes) is 4 bytes, so the pair
//   {row[w(m,k+1)], row[w(m,k)]} is a pool that serves two reduction positions of one weight row m.
//   The selector then depends on activation codes only: a(n,k) picks from the low half, 4 + a(n,k+1)
//   from the high half.  One permute therefore fetches the four products
//       (m, n0, k) (m, n0, k+1) (m, n1, k) (m, n1, k+1).
//   Pools depend on the weight tile only and selectors on the activation tile only, so both are
//   expanded ONCE per tile into LDS by the whole workgroup and then re-used: each pool by every
//   column of the tile, each selector by every row.  The unpacking work (the paper's measured
//   bottleneck, Sec. 5.4: ~80 % of its kernel) drops from O(M*N*K) to O((M+N)*K); the O(M*N*K)
//   loop is one permute plus half an add per four products.
//
// Accumulation (Sec. 3: 8-bit vertical adds, then a horizontal add; here exact int32)
//   Table entries are biased to be >= 0 (entry - min_entry <= 31), so four byte lanes of a register
//   can be added with plain 32-bit adds without carries between lanes for `flush` steps; then the
//   byte lanes are folded into int32 accumulators (v_dot4_u32_u8 against a 0/1 mask).  The bias is
//   taken out at the end: C = sum' + min_entry * (number of reduction positions that contributed).
//
// Wide tables (entry - min_entry up to 255, i.e. every int8 table): MODE = 1 fetches two products per
// permute instead of four, each zero-extended into a 16-bit lane (selector bytes 1 and 3 are 0x0C), so that
// lanes can take 65535 / range adds before they are folded into int32.  Half the rate, same exact result.
//
// Implicit im2col (NHWC): reduction index k = (kh*KW + kw)*Cin + ci.  The loader computes the source
// pixel of every (output pixel, filter tap) and, for taps outside the image (and rows beyond N,
// positions beyond K), writes the selector 0x0C, for which v_perm_b32 returns the constant 0:
// such positions add nothing, whatever the table holds.
//
// Small problems: SK > 1 splits K over SK groups of lanes inside one workgroup.  Each group owns the
// whole output tile for its share of the K stages, with LDS buffers of its own; the partial sums
// meet in LDS (integer atomics: any order gives the same sum) and group 0 stores.
#pragma once
#include "dg_common.h"

namespace dgperm {

typedef DgFastDiv FastDiv;

struct PermArgs {
    DgProblem p;
    uint32_t rows[4];       // biased table rows: byte a of rows[w] = LUT[4w+a] - min_entry
    int32_t min_entry;
    int32_t flush_dwords;   // fold the narrow lanes into int32 after this many 16-code groups
    int32_t tiles_m;
    FastDiv div_ow, div_oh, div_cin, div_kw;
    // how (tap, channel) moves when a group steps from one of its stages to the next (KS*SK codes)
    int32_t step_ci, step_kw, step_kh;
};

__device__ __forceinline__ uint32_t fdiv(uint32_t n, const FastDiv &f) { return dg_fdiv(n, f); }

__device__ __forceinline__ uint32_t perm(uint32_t hi, uint32_t lo, uint32_t sel)
{
    return __builtin_amdgcn_perm(hi, lo, sel);
}

// sum of the masked byte lanes of `v`, added to acc
__device__ __forceinline__ int32_t fold_bytes(uint32_t v, uint32_t ones, int32_t acc)
{
    return (int32_t)__builtin_amdgcn_udot4(v, ones, (uint32_t)acc, false);
}

// Waves per SIMD the compiler is asked to leave room for (it sizes its register budget to this).  Measured: the
// 16-bit-lane 8x8 tile gains from three waves per SIMD; every other shape is fastest with the compiler's own choice.
#ifndef DG_PERM_MIN_WAVES
#define DG_PERM_MIN_WAVES(TM, TN, SK, MODE) (((SK) == 1 && (MODE) == 1 && (TM) * (TN) == 64) ? 3 : 1)
#endif

template <int TM, int TN, int LM, int LN, int KS, int SK, int NBUF, int MODE>
struct PermShape {
    static constexpr int GT = LM * LN;         // lanes of one K-split group
    static constexpr int NT = GT * SK;         // lanes of the workgroup
    static constexpr int BM = LM * TM, BN = LN * TN, NP = BN / 2;
    static constexpr int QS = KS / 2;          // pools (pairs of reduction positions) per stage
    static constexpr int DW = KS / 16;         // 32-bit packed words per row per stage
    static constexpr int POOL_BYTES = NBUF * QS * BM * 8;   // per group, NBUF stages
    static constexpr int SELW = MODE == 1 ? 2 : 1;   // selector words per (pair q, column pair)
    // selector words one lane reads per pair q, padded to whole 128-bit reads (matters for TN = 14: 7 -> 8)
    static constexpr int SPL = (TN / 2 * SELW + 3) / 4 * 4 > TN / 2 * SELW && TN / 2 * SELW > 4 ? (TN / 2 * SELW + 3) / 4 * 4
                                                                                                : TN / 2 * SELW;
    static constexpr int SROW = LN * SPL;            // selector words per pair q
    static constexpr int SEL_BYTES = NBUF * QS * SROW * 4;
    static constexpr int RED_BYTES = SK > 1 ? TM * TN * GT * 4 : 0;
    static constexpr int LDS_BYTES = 128 + SK * (POOL_BYTES + SEL_BYTES) + RED_BYTES;
};

// TM x TN outputs per lane; LM x LN lanes per group; KS codes of K per LDS stage; SK K-split groups;
// NBUF = 2 overlaps the expansion of the next stage with the permutes of the current one, NBUF = 1 halves the
// LDS footprint (meant for shapes where every group has a single, long stage).
template <int TM, int TN, int LM, int LN, int KS, int SK, int NBUF, int MODE, bool MFAST>
__global__ void __launch_bounds__(LM *LN *SK, DG_PERM_MIN_WAVES(TM, TN, SK, MODE))
perm_lut_kernel(PermArgs a)
{
    using S = PermShape<TM, TN, LM, LN, KS, SK, NBUF, MODE>;
    constexpr int GT = S::GT, BM = S::BM, BN = S::BN, NP = S::NP, QS = S::QS, DW = S::DW, SELW = S::SELW;
    constexpr int SPL = S::SPL, SROW = S::SROW;
    static_assert(TM % 2 == 0 && TN % 2 == 0 && KS % 16 == 0, "tile shape");

    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x;
    const int g = SK > 1 ? tid / GT : 0;          // K-split group of this lane
    const int t = SK > 1 ? tid % GT : tid;        // lane within the group
    uint2 *s_table = (uint2 *)smem;               // pool for every value of a weight nibble
    // {row[w(k)], row[w(k+1)]} per (pair q, weight row).  Row ml*TM + i sits at slot (i/2)*2*LM + 2*ml + i%2, so that
    // the 128-bit reads of consecutive lanes (two rows each) fall on consecutive 16-byte chunks: no bank conflicts.
    uint2 *s_pool = (uint2 *)(smem + 128 + g * (S::POOL_BYTES + S::SEL_BYTES));          // [2][QS][BM]
    uint32_t *s_sel = (uint32_t *)((unsigned char *)s_pool + S::POOL_BYTES);            // [2][QS][NP]
    int32_t *s_red = (int32_t *)(smem + 128 + SK * (S::POOL_BYTES + S::SEL_BYTES));      // [TM*TN][GT]

    const DgProblem &p = a.p;
    const int ml = MFAST ? t % LM : t / LN;
    const int nl = MFAST ? t / LM : t % LN;
    const int tile_m = blockIdx.x % a.tiles_m;
    const int tile_n = blockIdx.x / a.tiles_m;
    const int m_base = tile_m * BM;
    const int n_base = tile_n * BN;
    const int cq = p.Cin / 4;                     // packed bytes per pixel

    if (tid < 16) s_table[tid] = make_uint2(a.rows[tid & 3], a.rows[tid >> 2]);
    if (SK > 1) {
#pragma unroll
        for (int i = 0; i < TM * TN; ++i)
            if (g == 0) s_red[i * GT + t] = 0;
    }
    __syncthreads();            // the pool table is visible; taken here, where every wave arrives at the same time

    // the per-row scales of the epilogue are requested now so that their latency hides behind the K loop
    const int m_first = m_base + ml * TM, n_first = n_base + nl * TN;
    float sc[TM];
    if (p.scale && g == 0) {
#pragma unroll
        for (int i = 0; i < TM; ++i) sc[i] = p.scale[min(m_first + i, p.M - 1)];
    }

    // ---- loader tasks (fixed per lane for the whole K loop) ---------------------------------
    // weight side: (LDS slot, word) -> 8 pools;  activation side: (column pair, word) -> 8 selectors
    constexpr int WTASKS = BM * DW, WPER = (WTASKS + GT - 1) / GT;
    constexpr int ATASKS = NP * DW, APER = (ATASKS + GT - 1) / GT;

    // When the group's lane count is a multiple of the tile's rows (column pairs), a lane keeps the same weight
    // row (column pair) in all of its tasks and only the word index moves: the address set-up is done once.
    constexpr bool W_FIXED = GT % BM == 0, A_FIXED = GT % NP == 0;
    const uint32_t *w_ptr[WPER];
    int w_slot[WPER], w_d[WPER];
#pragma unroll
    for (int i = 0; i < WPER; ++i) {
        const int task = t + i * GT;
        // consecutive lanes own consecutive LDS slots; the weight row follows from the slot
        w_slot[i] = W_FIXED ? t % BM : task % BM;
        w_d[i] = W_FIXED ? t / BM + i * (GT / BM) : task / BM;
        if (i == 0 || !W_FIXED) {
            const int slot = w_slot[i];
            const int row = ((slot >> 1) % LM) * TM + 2 * (slot / (2 * LM)) + (slot & 1);
            int m = m_base + row;
            if (m >= p.M) m = p.M - 1;                   // rows beyond M: read a valid row, never stored
            w_ptr[i] = (const uint32_t *)(p.Wp + (int64_t)m * (p.K / 4)) + w_d[i] + g * DW;
        } else {
            w_ptr[i] = w_ptr[0] + i * (GT / BM);
        }
    }
    int a_np[APER], a_sidx[APER], a_k0[APER], a_ci[APER], a_kh[APER], a_kw[APER];
    int a_ih0[APER][2], a_iw0[APER][2];                   // top-left source pixel of the filter window
    int a_off0[APER][2];                                  // byte offset of that pixel (may be negative)
    bool a_ok[APER][2];
#pragma unroll
    for (int i = 0; i < APER; ++i) {
        const int task = t + i * GT;
        a_np[i] = A_FIXED ? t % NP : task % NP;
        a_sidx[i] = (a_np[i] / (TN / 2)) * SPL + (a_np[i] % (TN / 2)) * SELW;   // word index of the pair in a selector row
        const int d = A_FIXED ? t / NP + i * (GT / NP) : task / NP;
        a_k0[i] = g * KS + 16 * d;                        // first reduction position of this lane's word
        const uint32_t tap = fdiv((uint32_t)a_k0[i], a.div_cin);
        a_ci[i] = a_k0[i] - (int)tap * p.Cin;
        a_kh[i] = (int)fdiv(tap, a.div_kw);
        a_kw[i] = (int)tap - a_kh[i] * p.KW;
        if (i == 0 || !A_FIXED) {
            // the pair's first column by division, its second by stepping one pixel on
            const int n0 = n_base + 2 * a_np[i];
            const uint32_t nn = n0 < p.N ? (uint32_t)n0 : 0u;
            const uint32_t row = fdiv(nn, a.div_ow);              // b*OH + oh
            int ow = (int)(nn - row * (uint32_t)p.OW);
            int b = (int)fdiv(row, a.div_oh);
            int oh = (int)row - b * p.OH;
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                a_ok[i][h] = (ATASKS % GT == 0 || task < ATASKS) && (n0 + h < p.N);
                a_ih0[i][h] = oh * p.sh - p.ph;
                a_iw0[i][h] = ow * p.sw - p.pw;
                a_off0[i][h] = ((b * p.H + a_ih0[i][h]) * p.W + a_iw0[i][h]) * cq;
                if (++ow == p.OW) {
                    ow = 0;
                    if (++oh == p.OH) {
                        oh = 0;
                        ++b;
                    }
                }
            }
        } else {
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                a_ok[i][h] = a_ok[0][h] && (ATASKS % GT == 0 || task < ATASKS);
                a_ih0[i][h] = a_ih0[0][h];
                a_iw0[i][h] = a_iw0[0][h];
                a_off0[i][h] = a_off0[0][h];
            }
        }
    }

    uint32_t w_reg[WPER];
    uint32_t a_reg[APER][2];
    bool a_valid[APER][2];

    // fetch the packed words of this group's stage `it` (stage index it*SK + g); calls come with it = 0, 1, 2, ...
    auto fetch = [&](int it) {
        const int k_stage = (it * SK + g) * KS;
#pragma unroll
        for (int i = 0; i < WPER; ++i) {
            const int k0 = k_stage + 16 * w_d[i];
            const bool ok = (WTASKS % GT == 0 || t + i * GT < WTASKS) && k0 < p.K;
            w_reg[i] = ok ? w_ptr[i][it * (SK * DW)] : 0u;
        }
#pragma unroll
        for (int i = 0; i < APER; ++i) {
            const int tap_off = (a_kh[i] * p.W + a_kw[i]) * cq + (a_ci[i] >> 2);
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int ih = a_ih0[i][h] + a_kh[i], iw = a_iw0[i][h] + a_kw[i];
                const bool ok = a_ok[i][h] && a_k0[i] < p.K && ih >= 0 && ih < p.H && iw >= 0 && iw < p.W;
                a_valid[i][h] = ok;
                a_reg[i][h] = ok ? *(const uint32_t *)(p.Xp + (a_off0[i][h] + tap_off)) : 0u;
            }
            // move to this lane's word in the group's next stage
            a_k0[i] += KS * SK;
            a_ci[i] += a.step_ci;
            const int carry = a_ci[i] >= p.Cin;
            a_ci[i] -= carry ? p.Cin : 0;
            a_kw[i] += a.step_kw + carry;
            a_kh[i] += a.step_kh;
            if (a_kw[i] >= p.KW) {
                a_kw[i] -= p.KW;
                a_kh[i] += 1;
            }
        }
    };

    auto expand = [&](int buf) {
        // weights: nibble q of the word = codes (2q, 2q+1) -> the pool stored for that nibble value
#pragma unroll
        for (int i = 0; i < WPER; ++i) {
            if (WTASKS % GT != 0 && t + i * GT >= WTASKS) break;
            const uint32_t w = w_reg[i];
#pragma unroll
            for (int q = 0; q < 8; ++q)
                s_pool[(buf * QS + 8 * w_d[i] + q) * BM + w_slot[i]] = s_table[(w >> (4 * q)) & 15u];
        }
        // activations: selector bytes [a(n0,2q), 4 + a(n0,2q+1), a(n1,2q), 4 + a(n1,2q+1)]
#pragma unroll
        for (int i = 0; i < APER; ++i) {
            if (ATASKS % GT != 0 && t + i * GT >= ATASKS) break;
            const int d = (t + i * GT) / NP;
            const uint32_t x0 = a_reg[i][0], x1 = a_reg[i][1];
            const uint32_t x0s = x0 >> 2, x1s = x1 >> 2;
            const uint32_t am = (a_valid[i][0] ? 0x00000303u : 0u) | (a_valid[i][1] ? 0x03030000u : 0u);
            const uint32_t om = (a_valid[i][0] ? 0x00000400u : 0x00000C0Cu) |
                                (a_valid[i][1] ? 0x04000000u : 0x0C0C0000u);
            // u0 = bytes [x0.b0, x0s.b0, x0.b1, x0s.b1] (packed bytes 0,1 of n0, plain and shifted by one code)
            const uint32_t u0_01 = perm(x0s, x0, 0x05010400u), u0_23 = perm(x0s, x0, 0x07030602u);
            const uint32_t u1_01 = perm(x1s, x1, 0x05010400u), u1_23 = perm(x1s, x1, 0x07030602u);
            uint32_t v[4];                                  // per packed byte: [n0, n0 shifted, n1, n1 shifted]
            v[0] = perm(u1_01, u0_01, 0x05040100u);
            v[1] = perm(u1_01, u0_01, 0x07060302u);
            v[2] = perm(u1_23, u0_23, 0x05040100u);
            v[3] = perm(u1_23, u0_23, 0x07060302u);
#pragma unroll
            for (int b = 0; b < 4; ++b) {
#pragma unroll
                for (int e = 0; e < 2; ++e) {
                    const uint32_t sel4 = (((e ? v[b] >> 4 : v[b])) & am) | om;      // four products per permute
                    const int q = 8 * d + 2 * b + e;
                    if (MODE == 0) {
                        s_sel[(buf * QS + q) * SROW + a_sidx[i]] = sel4;
                    } else {
                        // two products per permute: [even position of n0, zero, even position of n1, zero], then odd
                        uint2 *dst = (uint2 *)(s_sel + (buf * QS + q) * SROW + a_sidx[i]);
                        *dst = make_uint2((sel4 & 0x00FF00FFu) | 0x0C000C00u, ((sel4 >> 8) & 0x00FF00FFu) | 0x0C000C00u);
                    }
                }
            }
        }
    };

    // ---- accumulators -------------------------------------------------------------------------
    uint32_t acc8[TM][TN / 2];
    int32_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int j = 0; j < TN / 2; ++j) acc8[i][j] = 0;
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = 0;
    }
    auto flush = [&]() {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN / 2; ++j) {
                if (MODE == 0) {
                    acc[i][2 * j] = fold_bytes(acc8[i][j], 0x00000101u, acc[i][2 * j]);
                    acc[i][2 * j + 1] = fold_bytes(acc8[i][j], 0x01010000u, acc[i][2 * j + 1]);
                } else {
                    acc[i][2 * j] += (int32_t)(acc8[i][j] & 0xFFFFu);
                    acc[i][2 * j + 1] += (int32_t)(acc8[i][j] >> 16);
                }
                acc8[i][j] = 0;
            }
    };

    const int stages = (p.K + KS - 1) / KS;
    const int iters = (stages + SK - 1) / SK;       // stages per group (the last may be empty: all selectors 0x0C)
    fetch(0);
    expand(0);
    __syncthreads();

    int pending = 0;            // 16-code groups accumulated in byte lanes since the last fold
    for (int it = 0; it < iters; ++it) {
        const int buf = NBUF == 2 ? (it & 1) : 0;
        if (it + 1 < iters) fetch(it + 1);
#pragma unroll
        for (int d = 0; d < DW; ++d) {
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                uint2 pool[TM];
                uint32_t sel[TN / 2 * SELW];
                const uint2 *pq = s_pool + (buf * QS + 8 * d + q) * BM;
                const uint32_t *sq = s_sel + (buf * QS + 8 * d + q) * SROW;
#pragma unroll
                for (int i = 0; i < TM; ++i) pool[i] = pq[(i >> 1) * 2 * LM + 2 * ml + (i & 1)];
#pragma unroll
                for (int j = 0; j < TN / 2 * SELW; ++j) sel[j] = sq[nl * SPL + j];
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN / 2; ++j) {
                        if (MODE == 0)
                            acc8[i][j] += perm(pool[i].y, pool[i].x, sel[j]);
                        else
                            acc8[i][j] += perm(pool[i].y, pool[i].x, sel[2 * j]) +
                                          perm(pool[i].y, pool[i].x, sel[2 * j + 1]);
                    }
            }
            if (++pending == a.flush_dwords) {
                flush();
                pending = 0;
            }
        }
        if (NBUF == 2) {
            if (it + 1 < iters) expand(buf ^ 1);
            __syncthreads();
        } else if (it + 1 < iters) {
            __syncthreads();            // every lane is done reading the only buffer
            expand(0);
            __syncthreads();
        }
    }
    flush();

    if (SK > 1) {
        // partial sums of the K-split groups meet in LDS; integer adds commute, so the result is exact
#pragma unroll
        for (int c = 0; c < TN; ++c)
#pragma unroll
            for (int i = 0; i < TM; ++i) atomicAdd(&s_red[(c * TM + i) * GT + t], acc[i][c]);
        __syncthreads();
        if (g != 0) return;
#pragma unroll
        for (int c = 0; c < TN; ++c)
#pragma unroll
            for (int i = 0; i < TM; ++i) acc[i][c] = s_red[(c * TM + i) * GT + t];
    }

    // ---- epilogue: remove the bias, optional per-channel scale, store ------------------------------
    // This lane's outputs: rows m_first .. m_first+TM-1, columns n_first .. n_first+TN-1.  The contiguous output
    // axis (channels when MFAST, columns otherwise) is written with 64/128-bit stores when alignment allows.
    if (m_first >= p.M || n_first >= p.N) return;
    const int64_t scm = MFAST ? 1 : p.stride_cm, scn = p.stride_cn;   // MFAST is launched only when stride_cm == 1
    int32_t bias[TN];
    {
        const uint32_t row = fdiv((uint32_t)n_first, a.div_ow);
        int ow = n_first - (int)row * p.OW;
        int oh = (int)(row - fdiv(row, a.div_oh) * (uint32_t)p.OH);
        const int full = a.min_entry * p.K;
#pragma unroll
        for (int c = 0; c < TN; ++c) {
            bias[c] = full;
            if (p.ph | p.pw) {
                // filter taps inside the image: kh in [max(0, ph - oh*sh), min(KH, H + ph - oh*sh))
                const int h0 = p.ph - oh * p.sh, w0 = p.pw - ow * p.sw;
                const int th = min(p.KH, p.H + h0) - max(0, h0), tw = min(p.KW, p.W + w0) - max(0, w0);
                bias[c] = a.min_entry * p.Cin * max(th, 0) * max(tw, 0);
            }
            if (++ow == p.OW) {
                ow = 0;
                if (++oh == p.OH) oh = 0;
            }
        }
    }
    unsigned char *out = (unsigned char *)(p.scale ? (void *)p.Cf : (void *)p.C);   // both element types are 4 bytes
    out += 4 * ((int64_t)m_first * scm + (int64_t)n_first * scn);
    constexpr int VL = MFAST ? TM : TN;                      // elements along the contiguous axis
    constexpr int VEC = VL % 4 == 0 ? 4 : 2;
    const bool whole = MFAST ? (m_first + TM <= p.M) : (n_first + TN <= p.N);
    const int64_t other = MFAST ? scn : scm;                 // stride of the axis the loop below walks
    const int64_t contig = MFAST ? 1 : scn;                  // stride of the axis written within a line
    const bool vec_ok = whole && contig == 1 && ((uintptr_t)out % (4 * VEC) == 0) && (other % VEC == 0);
#pragma unroll
    for (int o = 0; o < (MFAST ? TN : TM); ++o) {            // one line per column (MFAST) or per row
        if (MFAST ? (n_first + o >= p.N) : (m_first + o >= p.M)) break;
        uint32_t bits[VL];
#pragma unroll
        for (int e = 0; e < VL; ++e) {
            const int i = MFAST ? e : o, c = MFAST ? o : e;
            const int32_t v = acc[i][c] + bias[c];
            bits[e] = p.scale ? __float_as_uint((float)v * sc[i]) : (uint32_t)v;
        }
        unsigned char *line = out + 4 * o * other;
        if (vec_ok) {
#pragma unroll
            for (int e = 0; e < VL; e += VEC) {
                if (VEC == 4)
                    *(uint4 *)(line + 4 * e) = make_uint4(bits[e], bits[e + 1], bits[e + 2], bits[e + 3]);
                else
                    *(uint2 *)(line + 4 * e) = make_uint2(bits[e], bits[e + 1]);
            }
        } else {
#pragma unroll
            for (int e = 0; e < VL; ++e)
                if (MFAST ? (m_first + e < p.M) : (n_first + e < p.N)) *(uint32_t *)(line + 4 * e * contig) = bits[e];
        }
    }
}

// Launch one instantiation; defined (explicitly instantiated) in the dg_perm_inst_*.hip files.
template <int TM, int TN, int LM, int LN, int KS, int SK, int NBUF, int MODE, bool MFAST>
dg_status perm_launch(const PermArgs &a, dim3 grid, hipStream_t stream);

#define DG_PERM_DEFINE_LAUNCH                                                                         \
    template <int TM, int TN, int LM, int LN, int KS, int SK, int NBUF, int MODE, bool MFAST>         \
    dg_status perm_launch(const PermArgs &a, dim3 grid, hipStream_t stream)                           \
    {                                                                                                 \
        using S = PermShape<TM, TN, LM, LN, KS, SK, NBUF, MODE>;                                      \
        auto kernel = perm_lut_kernel<TM, TN, LM, LN, KS, SK, NBUF, MODE, MFAST>;                     \
        static bool ready = false; /* raise the dynamic-LDS limit once per instantiation */           \
        if (!ready) {                                                                                 \
            hipError_t e = hipFuncSetAttribute((const void *)kernel,                                  \
                                               hipFuncAttributeMaxDynamicSharedMemorySize,            \
                                               S::LDS_BYTES);                                         \
            if (e != hipSuccess)                                                                      \
                return dg_fail(DG_ERR_HIP, "perm kernel LDS attribute: %s", hipGetErrorString(e));    \
            ready = true;                                                                             \
        }                                                                                             \
        hipLaunchKernelGGL(kernel, grid, dim3(S::NT), S::LDS_BYTES, stream, a);                       \
        return dg_check_launch("perm_lut_kernel");                                                    \
    }
#define DG_PERM_INSTANTIATE(TM, TN, LM, LN, KS, SK, NBUF, MODE)                                                     \
    template dg_status perm_launch<TM, TN, LM, LN, KS, SK, NBUF, MODE, true>(const PermArgs &, dim3, hipStream_t); \
    template dg_status perm_launch<TM, TN, LM, LN, KS, SK, NBUF, MODE, false>(const PermArgs &, dim3, hipStream_t);

}   // namespace dgperm
