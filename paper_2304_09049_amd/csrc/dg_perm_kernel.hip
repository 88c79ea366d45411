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
// Implicit im2col (NHWC): reduction index k = (kh*KW + kw)*Cin + ci.  The loader computes the source
// pixel of every (output pixel, filter tap) and, for taps outside the image (and rows beyond N,
// positions beyond K), writes the selector 0x0C, for which v_perm_b32 returns the constant 0:
// such positions add nothing, whatever the table holds.
#include "dg_common.h"

namespace {

struct PermArgs {
    DgProblem p;
    uint32_t rows[4];       // biased table rows: byte a of rows[w] = LUT[4w+a] - min_entry
    int32_t min_entry;
    int32_t flush_dwords;   // fold byte lanes into int32 after this many 16-code groups (8 permutes each)
    int32_t tiles_m;
};

__device__ __forceinline__ uint32_t perm(uint32_t hi, uint32_t lo, uint32_t sel)
{
    return __builtin_amdgcn_perm(hi, lo, sel);
}

// sum of the masked byte lanes of `v`, added to acc
__device__ __forceinline__ int32_t fold_bytes(uint32_t v, uint32_t ones, int32_t acc)
{
    return (int32_t)__builtin_amdgcn_udot4(v, ones, (uint32_t)acc, false);
}

// TM x TN outputs per lane; LM x LN lanes per workgroup; KS codes of K per LDS stage.
template <int TM, int TN, int LM, int LN, int KS, bool MFAST>
__global__ void __launch_bounds__(LM *LN)
perm_lut_kernel(PermArgs a)
{
    constexpr int NT = LM * LN;
    constexpr int BM = LM * TM, BN = LN * TN, NP = BN / 2;
    constexpr int QS = KS / 2;     // pools (pairs of reduction positions) per stage
    constexpr int DW = KS / 16;    // 32-bit packed words per row per stage
    static_assert(TN % 2 == 0 && KS % 16 == 0, "tile shape");

    __shared__ uint2 s_pool[2][QS][BM];       // {row[w(k)], row[w(k+1)]} per (pair q, weight row)
    __shared__ uint32_t s_sel[2][QS][NP];     // selector per (pair q, column pair)
    __shared__ uint2 s_table[16];             // pool for every value of a weight nibble

    const DgProblem &p = a.p;
    const int tid = threadIdx.x;
    const int ml = MFAST ? tid % LM : tid / LN;
    const int nl = MFAST ? tid / LM : tid % LN;
    const int tile_m = blockIdx.x % a.tiles_m;
    const int tile_n = blockIdx.x / a.tiles_m;
    const int m_base = tile_m * BM;
    const int n_base = tile_n * BN;

    if (tid < 16) s_table[tid] = make_uint2(a.rows[tid & 3], a.rows[tid >> 2]);

    // ---- loader tasks (fixed per lane for the whole K loop) ---------------------------------
    // weight side: (row, word) -> 8 pools
    constexpr int WTASKS = BM * DW, WPER = (WTASKS + NT - 1) / NT;
    // activation side: (column pair, word) -> 8 selectors
    constexpr int ATASKS = NP * DW, APER = (ATASKS + NT - 1) / NT;

    const uint32_t *w_ptr[WPER];
    int w_row[WPER], w_d[WPER];
#pragma unroll
    for (int t = 0; t < WPER; ++t) {
        const int task = tid + t * NT;
        w_row[t] = task % BM;
        w_d[t] = task / BM;
        int m = m_base + w_row[t];
        if (m >= p.M) m = p.M - 1;                       // rows beyond M: read a valid row, never stored
        w_ptr[t] = (const uint32_t *)(p.Wp + (int64_t)m * (p.K / 4)) + w_d[t];
    }
    int a_np[APER], a_d[APER];
    int a_ih0[APER][2], a_iw0[APER][2];                   // top-left source pixel of the filter window
    int64_t a_img[APER][2];                               // pixel index of the image's (0,0)
    bool a_ok[APER][2];
#pragma unroll
    for (int t = 0; t < APER; ++t) {
        const int task = tid + t * NT;
        a_np[t] = task % NP;
        a_d[t] = task / NP;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int n = n_base + 2 * a_np[t] + h;
            a_ok[t][h] = (task < ATASKS) && (n < p.N);
            const int nn = a_ok[t][h] ? n : 0;
            const int ow = nn % p.OW, oh = (nn / p.OW) % p.OH, b = nn / (p.OW * p.OH);
            a_ih0[t][h] = oh * p.sh - p.ph;
            a_iw0[t][h] = ow * p.sw - p.pw;
            a_img[t][h] = (int64_t)b * p.H * p.W;
        }
    }

    uint32_t w_reg[WPER];
    uint32_t a_reg[APER][2];
    bool a_valid[APER][2];

    auto fetch = [&](int stage) {
        const int k_stage = stage * KS;
#pragma unroll
        for (int t = 0; t < WPER; ++t) {
            const int k0 = k_stage + 16 * w_d[t];
            const bool ok = (WTASKS % NT == 0 || tid + t * NT < WTASKS) && k0 < p.K;
            w_reg[t] = ok ? w_ptr[t][k_stage / 16] : 0u;
        }
#pragma unroll
        for (int t = 0; t < APER; ++t) {
            const int k0 = k_stage + 16 * a_d[t];
            const int tap = k0 / p.Cin, ci = k0 - tap * p.Cin;
            const int kh = tap / p.KW, kw = tap - kh * p.KW;
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int ih = a_ih0[t][h] + kh, iw = a_iw0[t][h] + kw;
                const bool ok = a_ok[t][h] && k0 < p.K && ih >= 0 && ih < p.H && iw >= 0 && iw < p.W;
                a_valid[t][h] = ok;
                const int64_t pix = a_img[t][h] + (int64_t)ih * p.W + iw;
                a_reg[t][h] = ok ? *((const uint32_t *)(p.Xp + pix * (p.Cin / 4)) + ci / 16) : 0u;
            }
        }
    };

    auto expand = [&](int buf) {
        // weights: nibble q of the word = codes (2q, 2q+1) -> the pool stored for that nibble value
#pragma unroll
        for (int t = 0; t < WPER; ++t) {
            if (WTASKS % NT != 0 && tid + t * NT >= WTASKS) break;
            const uint32_t w = w_reg[t];
#pragma unroll
            for (int q = 0; q < 8; ++q)
                s_pool[buf][8 * w_d[t] + q][w_row[t]] = s_table[(w >> (4 * q)) & 15u];
        }
        // activations: selector bytes [a(n0,2q), 4 + a(n0,2q+1), a(n1,2q), 4 + a(n1,2q+1)]
#pragma unroll
        for (int t = 0; t < APER; ++t) {
            if (ATASKS % NT != 0 && tid + t * NT >= ATASKS) break;
            const uint32_t x0 = a_reg[t][0], x1 = a_reg[t][1];
            const uint32_t x0s = x0 >> 2, x1s = x1 >> 2;
            const uint32_t am = (a_valid[t][0] ? 0x00000303u : 0u) | (a_valid[t][1] ? 0x03030000u : 0u);
            const uint32_t om = (a_valid[t][0] ? 0x00000400u : 0x00000C0Cu) |
                                (a_valid[t][1] ? 0x04000000u : 0x0C0C0000u);
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
                s_sel[buf][8 * a_d[t] + 2 * b][a_np[t]] = (v[b] & am) | om;
                s_sel[buf][8 * a_d[t] + 2 * b + 1][a_np[t]] = ((v[b] >> 4) & am) | om;
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
                acc[i][2 * j] = fold_bytes(acc8[i][j], 0x00000101u, acc[i][2 * j]);
                acc[i][2 * j + 1] = fold_bytes(acc8[i][j], 0x01010000u, acc[i][2 * j + 1]);
                acc8[i][j] = 0;
            }
    };

    const int stages = (p.K + KS - 1) / KS;
    fetch(0);
    __syncthreads();            // s_table is ready
    expand(0);
    __syncthreads();

    int pending = 0;            // 16-code groups accumulated in byte lanes since the last fold
    for (int s = 0; s < stages; ++s) {
        const int buf = s & 1;
        if (s + 1 < stages) fetch(s + 1);
#pragma unroll
        for (int d = 0; d < DW; ++d) {
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                uint2 pool[TM];
                uint32_t sel[TN / 2];
#pragma unroll
                for (int i = 0; i < TM; ++i) pool[i] = s_pool[buf][8 * d + q][ml * TM + i];
#pragma unroll
                for (int j = 0; j < TN / 2; ++j) sel[j] = s_sel[buf][8 * d + q][nl * (TN / 2) + j];
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN / 2; ++j) acc8[i][j] += perm(pool[i].y, pool[i].x, sel[j]);
            }
            if (++pending == a.flush_dwords) {
                flush();
                pending = 0;
            }
        }
        if (s + 1 < stages) expand(buf ^ 1);
        __syncthreads();
    }
    flush();

    // ---- epilogue: remove the bias, optional per-channel scale, store ------------------------------
#pragma unroll
    for (int c = 0; c < TN; ++c) {
        const int n = n_base + nl * TN + c;
        if (n >= p.N) continue;
        int taps = p.KH * p.KW;
        if (p.ph | p.pw) {                                 // count the filter taps inside the image
            const int ow = n % p.OW, oh = (n / p.OW) % p.OH;
            int th = 0, tw = 0;
            for (int kh = 0; kh < p.KH; ++kh) {
                const int ih = oh * p.sh - p.ph + kh;
                th += (ih >= 0 && ih < p.H);
            }
            for (int kw = 0; kw < p.KW; ++kw) {
                const int iw = ow * p.sw - p.pw + kw;
                tw += (iw >= 0 && iw < p.W);
            }
            taps = th * tw;
        }
        const int32_t bias = a.min_entry * taps * p.Cin;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int m = m_base + ml * TM + i;
            if (m >= p.M) continue;
            const int32_t v = acc[i][c] + bias;
            const int64_t o = (int64_t)m * p.stride_cm + (int64_t)n * p.stride_cn;
            if (p.scale)
                p.Cf[o] = (float)v * p.scale[m];
            else
                p.C[o] = v;
        }
    }
}

struct PermPlan {
    int BM, BN;
    const char *name;
    void (*launch)(const PermArgs &, dim3, hipStream_t);
};

template <int TM, int TN, int LM, int LN, int KS, bool MFAST>
void launch_cfg(const PermArgs &a, dim3 grid, hipStream_t stream)
{
    hipLaunchKernelGGL((perm_lut_kernel<TM, TN, LM, LN, KS, MFAST>), grid, dim3(LM * LN), 0, stream, a);
}

PermPlan plan_for(const DgProblem &p)
{
    const bool mfast = (p.stride_cm == 1);
    if (p.M > 64) {
        if (mfast) return {128, 128, "perm_8x8_128x128", launch_cfg<8, 8, 16, 16, 32, true>};
        return {128, 128, "perm_8x8_128x128", launch_cfg<8, 8, 16, 16, 32, false>};
    }
    if (mfast) return {64, 128, "perm_4x8_64x128", launch_cfg<4, 8, 16, 16, 32, true>};
    return {64, 128, "perm_4x8_64x128", launch_cfg<4, 8, 16, 16, 32, false>};
}

}   // namespace

bool dg_perm_supports(const dg_lut *lut, const DgProblem &p)
{
    if (lut->max_entry - lut->min_entry > 31) return false;      // byte lanes need >= 8 carry-free adds
    if (p.Cin % 16 != 0) return false;                           // a 32-bit packed word never straddles taps
    if ((uintptr_t)p.Wp % 4 != 0 || (uintptr_t)p.Xp % 4 != 0) return false;
    return true;
}

const char *dg_perm_config_name(const dg_lut *, const DgProblem &p) { return plan_for(p).name; }

dg_status dg_launch_perm(const dg_lut *lut, const DgProblem &p, hipStream_t stream)
{
    PermArgs a;
    a.p = p;
    a.min_entry = lut->min_entry;
    const int range = lut->max_entry - lut->min_entry;
    for (int w = 0; w < 4; ++w) {
        uint32_t r = 0;
        for (int c = 0; c < 4; ++c) r |= (uint32_t)(lut->entry[4 * w + c] - lut->min_entry) << (8 * c);
        a.rows[w] = r;
    }
    // one 16-code group adds 8 entries to each byte lane; lanes hold at most 255
    const int adds = range > 0 ? 255 / range : 1 << 20;
    int fd = adds / 8;
    if (fd > 64) fd = 64;
    a.flush_dwords = fd;
    const PermPlan plan = plan_for(p);
    a.tiles_m = (p.M + plan.BM - 1) / plan.BM;
    const int64_t tiles_n = ((int64_t)p.N + plan.BN - 1) / plan.BN;
    const int64_t blocks = tiles_n * a.tiles_m;
    if (blocks > INT32_MAX) return dg_fail(DG_ERR_UNSUPPORTED, "perm kernel: too many tiles for one grid");
    plan.launch(a, dim3((unsigned)blocks), stream);
    return dg_check_launch("perm_lut_kernel");
}
