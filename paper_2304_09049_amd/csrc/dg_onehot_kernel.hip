// Table lookup on the matrix cores by one-hot selection -- a TABLE kernel (it works for any 16 int8 entries,
// whether or not they factor into level vectors), unlike the decode-and-multiply comparison kernel.
//
//   C[m][n] = sum_k T[w(m,k)][a(n,k)] = sum_k sum_{v<4} T[w(m,k)][v] * [a(n,k) == v]
//
// so with A'[m][4k+v] = T[w(m,k)][v] (the table ROW of the weight code, 4 int8) and B'[n][4k+v] = [a(n,k) == v]
// (a one-hot byte quadruple) the layer is an int8 contraction of length 4K: each multiply is by 0 or 1, i.e. the
// MFMA unit SELECTS one table entry per reduction position and adds it.  Four times the MFMA work of the
// rank-1 decode kernel, but every table is accepted and the VALU only expands codes.
//
// Expansion: a packed byte holds two nibbles = two code pairs; an LDS table maps a weight nibble to its two rows
// (8 bytes) and an activation nibble to its two one-hot quadruples (8 bytes), so a lane builds a 16-byte MFMA
// operand (4 reduction positions) from one packed byte with two 64-bit LDS reads.  A second, all-zero table
// stands in for filter taps outside the image.  Wave tiles, global loads and the epilogue follow the
// comparison kernel: each wave owns (WM*32) x (WN*32) outputs, no barrier after the tables are written.
#include "dg_common.h"

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

struct OneHotArgs {
    DgProblem p;
    uint32_t rows[4];        // rows[w] = bytes T[w][0..3] (signed int8, as stored)
    int32_t tiles_m;
    int64_t wave_tiles;
};

template <int CH>
struct Words {
    uint32_t v[CH];
};

template <int CH>
__device__ __forceinline__ Words<CH> load_words(const uint8_t *ptr, bool ok)
{
    Words<CH> w;
    if (CH == 4) {
        const uint4 t = ok ? *(const uint4 *)ptr : make_uint4(0, 0, 0, 0);
        w.v[0] = t.x, w.v[1 % CH] = t.y, w.v[2 % CH] = t.z, w.v[3 % CH] = t.w;
    } else if (CH == 2) {
        const uint2 t = ok ? *(const uint2 *)ptr : make_uint2(0, 0);
        w.v[0] = t.x, w.v[1 % CH] = t.y;
    } else {
        w.v[0] = ok ? *(const uint32_t *)ptr : 0u;
    }
    return w;
}

// one packed byte (4 codes) -> 16 operand bytes: two table reads of 8 bytes each
__device__ __forceinline__ v4i expand_byte(const uint2 *table, uint32_t byte)
{
    const uint2 lo = table[byte & 15u], hi = table[byte >> 4];
    v4i r;
    r[0] = (int)lo.x, r[1] = (int)lo.y, r[2] = (int)hi.x, r[3] = (int)hi.y;
    return r;
}

template <int WM, int WN, int CH>
__global__ void __launch_bounds__(256)
onehot_mfma_kernel(OneHotArgs a)
{
    // [0..15] weight nibble -> {row[w even], row[w odd]}; [16..31] activation nibble -> one-hot quadruples;
    // [32..47] zeros (a tap outside the image selects nothing)
    __shared__ uint2 s_table[48];
    if (threadIdx.x < 16) {
        const int t = threadIdx.x;
        s_table[t] = make_uint2(a.rows[t & 3], a.rows[t >> 2]);
        s_table[16 + t] = make_uint2(1u << (8 * (t & 3)), 1u << (8 * (t >> 2)));
        s_table[32 + t] = make_uint2(0u, 0u);
    }
    __syncthreads();

    const DgProblem &p = a.p;
    const int lane = threadIdx.x & 63;
    const int64_t wave_tile = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (wave_tile >= a.wave_tiles) return;                 // whole waves leave; there is no barrier below
    const int r = lane & 31, h = lane >> 5;
    const int m0 = (int)(wave_tile % a.tiles_m) * (WM * 32);
    const int n0 = (int)(wave_tile / a.tiles_m) * (WN * 32);
    const int cq = p.Cin / 4;
    constexpr int CHUNK = 32 * CH;                          // codes of K per chunk (16*CH per lane half)

    const uint8_t *w_ptr[WM];
#pragma unroll
    for (int bm = 0; bm < WM; ++bm) {
        int m = m0 + bm * 32 + r;
        if (m >= p.M) m = p.M - 1;
        w_ptr[bm] = p.Wp + (int64_t)m * (p.K / 4) + h * (4 * CH);
    }
    bool x_ok[WN];
    int x_ih0[WN], x_iw0[WN];
    int64_t x_off0[WN];
#pragma unroll
    for (int bn = 0; bn < WN; ++bn) {
        const int n = n0 + bn * 32 + r;
        x_ok[bn] = n < p.N;
        const int nn = x_ok[bn] ? n : 0;
        const int ow = nn % p.OW, oh = (nn / p.OW) % p.OH, b = nn / (p.OW * p.OH);
        x_ih0[bn] = oh * p.sh - p.ph;
        x_iw0[bn] = ow * p.sw - p.pw;
        x_off0[bn] = (((int64_t)b * p.H + x_ih0[bn]) * p.W + x_iw0[bn]) * cq + h * (4 * CH);
    }

    v16i acc[WM][WN];
#pragma unroll
    for (int bm = 0; bm < WM; ++bm)
#pragma unroll
        for (int bn = 0; bn < WN; ++bn)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[bm][bn][e] = 0;

    int kh = 0, kw = 0, ci = 0;
    Words<CH> wa[WM], wb[WN];
    bool vb[WN];
    auto fetch = [&](int chunk) {
#pragma unroll
        for (int bm = 0; bm < WM; ++bm) wa[bm] = load_words<CH>(w_ptr[bm] + (int64_t)chunk * (CHUNK / 4), true);
        const int64_t tap_off = ((int64_t)kh * p.W + kw) * cq + ci / 4;
#pragma unroll
        for (int bn = 0; bn < WN; ++bn) {
            const int ih = x_ih0[bn] + kh, iw = x_iw0[bn] + kw;
            vb[bn] = x_ok[bn] && ih >= 0 && ih < p.H && iw >= 0 && iw < p.W;
            wb[bn] = load_words<CH>(p.Xp + x_off0[bn] + tap_off, vb[bn]);
        }
        ci += CHUNK;
        if (ci == p.Cin) {
            ci = 0;
            if (++kw == p.KW) {
                kw = 0;
                ++kh;
            }
        }
    };

    const int chunks = p.K / CHUNK;
    fetch(0);
    for (int c = 0; c < chunks; ++c) {
        Words<CH> ca[WM], cb[WN];
        const uint2 *tb[WN];
#pragma unroll
        for (int bm = 0; bm < WM; ++bm) ca[bm] = wa[bm];
#pragma unroll
        for (int bn = 0; bn < WN; ++bn) {
            cb[bn] = wb[bn];
            tb[bn] = s_table + (vb[bn] ? 16 : 32);
        }
        if (c + 1 < chunks) fetch(c + 1);
#pragma unroll
        for (int s = 0; s < CH; ++s) {
#pragma unroll
            for (int b = 0; b < 4; ++b) {                    // one packed byte = 4 reduction positions = one MFMA step
                v4i fa[WM], fb[WN];
#pragma unroll
                for (int bm = 0; bm < WM; ++bm) fa[bm] = expand_byte(s_table, (ca[bm].v[s] >> (8 * b)) & 0xFFu);
#pragma unroll
                for (int bn = 0; bn < WN; ++bn) fb[bn] = expand_byte(tb[bn], (cb[bn].v[s] >> (8 * b)) & 0xFFu);
#pragma unroll
                for (int bm = 0; bm < WM; ++bm)
#pragma unroll
                    for (int bn = 0; bn < WN; ++bn)
                        acc[bm][bn] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[bm], fb[bn], acc[bm][bn], 0, 0, 0);
            }
        }
    }

#pragma unroll
    for (int bn = 0; bn < WN; ++bn) {
        const int n = n0 + bn * 32 + r;
        if (n >= p.N) continue;
#pragma unroll
        for (int bm = 0; bm < WM; ++bm)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int m = m0 + bm * 32 + 8 * (e / 4) + 4 * h + (e % 4);
                if (m >= p.M) continue;
                const int64_t o = (int64_t)m * p.stride_cm + (int64_t)n * p.stride_cn;
                if (p.scale)
                    p.Cf[o] = (float)acc[bm][bn][e] * p.scale[m];
                else
                    p.C[o] = acc[bm][bn][e];
            }
    }
}

template <int WM, int WN>
void launch_ch(const OneHotArgs &a, int ch, dim3 grid, hipStream_t stream)
{
    if (ch == 4)
        hipLaunchKernelGGL((onehot_mfma_kernel<WM, WN, 4>), grid, dim3(256), 0, stream, a);
    else if (ch == 2)
        hipLaunchKernelGGL((onehot_mfma_kernel<WM, WN, 2>), grid, dim3(256), 0, stream, a);
    else
        hipLaunchKernelGGL((onehot_mfma_kernel<WM, WN, 1>), grid, dim3(256), 0, stream, a);
}

}   // namespace

bool dg_onehot_supports(const dg_lut *lut, const DgProblem &p)
{
    if (lut->min_entry < -128 || lut->max_entry > 127) return false;   // entries are MFMA int8 operands
    if (p.Cin % 32 != 0) return false;
    const int ch = p.Cin % 128 == 0 ? 4 : (p.Cin % 64 == 0 ? 2 : 1);
    if ((uintptr_t)p.Wp % (4 * ch) != 0 || (uintptr_t)p.Xp % (4 * ch) != 0) return false;
    return true;
}

dg_status dg_launch_onehot(const dg_lut *lut, const DgProblem &p, hipStream_t stream)
{
    OneHotArgs a;
    a.p = p;
    for (int w = 0; w < 4; ++w) {
        uint32_t r = 0;
        for (int c = 0; c < 4; ++c) r |= (uint32_t)(uint8_t)(int8_t)lut->entry[4 * w + c] << (8 * c);
        a.rows[w] = r;
    }
    const int ch = p.Cin % 128 == 0 ? 4 : (p.Cin % 64 == 0 ? 2 : 1);
    auto tiles = [&](int wm, int wn) {
        return ((int64_t)(p.M + wm * 32 - 1) / (wm * 32)) * (((int64_t)p.N + wn * 32 - 1) / (wn * 32));
    };
    int wm = 2, wn = 1;
    if (tiles(2, 4) >= 1024) wm = 2, wn = 4;
    else if (tiles(2, 2) >= 512) wm = 2, wn = 2;
    a.tiles_m = (p.M + wm * 32 - 1) / (wm * 32);
    a.wave_tiles = tiles(wm, wn);
    const int64_t blocks = (a.wave_tiles + 3) / 4;
    if (blocks > INT32_MAX) return dg_fail(DG_ERR_UNSUPPORTED, "one-hot kernel: too many tiles for one grid");
    const dim3 grid((unsigned)blocks);
    if (wn == 4)
        launch_ch<2, 4>(a, ch, grid, stream);
    else if (wn == 2)
        launch_ch<2, 2>(a, ch, grid, stream);
    else
        launch_ch<2, 1>(a, ch, grid, stream);
    return dg_check_launch("onehot_mfma_kernel");
}
