// The matrix-core COMPARISON kernel -- not a table kernel.
//
// When the table is the outer product of two level vectors (which is what dg_build_lut builds),
// the sum of fetched table entries equals the integer dot product of the decoded levels, so the
// layer is a dense int8 contraction and can run on the MFMA units.  This kernel decodes the 2-bit
// codes to int8 levels in registers (a 4-entry v_perm_b32 lookup per 4 codes) and issues
// v_mfma_i32_32x32x32_i8.  It exists to be measured against the table kernels on the same layers;
// DG_KERNEL_AUTO never selects it.
//
// Each wave owns a (WM*32) x (WN*32) output tile and runs on its own: packed operands come straight
// from global memory (a lane reads CH consecutive 32-bit words of one weight row / one activation
// pixel, prefetched one chunk ahead), there is no LDS staging and no barrier.  Integer sums do not
// depend on the order of the reduction, so the kernel assigns reduction positions to MFMA operand
// bytes in whatever order makes the loads contiguous; both operands use the same assignment.
#include "dg_mfma_tile.h"

namespace {

typedef dg_v4i v4i;
typedef dg_v16i v16i;

struct MfmaArgs {
    DgProblem p;
    uint32_t lv_w, lv_a;     // the four int8 levels of each side, one per byte, in code order
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

// 16 codes of one packed word -> 16 int8 levels (4 registers).  Register j holds codes j, 4+j, 8+j, 12+j.
// With am = 0 and om = 0x0C0C0C0C every selector is 0x0C and the result is all zero (a tap outside the image).
__device__ __forceinline__ v4i decode(uint32_t word, uint32_t levels, uint32_t am, uint32_t om)
{
    v4i r;
    r[0] = (int)__builtin_amdgcn_perm(0u, levels, (word & am) | om);
    r[1] = (int)__builtin_amdgcn_perm(0u, levels, ((word >> 2) & am) | om);
    r[2] = (int)__builtin_amdgcn_perm(0u, levels, ((word >> 4) & am) | om);
    r[3] = (int)__builtin_amdgcn_perm(0u, levels, ((word >> 6) & am) | om);
    return r;
}

template <int WM, int WN, int CH, bool TR>
__global__ void __launch_bounds__(256)
mfma_i8_kernel(MfmaArgs a)
{
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
        if (m >= p.M) m = p.M - 1;                          // read a valid row; never stored
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
    float sc_cols[WM];                                      // the epilogue's scales, fetched now
    dg_mfma_column_scales<WM, TR>(p, m0, lane, sc_cols);

    // the chunk's filter tap (same for every lane: a chunk never straddles taps since Cin % CHUNK == 0)
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
            vb[bn] = x_ok[bn] & ((uint32_t)ih < (uint32_t)p.H) & ((uint32_t)iw < (uint32_t)p.W);
            // always load (a tap outside the image reads the first pixel instead and is masked later): a load under
            // a branch would make the compiler wait for it at once, and the prefetch would hide nothing
            wb[bn] = load_words<CH>(vb[bn] ? p.Xp + x_off0[bn] + tap_off : p.Xp + h * (4 * CH), true);
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
        uint32_t am[WN], om[WN];
#pragma unroll
        for (int bm = 0; bm < WM; ++bm) ca[bm] = wa[bm];
#pragma unroll
        for (int bn = 0; bn < WN; ++bn) {
            cb[bn] = wb[bn];
            am[bn] = vb[bn] ? 0x03030303u : 0u;
            om[bn] = vb[bn] ? 0u : 0x0C0C0C0Cu;
        }
        fetch(c + 1 < chunks ? c + 1 : c);                  // unconditional (the last one re-reads in bounds and is unused)
#pragma unroll
        for (int s = 0; s < CH; ++s) {
            v4i fa[WM], fb[WN];
#pragma unroll
            for (int bm = 0; bm < WM; ++bm) fa[bm] = decode(ca[bm].v[s], a.lv_w, 0x03030303u, 0u);
#pragma unroll
            for (int bn = 0; bn < WN; ++bn) fb[bn] = decode(cb[bn].v[s], a.lv_a, am[bn], om[bn]);
#pragma unroll
            for (int bm = 0; bm < WM; ++bm)
#pragma unroll
                for (int bn = 0; bn < WN; ++bn)
                    acc[bm][bn] = dg_mfma_step<TR>(fa[bm], fb[bn], acc[bm][bn]);
        }
    }

    dg_mfma_store_tile<WM, WN, TR>(p, acc, m0, n0, lane, sc_cols);
}

template <int WM, int WN, bool TR>
void launch_ch(const MfmaArgs &a, int ch, dim3 grid, hipStream_t stream)
{
    if (ch == 4)
        hipLaunchKernelGGL((mfma_i8_kernel<WM, WN, 4, TR>), grid, dim3(256), 0, stream, a);
    else if (ch == 2)
        hipLaunchKernelGGL((mfma_i8_kernel<WM, WN, 2, TR>), grid, dim3(256), 0, stream, a);
    else
        hipLaunchKernelGGL((mfma_i8_kernel<WM, WN, 1, TR>), grid, dim3(256), 0, stream, a);
}

template <bool TR>
void launch_tile(const MfmaArgs &a, int wm, int wn, int ch, dim3 grid, hipStream_t stream)
{
    if (wm == 4)
        launch_ch<4, 4, TR>(a, ch, grid, stream);
    else if (wn == 4)
        launch_ch<2, 4, TR>(a, ch, grid, stream);
    else
        launch_ch<2, 1, TR>(a, ch, grid, stream);
}

}   // namespace

bool dg_mfma_supports(const dg_lut *, const DgProblem &p)
{
    if (p.Cin % 32 != 0) return false;                     // a lane half reads whole 32-bit words of one tap
    const int ch = p.Cin % 128 == 0 ? 4 : (p.Cin % 64 == 0 ? 2 : 1);
    if ((uintptr_t)p.Wp % (4 * ch) != 0 || (uintptr_t)p.Xp % (4 * ch) != 0) return false;
    return true;
}

dg_status dg_launch_mfma(const dg_lut *lut, const DgProblem &p, hipStream_t stream)
{
    MfmaArgs a;
    a.p = p;
    a.lv_w = a.lv_a = 0;
    for (int c = 0; c < 4; ++c) {
        a.lv_w |= (uint32_t)(uint8_t)lut->levels_w[c] << (8 * c);
        a.lv_a |= (uint32_t)(uint8_t)lut->levels_a[c] << (8 * c);
    }
    const int ch = p.Cin % 128 == 0 ? 4 : (p.Cin % 64 == 0 ? 2 : 1);
    auto tiles = [&](int wm, int wn) {
        return ((int64_t)(p.M + wm * 32 - 1) / (wm * 32)) * (((int64_t)p.N + wn * 32 - 1) / (wn * 32));
    };
    // wave tiles: 128 x 128 when they still give every SIMD two rounds, else 64 x 128, else 64 x 32
    int wm = 2, wn = 1;
    if (p.M >= 128 && tiles(4, 4) >= 2048) wm = 4, wn = 4;
    else if (tiles(2, 4) >= 1024) wm = 2, wn = 4;
    a.tiles_m = (p.M + wm * 32 - 1) / (wm * 32);
    a.wave_tiles = tiles(wm, wn);
    const int64_t blocks = (a.wave_tiles + 3) / 4;
    if (blocks > INT32_MAX) return dg_fail(DG_ERR_UNSUPPORTED, "mfma kernel: too many tiles for one grid");
    const dim3 grid((unsigned)blocks);
    // the output axis with stride 1 goes on the MFMA columns (see dg_mfma_tile.h)
    if (p.stride_cm == 1 && p.stride_cn != 1)
        launch_tile<true>(a, wm, wn, ch, grid, stream);
    else
        launch_tile<false>(a, wm, wn, ch, grid, stream);
    return dg_check_launch("mfma_i8_kernel");
}
