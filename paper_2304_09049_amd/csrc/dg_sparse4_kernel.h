// 4-bit codes (the 256-entry table of Sec. 3.3 / Table 2) selected by the sparse matrix instruction.
//
// A one-hot run of 16 bytes is four groups of four with a single 1 among them, and v_smfmac_i32_32x32x64_i8 takes its
// row operand as two kept bytes out of every four plus their 2-bit positions (see dg_onehot_kernel.h for the layout).
// For activation code c the kept bytes of group g are (c / 4 == g, 0) and the position of the first is c % 4 in every
// group: the values are `1 << 16 * (c / 4)` as a 64-bit shift, the index fields (c % 4) * 0x1111.  The instruction then
// picks byte c out of the 16 bytes T[w][0..15] that the dense operand holds for the position -- the weight code's table
// row, one conflict-free 16-byte LDS read.  One instruction covers 4 positions per lane pair (the dense MFMA of the
// one-hot kernel: 2), and the weight operand costs 2 VALU instructions per position instead of 14.
//
// Positions of instruction s (0..3) of a chunk's word t: lane half h of the activation block holds the word's codes 2s and
// 2s+1 (index register and kept bytes); the weight lane (column, half P) supplies, as operand bytes 16h'..16h'+15, the
// row of code 2s+P of the weight word at lane half h''s positions, h' = 0, 1.
#pragma once

#include "dg_onehot_kernel.h"

namespace dgoh {

struct Sparse4Args {
    DgProblem p;
    uint32_t rows[16][4];        // rows[w] = bytes T[w][0..15]
    FastDiv div_ow, div_oh;
    int32_t tiles_m;
    int64_t wave_tiles;
};

// CH = 32-bit words (8 codes) per lane half and chunk.  A wavefront owns a 64 x 128 tile; no LDS besides its own copy
// of the row table, no barrier.
template <int CH>
__global__ void __launch_bounds__(256, 2)
sparse4_kernel(Sparse4Args a)
{
    constexpr int WM = 2, WN = 4;
    __shared__ uint4 s_rows[4 * 16];
    const DgProblem &p = a.p;
    const int lane = threadIdx.x & 63, w4 = threadIdx.x >> 6;
    const int64_t wave_tile = (int64_t)xcd_contiguous(blockIdx.x, gridDim.x) * 4 + w4;
    if (wave_tile >= a.wave_tiles) return;                  // whole waves leave; there is no barrier
    uint4 *rows = s_rows + 16 * w4;
    if (lane < 16) rows[lane] = make_uint4(a.rows[lane][0], a.rows[lane][1], a.rows[lane][2], a.rows[lane][3]);
    __builtin_amdgcn_wave_barrier();                        // (LDS operations of one wavefront execute in order)

    const int r = lane & 31, h = lane >> 5;
    const int m0 = (int)(wave_tile % a.tiles_m) * 64;
    const int n0 = (int)(wave_tile / a.tiles_m) * 128;
    const int cq = p.Cin / 2;                               // packed bytes per pixel
    constexpr int CHUNK = 16 * CH;                          // codes of K per chunk
    const int chunks = p.K / CHUNK;

    const uint8_t *w_ptr[WM];
#pragma unroll
    for (int bm = 0; bm < WM; ++bm) w_ptr[bm] = p.Wp + (int64_t)min(m0 + bm * 32 + r, p.M - 1) * (p.K / 2);
    Column col[WN];
#pragma unroll
    for (int bn = 0; bn < WN; ++bn) col[bn] = make_column(p, a.div_ow, a.div_oh, n0 + bn * 32 + r, cq, h * (4 * CH));
    v16i acc[WM][WN];
#pragma unroll
    for (int bm = 0; bm < WM; ++bm)
#pragma unroll
        for (int bn = 0; bn < WN; ++bn)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[bm][bn][e] = 0;
    float sc_cols[WM];
    dg_mfma_column_scales<WM, true>(p, m0, lane, sc_cols);

    int kh = 0, kw = 0, ci = 0;
    Words<CH> wa[WM][2], wb[WN];
    bool vb[WN];
    auto fetch = [&](int chunk) {                            // `chunk` is clamped: a fetch past the end is unused
        const int cw = min(chunk, chunks - 1);
#pragma unroll
        for (int bm = 0; bm < WM; ++bm)
#pragma unroll
            for (int run = 0; run < 2; ++run) wa[bm][run] = load_words<CH>(w_ptr[bm] + (int64_t)cw * (8 * CH) + run * (4 * CH));
        const int64_t tap_off = ((int64_t)kh * p.W + kw) * cq + ci / 2;
#pragma unroll
        for (int bn = 0; bn < WN; ++bn) {
            const int ih = col[bn].ih0 + kh, iw = col[bn].iw0 + kw;
            vb[bn] = col[bn].ok & ((uint32_t)ih < (uint32_t)p.H) & ((uint32_t)iw < (uint32_t)p.W);
            // always load (a tap outside the image reads the first pixel instead and its kept bytes are zero)
            wb[bn] = load_words<CH>(vb[bn] ? p.Xp + col[bn].off0 + tap_off : p.Xp + h * (4 * CH));
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

    fetch(0);
    for (int c = 0; c < chunks; ++c) {
        Words<CH> ca[WM][2], cb[WN];
        uint64_t one[WN];
#pragma unroll
        for (int bm = 0; bm < WM; ++bm) ca[bm][0] = wa[bm][0], ca[bm][1] = wa[bm][1];
#pragma unroll
        for (int bn = 0; bn < WN; ++bn) {
            cb[bn] = wb[bn];
            one[bn] = vb[bn] ? 1u : 0u;
        }
        fetch(c + 1);                                        // unconditional (the last one re-reads in bounds and is unused)
#pragma unroll
        for (int t = 0; t < CH; ++t)
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                v8i dn[WM];
#pragma unroll
                for (int bm = 0; bm < WM; ++bm) {
                    const uint4 r0 = rows[(ca[bm][0].v[t] >> (8 * s + 4 * h)) & 15u], r1 = rows[(ca[bm][1].v[t] >> (8 * s + 4 * h)) & 15u];
                    dn[bm] = (v8i){(int)r0.x, (int)r0.y, (int)r0.z, (int)r0.w, (int)r1.x, (int)r1.y, (int)r1.z, (int)r1.w};
                }
#pragma unroll
                for (int bn = 0; bn < WN; ++bn) {
                    const uint32_t pair = cb[bn].v[t] >> (8 * s);                   // codes 2s (low nibble) and 2s+1
                    const uint64_t k0 = one[bn] << ((pair & 0xCu) << 2), k1 = one[bn] << ((pair & 0xC0u) >> 2);
                    const v4i kept = {(int)(uint32_t)k0, (int)(uint32_t)(k0 >> 32), (int)(uint32_t)k1, (int)(uint32_t)(k1 >> 32)};
                    const int idx = (int)(((pair & 3u) | ((pair & 0x30u) << 12)) * 0x1111u);
#pragma unroll
                    for (int bm = 0; bm < WM; ++bm)
                        acc[bm][bn] = __builtin_amdgcn_smfmac_i32_32x32x64_i8(kept, dn[bm], acc[bm][bn], idx, 0, 0);
                }
            }
    }
    dg_mfma_store_tile<WM, WN, true>(p, acc, m0, n0, lane, sc_cols);
}

inline void launch_sparse4(const DgProblem &p, const uint32_t (&rows)[16][4], int ch, hipStream_t stream)
{
    Sparse4Args a;
    a.p = p;
    for (int w = 0; w < 16; ++w)
        for (int i = 0; i < 4; ++i) a.rows[w][i] = rows[w][i];
    a.tiles_m = (p.M + 63) / 64;
    a.wave_tiles = (int64_t)a.tiles_m * (((int64_t)p.N + 127) / 128);
    a.div_ow = make_div((uint32_t)p.OW), a.div_oh = make_div((uint32_t)p.OH);
    const dim3 grid((unsigned)((a.wave_tiles + 3) / 4));
    if (ch == 2)
        hipLaunchKernelGGL((sparse4_kernel<2>), grid, dim3(256), 0, stream, a);
    else
        hipLaunchKernelGGL((sparse4_kernel<1>), grid, dim3(256), 0, stream, a);
}

}   // namespace dgoh
