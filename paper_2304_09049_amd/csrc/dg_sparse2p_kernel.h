// 2-bit codes with table entries beyond int8, selected by the sparse matrix instruction from two int8 planes.
//
// T = 256 * hi + lo with lo = ((T + 128) mod 256) - 128 (as in the dense-instruction kernel's two-plane form): the two
// planes are two dense operands for the same 32 weight rows, built from the same table indices (the row-pair table of
// the high plane sits 128 bytes behind that of the low plane in LDS), each selected into sums of its own by the same
// activation index registers, and the result is 256 * sum_hi + sum_lo.  Operand construction and instruction layout are
// those of the one-plane form (dg_onehot_kernel.h, BITS = 20).  A wavefront owns a 32 x 128 tile; large layers only.
#pragma once

#include "dg_onehot_kernel.h"

namespace dgoh {

struct Sparse2pArgs {
    DgProblem p;
    uint32_t rows[2][4];         // rows[plane][w] = bytes plane(T[w][0..3])
    FastDiv div_ow, div_oh;
    int32_t tiles_m;
    int64_t wave_tiles;
};

template <int CH>
__global__ void __launch_bounds__(256, 2)
sparse2p_kernel(Sparse2pArgs a)
{
    constexpr int WN = 4;
    __shared__ uint2 s_rows[4 * 32];                        // per wavefront: 16 row pairs of the low plane, then of the high
    const DgProblem &p = a.p;
    const int lane = threadIdx.x & 63, w4 = threadIdx.x >> 6;
    const int64_t wave_tile = (int64_t)xcd_contiguous(blockIdx.x, gridDim.x) * 4 + w4;
    if (wave_tile >= a.wave_tiles) return;                  // whole waves leave; there is no barrier
    uint2 *rows = s_rows + 32 * w4;
    if (lane < 32) {
        const int plane = lane >> 4, c0 = lane & 3, c1 = (lane >> 2) & 3;
        const uint32_t *r = a.rows[plane];
        const uint32_t r0 = c0 == 0 ? r[0] : (c0 == 1 ? r[1] : (c0 == 2 ? r[2] : r[3]));
        const uint32_t r1 = c1 == 0 ? r[0] : (c1 == 1 ? r[1] : (c1 == 2 ? r[2] : r[3]));
        rows[lane] = make_uint2(r0, r1);
    }
    __builtin_amdgcn_wave_barrier();                        // (LDS operations of one wavefront execute in order)

    const int r = lane & 31, h = lane >> 5;
    const int m0 = (int)(wave_tile % a.tiles_m) * 32;
    const int n0 = (int)(wave_tile / a.tiles_m) * 128;
    const int cq = p.Cin / 4;                               // packed bytes per pixel
    constexpr int CHUNK = 32 * CH;                          // codes of K per chunk
    const int chunks = p.K / CHUNK;
    const uint32_t pick = sparse_pick(h);

    const uint8_t *w_ptr = p.Wp + (int64_t)min(m0 + r, p.M - 1) * (p.K / 4);
    Column col[WN];
#pragma unroll
    for (int bn = 0; bn < WN; ++bn) col[bn] = make_column(p, a.div_ow, a.div_oh, n0 + bn * 32 + r, cq, h * (4 * CH));
    v16i acc[2][WN];
#pragma unroll
    for (int pl = 0; pl < 2; ++pl)
#pragma unroll
        for (int bn = 0; bn < WN; ++bn)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[pl][bn][e] = 0;
    float sc_cols[1];
    dg_mfma_column_scales<1, true>(p, m0, lane, sc_cols);

    int kh = 0, kw = 0, ci = 0;
    Words<CH> wa[2], wb[WN];
    bool vb[WN];
    auto fetch = [&](int chunk) {                            // `chunk` is clamped: a fetch past the end is unused
        const int cw = min(chunk, chunks - 1);
#pragma unroll
        for (int run = 0; run < 2; ++run) wa[run] = load_words<CH>(w_ptr + (int64_t)cw * (8 * CH) + run * (4 * CH));
        const int64_t tap_off = ((int64_t)kh * p.W + kw) * cq + ci / 4;
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
        Words<CH> ca[2], cb[WN];
        v4i ones[WN][2];
        ca[0] = wa[0], ca[1] = wa[1];
#pragma unroll
        for (int bn = 0; bn < WN; ++bn) {
            cb[bn] = wb[bn];
            // the kept bytes: (1, 0) per position with the even codes, (0, 1) with the odd; zeros outside the image
            const int x = vb[bn] ? 0x00010001 : 0, y = vb[bn] ? 0x01000100 : 0;
            ones[bn][0] = (v4i){x, x, x, x};
            ones[bn][1] = (v4i){y, y, y, y};
        }
        fetch(c + 1);                                        // unconditional (the last one re-reads in bounds and is unused)
#pragma unroll
        for (int t = 0; t < CH; ++t) {
            v8i dn[2][2];                                    // [plane][even, odd codes]; the index arithmetic is common
#pragma unroll
            for (int pl = 0; pl < 2; ++pl) sparse_dense_rows(rows + 16 * pl, ca[0].v[t], ca[1].v[t], pick, dn[pl][0], dn[pl][1]);
#pragma unroll
            for (int par = 0; par < 2; ++par)
#pragma unroll
                for (int bn = 0; bn < WN; ++bn) {
                    const int idx = (int)cb[bn].v[t];      // as packed: the byte that is 1 picks by its own code
#pragma unroll
                    for (int pl = 0; pl < 2; ++pl)
                        acc[pl][bn] = __builtin_amdgcn_smfmac_i32_32x32x64_i8(ones[bn][par], dn[pl][par], acc[pl][bn], idx, 0, 0);
                }
        }
    }
    v16i out[1][WN];
#pragma unroll
    for (int bn = 0; bn < WN; ++bn)
#pragma unroll
        for (int e = 0; e < 16; ++e) out[0][bn][e] = (int)((uint32_t)acc[0][bn][e] + ((uint32_t)acc[1][bn][e] << 8));
    dg_mfma_store_tile<1, WN, true>(p, out, m0, n0, lane, sc_cols);
}

inline void launch_sparse2p(const DgProblem &p, const uint32_t (&rows)[2][4], int ch, hipStream_t stream)
{
    Sparse2pArgs a;
    a.p = p;
    for (int pl = 0; pl < 2; ++pl)
        for (int w = 0; w < 4; ++w) a.rows[pl][w] = rows[pl][w];
    a.tiles_m = (p.M + 31) / 32;
    a.wave_tiles = (int64_t)a.tiles_m * (((int64_t)p.N + 127) / 128);
    a.div_ow = make_div((uint32_t)p.OW), a.div_oh = make_div((uint32_t)p.OH);
    const dim3 grid((unsigned)((a.wave_tiles + 3) / 4));
    if (ch == 2)
        hipLaunchKernelGGL((sparse2p_kernel<2>), grid, dim3(256), 0, stream, a);
    else
        hipLaunchKernelGGL((sparse2p_kernel<1>), grid, dim3(256), 0, stream, a);
}

}   // namespace dgoh
