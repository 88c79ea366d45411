// Accumulator tiles of v_mfma_i32_32x32x32_i8 and their way to memory, shared by the two matrix-core kernels.
//
// A 32x32 accumulator block lives in 16 registers per lane: the lane holds MFMA column (lane % 32) and MFMA rows
// 8*(e/4) + 4*(lane/32) + e%4, e = 0..15.  Which problem axis sits on the MFMA columns is the kernel's choice (the two
// operands have the same lane layout, so swapping them transposes the block): the axis whose output stride is 1
// goes on the columns, so that the 32 lanes of a half wavefront store 128 contiguous bytes.
//   TR == false: MFMA rows = m, columns = n  (acc = mfma(weights, activations)) -- row-major GEMM output, n contiguous
//   TR == true : MFMA rows = n, columns = m  (acc = mfma(activations, weights)) -- NHWC convolution output, m contiguous
#pragma once

#include "dg_common.h"
#include "dg_quant.h"

typedef int dg_v4i __attribute__((ext_vector_type(4)));
typedef int dg_v16i __attribute__((ext_vector_type(16)));

template <bool TR>
__device__ __forceinline__ dg_v16i dg_mfma_step(dg_v4i w, dg_v4i x, dg_v16i acc)
{
    return TR ? __builtin_amdgcn_mfma_i32_32x32x32_i8(x, w, acc, 0, 0, 0)
              : __builtin_amdgcn_mfma_i32_32x32x32_i8(w, x, acc, 0, 0, 0);
}

// With TR a lane stores one channel m per row block whatever the element, so its scales can be fetched long before the
// stores: dg_mfma_column_scales at the start of the kernel, handed to dg_mfma_store_tile at the end.
template <int WM, bool TR>
__device__ __forceinline__ void dg_mfma_column_scales(const DgProblem &p, int m0, int lane, float (&sc)[WM])
{
#pragma unroll
    for (int bm = 0; bm < WM; ++bm) {
        const int m = min(m0 + bm * 32 + (lane & 31), p.M - 1);
        sc[bm] = (TR && p.scale) ? p.scale[m] : 0.0f;
    }
}

// Store one 32x32 block whose first row / column sit at (mb, nb): int32 as it is, or float(acc) * scale[m] (one
// conversion, one multiply); `sc` is the lane's prefetched scale (TR only).
// OR of `v` over the four lanes of a quad (two DPP quad permutes); every lane gets the result.
__device__ __forceinline__ uint32_t dg_quad_or(uint32_t v)
{
    v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xF, 0xF, true);    // quad_perm [1,0,3,2]
    v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E, 0xF, 0xF, true);    // quad_perm [2,3,0,1]
    return v;
}

// Re-quantising store of one block (TR layout only: the lanes of a quad hold four consecutive channels of one output
// pixel).  Each lane turns its 16 sums into 2-bit codes.  For four consecutive pixels (accumulator registers 4q .. 4q+3)
// a lane places its four codes in the four bytes of a word, at the bit position of its channel within the packed byte;
// one OR across the quad (two DPP permutes) completes the four packed bytes in every lane, and lane i of the quad
// stores the byte of pixel i -- so all lanes store.  Call with all 64 lanes active.
__device__ __forceinline__ void dg_mfma_requant_block(const DgProblem &p, const dg_v16i &acc, int mb, int nb, int lane,
                                                      float sc)
{
    const int r = lane & 31, h = lane >> 5, q = r & 3;
    const bool live = mb + r < p.M;                       // (M % 4 == 0: a quad is inside M or outside as a whole)
    const float lo_f = (float)p.q_lo, hi_f = (float)(p.q_lo + 3);
    const int64_t row_bytes = p.M / 4;
#pragma unroll
    for (int e4 = 0; e4 < 4; ++e4) {
        uint32_t word = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float y = __fmul_rn((float)acc[4 * e4 + i], sc);
            word |= dg_quantize_code_clamped(y, p.q_scale, p.q_zero, lo_f, hi_f) << (8 * i);
        }
        word = dg_quad_or(live ? word << (2 * q) : 0u);   // byte i = the packed byte of pixel i
        const int n = nb + 8 * e4 + 4 * h + q;            // the pixel whose byte this lane stores
        if (live && n < p.N) p.Qp[(int64_t)n * row_bytes + (mb + r) / 4] = (uint8_t)(word >> (8 * q));
    }
}

template <bool TR>
__device__ __forceinline__ void dg_mfma_store_block(const DgProblem &p, const dg_v16i &acc, int mb, int nb, int lane,
                                                    float sc)
{
    if (TR && p.Qp) {
        dg_mfma_requant_block(p, acc, mb, nb, lane, sc);
        return;
    }
    const int r = lane & 31, h = lane >> 5;
    // (mb and nb are the same in every lane of the wavefront: say so, and the block's base address is scalar arithmetic)
    const int colb = __builtin_amdgcn_readfirstlane(TR ? mb : nb), rowb = __builtin_amdgcn_readfirstlane(TR ? nb : mb);
    const int col_limit = TR ? p.M : p.N, row_limit = TR ? p.N : p.M;
    const int64_t row_stride = TR ? p.stride_cn : p.stride_cm, col_stride = TR ? p.stride_cm : p.stride_cn;
    // A block wholly inside the output whose 32 x 32 footprint spans less than 2^30 elements (strides may be negative):
    // one uniform base address, a 32-bit offset per lane, then steps of the row stride -- no bounds test and no 64-bit
    // arithmetic per element.  The stores are streaming (non-temporal) stores: the output is written once and read by
    // a later kernel, it has no business in this one's caches.
    const int64_t span = 32 * ((row_stride < 0 ? -row_stride : row_stride) + (col_stride < 0 ? -col_stride : col_stride));
    if (colb + 32 <= col_limit && rowb + 32 <= row_limit && span < ((int64_t)1 << 30)) {
        const int64_t base = (int64_t)colb * col_stride + (int64_t)rowb * row_stride;
        const int rs = (int)row_stride, off0 = r * (int)col_stride + 4 * h * rs;
        if (p.scale) {
            float *out = p.Cf + base;
            const float *scale_rows = p.scale + rowb + 4 * h;          // (row-major GEMM output: the scale goes with the row)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int k = 8 * (e / 4) + (e % 4);
                __builtin_nontemporal_store((float)acc[e] * (TR ? sc : scale_rows[k]), out + (off0 + k * rs));
            }
        } else {
            int32_t *out = p.C + base;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int k = 8 * (e / 4) + (e % 4);
                __builtin_nontemporal_store(acc[e], out + (off0 + k * rs));
            }
        }
        return;
    }
    // a block on the output's edge: every element tested
    const int col = colb + r;
    if (col >= col_limit) return;
    const int row0 = rowb + 4 * h;
    const int64_t first = (int64_t)col * col_stride + (int64_t)row0 * row_stride;
#pragma unroll
    for (int e = 0; e < 16; ++e) {
        const int k = 8 * (e / 4) + (e % 4);
        if (row0 + k >= row_limit) continue;
        const int64_t o = first + k * row_stride;
        if (p.scale)
            __builtin_nontemporal_store((float)acc[e] * (TR ? sc : p.scale[row0 + k]), p.Cf + o);
        else
            __builtin_nontemporal_store(acc[e], p.C + o);
    }
}

// Store the (WM*32) x (WN*32) tile at (m0, n0).
template <int WM, int WN, bool TR>
__device__ __forceinline__ void dg_mfma_store_tile(const DgProblem &p, const dg_v16i (&acc)[WM][WN], int m0, int n0,
                                                   int lane, const float (&sc_cols)[WM])
{
#pragma unroll
    for (int bm = 0; bm < WM; ++bm)
#pragma unroll
        for (int bn = 0; bn < WN; ++bn)
            dg_mfma_store_block<TR>(p, acc[bm][bn], m0 + bm * 32, n0 + bn * 32, lane, sc_cols[bm]);
}
