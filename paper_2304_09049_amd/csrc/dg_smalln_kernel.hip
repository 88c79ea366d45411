// Table kernel for few activation rows (GEMV-like shapes: small N, large M and K).
//
// With N small the weights are streamed once and everything else is re-used, so the roles of the
// permute operands are mirrored with respect to the main kernel: the 8-byte permute POOL is built from
// the activations -- {column[a(n,k+1)], column[a(n,k)]}, a table column being the four products of one
// activation code with the four weight codes -- and is held in registers for the whole kernel, while the
// SELECTOR is cut from the streamed weight codes of two rows: [w(m0,k), 4 + w(m0,k+1), w(m1,k), 4 + w(m1,k+1)].
// One v_perm_b32 fetches four products; v_dot4_u32_u8 against 0/1 masks adds the two of each row to that
// row's int32 sum (entries are biased to 0..255; the bias, min_entry * K, is taken out at the end).
//
// K is split across the 256 lanes of a workgroup (32 codes = 8 packed bytes per lane per 8192-code chunk, so
// a weight row is read with fully coalesced 8-byte loads).  Every lane thus holds a partial sum of every
// row; the partial sums of a wavefront are added with DPP row operations (the paper's Listing 1 plays this
// role for an AVX2 register), the four wavefronts meet in LDS.
#include "dg_codes.h"
#include "dg_common.h"

namespace {

constexpr int KT = 32;            // codes of K per lane per chunk
constexpr int KC = 256 * KT;      // codes of K per chunk

struct SmallNArgs {
    DgProblem p;
    uint32_t cols[4];             // biased table columns: byte w of cols[c] = LUT[4w+c] - min_entry
    int32_t min_entry;
    int32_t blocks_per_wg;        // consecutive row blocks per workgroup
};

__device__ __forceinline__ uint32_t perm(uint32_t hi, uint32_t lo, uint32_t sel)
{
    return __builtin_amdgcn_perm(hi, lo, sel);
}

// Sum over the 64 lanes of a wavefront, returned in every lane (as a uniform value).
__device__ __forceinline__ int wave_sum(int v)
{
    v += __builtin_amdgcn_update_dpp(0, v, 0xB1, 0xF, 0xF, true);    // quad_perm [1,0,3,2]
    v += __builtin_amdgcn_update_dpp(0, v, 0x4E, 0xF, 0xF, true);    // quad_perm [2,3,0,1]
    v += __builtin_amdgcn_update_dpp(0, v, 0x141, 0xF, 0xF, true);   // row_half_mirror
    v += __builtin_amdgcn_update_dpp(0, v, 0x140, 0xF, 0xF, true);   // row_mirror: every lane has its row's sum
    return __builtin_amdgcn_readlane(v, 0) + __builtin_amdgcn_readlane(v, 16) +
           __builtin_amdgcn_readlane(v, 32) + __builtin_amdgcn_readlane(v, 48);
}

// 16 codes of two rows -> 8 selectors [x0 code 2q, 4 + x0 code 2q+1, x1 code 2q, 4 + x1 code 2q+1].
// `am`/`om` = 0x03030303 / 0x04000400 for live lanes, 0 / 0x0C0C0C0C for lanes beyond K (all products 0).
__device__ __forceinline__ void selectors(uint32_t x0, uint32_t x1, uint32_t am, uint32_t om, uint32_t *sel)
{
    const uint32_t x0s = x0 >> 2, x1s = x1 >> 2;
    const uint32_t u0_01 = perm(x0s, x0, 0x05010400u), u0_23 = perm(x0s, x0, 0x07030602u);
    const uint32_t u1_01 = perm(x1s, x1, 0x05010400u), u1_23 = perm(x1s, x1, 0x07030602u);
    uint32_t v[4];
    v[0] = perm(u1_01, u0_01, 0x05040100u);
    v[1] = perm(u1_01, u0_01, 0x07060302u);
    v[2] = perm(u1_23, u0_23, 0x05040100u);
    v[3] = perm(u1_23, u0_23, 0x07060302u);
#pragma unroll
    for (int b = 0; b < 4; ++b) {
        sel[2 * b] = (v[b] & am) | om;
        sel[2 * b + 1] = ((v[b] >> 4) & am) | om;
    }
}

// NC activation rows per pass; RB weight rows per block (all of a block's words are loaded before any is used).
// RAW: the activations are codes one per byte ([N][K] bytes at p.Xp), packed in registers as they are loaded -- for a
// problem this small the packing kernel's launch would cost a third of the whole.
template <int NC, int RB, bool RAW>
__global__ void __launch_bounds__(256)
smalln_kernel(SmallNArgs a)
{
    __shared__ uint2 s_table[16];             // activation nibble (a_even | a_odd << 2) -> {col[a_even], col[a_odd]}
    __shared__ int32_t s_red[4][RB][NC];      // per-wavefront sums of the current row block

    const DgProblem &p = a.p;
    const int t = threadIdx.x, wave = t >> 6, lane = t & 63;
    if (t < 16) s_table[t] = make_uint2(a.cols[t & 3], a.cols[t >> 2]);
    __syncthreads();

    const int row_bytes = p.K / 4;
    const int chunks = (p.K + KC - 1) / KC;
    const int first_block = blockIdx.x * a.blocks_per_wg;
    const int total_blocks = (p.M + RB - 1) / RB;

    for (int n0 = 0; n0 < p.N; n0 += NC) {
        for (int blk = first_block; blk < first_block + a.blocks_per_wg && blk < total_blocks; ++blk) {
            const int row0 = blk * RB;
            for (int chunk = 0; chunk < chunks; ++chunk) {
                const int kt = chunk * KC + t * KT;            // this lane's first reduction position
                const bool live = kt < p.K;
                const uint32_t am = live ? 0x03030303u : 0u, om = live ? 0x04000400u : 0x0C0C0C0Cu;
                const int koff = live ? kt / 4 : 0;

                // all weight words of the row block first: RB independent 8-byte loads in flight per lane
                uint2 w[RB];
#pragma unroll
                for (int r = 0; r < RB; ++r) {
                    int m = row0 + r;
                    if (m >= p.M) m = p.M - 1;                 // rows beyond M: a valid row, never stored
                    w[r] = *(const uint2 *)(p.Wp + (int64_t)m * row_bytes + koff);
                }
                // pools of this lane's 32 positions, for NC activation rows
                uint2 pool[NC][KT / 2];
#pragma unroll
                for (int c = 0; c < NC; ++c) {
                    int n = n0 + c;
                    if (n >= p.N) n = p.N - 1;
                    uint2 x;
                    if constexpr (RAW) {
                        const uint4 *codes = (const uint4 *)(p.Xp + (int64_t)n * p.K + 4 * koff);
                        x = make_uint2(dg_pack_codes16(codes[0]), dg_pack_codes16(codes[1]));
                    } else {
                        x = *(const uint2 *)(p.Xp + (int64_t)n * row_bytes + koff);
                    }
#pragma unroll
                    for (int q = 0; q < 8; ++q) {
                        pool[c][q] = s_table[(x.x >> (4 * q)) & 15u];
                        pool[c][8 + q] = s_table[(x.y >> (4 * q)) & 15u];
                    }
                }
#pragma unroll
                for (int rp = 0; rp < RB / 2; ++rp) {
                    uint32_t sel[KT / 2];
                    selectors(w[2 * rp].x, w[2 * rp + 1].x, am, om, sel);
                    selectors(w[2 * rp].y, w[2 * rp + 1].y, am, om, sel + 8);
#pragma unroll
                    for (int c = 0; c < NC; ++c) {
                        uint32_t s0 = 0, s1 = 0;
#pragma unroll
                        for (int q = 0; q < KT / 2; ++q) {
                            const uint32_t r4 = perm(pool[c][q].y, pool[c][q].x, sel[q]);
                            s0 = __builtin_amdgcn_udot4(r4, 0x00000101u, s0, false);
                            s1 = __builtin_amdgcn_udot4(r4, 0x01010000u, s1, false);
                        }
                        const int t0 = wave_sum((int)s0), t1 = wave_sum((int)s1);
                        if (lane == 0) {
                            if (chunk == 0) {
                                s_red[wave][2 * rp][c] = t0;
                                s_red[wave][2 * rp + 1][c] = t1;
                            } else {
                                s_red[wave][2 * rp][c] += t0;
                                s_red[wave][2 * rp + 1][c] += t1;
                            }
                        }
                    }
                }
            }
            __syncthreads();
            if (t < RB * NC) {
                const int r = t / NC, c = t % NC;
                const int m = row0 + r, n = n0 + c;
                if (m < p.M && n < p.N) {
                    const int32_t v = s_red[0][r][c] + s_red[1][r][c] + s_red[2][r][c] + s_red[3][r][c] +
                                      a.min_entry * p.K;
                    const int64_t o = (int64_t)m * p.stride_cm + (int64_t)n * p.stride_cn;
                    if (p.scale)
                        p.Cf[o] = (float)v * p.scale[m];
                    else
                        p.C[o] = v;
                }
            }
            __syncthreads();
        }
    }
}

}   // namespace

bool dg_smalln_supports(const dg_lut *lut, const DgProblem &p)
{
    if (lut->max_entry - lut->min_entry > 255) return false;     // a biased entry must fit the byte a permute fetches
    if (p.KH != 1 || p.KW != 1 || p.ph != 0 || p.pw != 0 || p.sh != 1 || p.sw != 1) return false;   // rows of K codes
    if (p.K % KT != 0) return false;                             // a lane reads whole 8-byte groups
    if ((uintptr_t)p.Wp % 8 != 0 || (uintptr_t)p.Xp % 8 != 0) return false;
    return true;
}

namespace {

template <bool RAW>
dg_status launch(const dg_lut *lut, const DgProblem &p, hipStream_t stream)
{
    SmallNArgs a;
    a.p = p;
    a.min_entry = lut->min_entry;
    for (int c = 0; c < 4; ++c) {
        uint32_t col = 0;
        for (int w = 0; w < 4; ++w) col |= (uint32_t)(lut->entry[4 * w + c] - lut->min_entry) << (8 * w);
        a.cols[c] = col;
    }
    // one activation row: 8-row blocks (more workgroups in flight while the weights stream in); more rows: 16-row
    // blocks (the activation pools are rebuilt per block, so longer blocks amortise them)
    const int rb = p.N >= 2 ? 16 : 8;
    const int total_blocks = (p.M + rb - 1) / rb;
    // about four workgroups per compute unit; longer runs of row blocks per workgroup beyond that
    int per_wg = (total_blocks + 1023) / 1024;
    if (per_wg < 1) per_wg = 1;
    a.blocks_per_wg = per_wg;
    const dim3 grid((unsigned)((total_blocks + per_wg - 1) / per_wg));
    if (p.N >= 4)
        hipLaunchKernelGGL((smalln_kernel<4, 16, RAW>), grid, dim3(256), 0, stream, a);
    else if (p.N >= 2)
        hipLaunchKernelGGL((smalln_kernel<2, 16, RAW>), grid, dim3(256), 0, stream, a);
    else
        hipLaunchKernelGGL((smalln_kernel<1, 8, RAW>), grid, dim3(256), 0, stream, a);
    return dg_check_launch("smalln_kernel");
}

}   // namespace

dg_status dg_launch_smalln(const dg_lut *lut, const DgProblem &p, hipStream_t stream)
{
    return launch<false>(lut, p, stream);
}

// p.Xp = the activation codes one per byte, 16-byte aligned
dg_status dg_launch_smalln_codes(const dg_lut *lut, const DgProblem &p, hipStream_t stream)
{
    return launch<true>(lut, p, stream);
}
