// 2-bit table kernel for GEMMs with few activation rows (N <= 16 per pass; large M and K: the weights are streamed once
// and are all of the traffic), on the sparse matrix instruction v_smfmac_i32_16x16x128_i8.
//
// Here the WEIGHTS are the instruction's sparse operand: its kept bytes are the constants (1, 0) (even codes) or (0, 1)
// (odd codes) and its index register is the packed weight word as loaded -- so the streamed operand costs no
// instruction at all -- and the instruction's index multiplexer picks, out of the four bytes the dense
// operand holds per reduction position, the entry of the weight code: the dense operand is the table COLUMN of the
// activation code, T[0..3][a(n,k)], fetched from a 16-entry table of column pairs in LDS as in the tiled
// sparse-instruction kernel (dg_onehot_kernel.h, with the roles of weights and activations exchanged).
//
// Instruction layout (measured): lane (i = lane % 16, q = lane / 16) of the sparse operand holds row i, 16 kept bytes j
// and the 2-bit fields j of its own index register; kept byte j multiplies byte 16 (q / 2) + 4 ((j % 8) / 2) + field_j of
// the dense lane (column, 2 (q % 2) + j / 8).  Sums: lane l, register e = row 4 (l / 16) + e, column l % 16.
//
// Work split: a workgroup owns 16 R weight rows and all of K; its wavefronts split K in super-steps of 256 positions
// (one 16-byte load per lane and row block), build the dense operands of their positions once and use them for all R
// row blocks; the wavefronts' sums meet in LDS by integer atomics (exact in any order).
#include <cstdlib>
#include <cstring>

#include "dg_onehot_kernel.h"

namespace {

using dgoh::v4i;
using dgoh::v8i;

struct FewNArgs {
    DgProblem p;
    uint32_t cols[4];            // cols[a] = bytes T[0..3][a]: the table column of activation code a
    int32_t supersteps;          // K / 256
};

constexpr int SPW = 4;           // super-steps a wavefront loads at a time

// The dense operands of the two instructions (even codes, odd codes) that consume one packed weight word per lane
// group: dwords 0-3 from activation word w0, dwords 4-7 from w1, each the table column of one code of the 16-bit half
// `pick` selects (dg_onehot_kernel.h, sparse_dense_rows, describes the arrangement).  The table of column pairs is ONE
// copy at a fixed LDS address shared by the workgroup's wavefronts, so a read's address is just the 4-bit index times
// 8: one bit-field extract per read (the indices are kept pre-multiplied, a byte each).
__device__ __forceinline__ void dense_columns(const uint2 *table, uint32_t w0, uint32_t w1, uint32_t pick, v8i &even, v8i &odd)
{
    const uint32_t v = __builtin_amdgcn_perm(w1, w0, pick), t = v >> 2;
    uint32_t e = ((v & 0x03030303u) | (t & 0x0C0C0C0Cu)) << 3;        // byte b: 8 * (code 4b | code 4b+2 << 2)
    uint32_t o = ((t & 0x03030303u) | ((v >> 4) & 0x0C0C0C0Cu)) << 3; // byte b: 8 * (code 4b+1 | code 4b+3 << 2)
    // (kept as they are: a byte of them IS an LDS offset, one bit-field extract away; left to itself the compiler
    // folds the multiplication into a shift and a mask per read)
    asm volatile("" : "+v"(e), "+v"(o));
    const char *base = (const char *)table;
#pragma unroll
    for (int b = 0; b < 4; ++b) {
        const uint2 x = *(const uint2 *)(base + ((e >> (8 * b)) & 255u)), y = *(const uint2 *)(base + ((o >> (8 * b)) & 255u));
        even[2 * b] = (int)x.x, even[2 * b + 1] = (int)x.y;
        odd[2 * b] = (int)y.x, odd[2 * b + 1] = (int)y.y;
    }
}

// R: row blocks of 16 rows per workgroup.
// (one workgroup of up to 16 wavefronts per compute unit)
template <int R>
__global__ void __launch_bounds__(1024, 1)
fewn_kernel(FewNArgs a)
{
    __shared__ uint2 s_table[16];                           // entry (c0 | c1 << 2) = {column of code c0, column of code c1}
    __shared__ int32_t s_sum[R * 4 * 64];                   // [row block][sum register][lane]
    const DgProblem &p = a.p;
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6, waves = blockDim.x >> 6;
    for (int i = threadIdx.x; i < R * 256; i += blockDim.x) s_sum[i] = 0;
    if (threadIdx.x < 16) s_table[threadIdx.x] = make_uint2(a.cols[threadIdx.x & 3], a.cols[threadIdx.x >> 2]);
    const int i16 = lane & 15, q = lane >> 4;
    const int m0 = blockIdx.x * (16 * R), n0 = blockIdx.y * 16;
    const int64_t row_bytes = p.K / 4;
    // weight rows (rows beyond M re-read row M - 1: their sums are not stored), this lane's 16 bytes of a super-step
    const uint8_t *w_ptr[R];
#pragma unroll
    for (int rb = 0; rb < R; ++rb) w_ptr[rb] = p.Wp + (int64_t)min(m0 + 16 * rb + i16, p.M - 1) * row_bytes + 16 * q;
    // activation row (columns beyond N re-read row N - 1): the words whose codes this lane's dense registers cover
    const uint8_t *x_ptr = p.Xp + (int64_t)min(n0 + i16, p.N - 1) * row_bytes + 16 * (q >> 1);
    const uint32_t pick = dgoh::sparse_pick(q & 1);
    // the kept bytes: (1, 0) per position with the even codes, (0, 1) with the odd; the index of both is the packed word
    // (of a 4-bit field the low half is the first kept byte's index, the high half the second's; the byte that is 0 may
    // pick anything)
    const v4i ones_even = {0x00010001, 0x00010001, 0x00010001, 0x00010001};
    const v4i ones_odd = {0x01000100, 0x01000100, 0x01000100, 0x01000100};

    v4i acc[R];
#pragma unroll
    for (int rb = 0; rb < R; ++rb) acc[rb] = (v4i){0, 0, 0, 0};

    // this wavefront's super-steps: a contiguous run, SPW at a time (all their loads in flight together)
    const int per = (a.supersteps + waves - 1) / waves;
    const int s0 = min(wv * per, a.supersteps), s1 = min(s0 + per, a.supersteps);
    bool table_ready = false;
    for (int sg = s0; sg < s1; sg += SPW) {
        uint4 wq[SPW][R], x0[SPW], x1[SPW];
#pragma unroll
        for (int u = 0; u < SPW; ++u) {
            const int64_t off = (int64_t)min(sg + u, s1 - 1) * 64;      // (a step past the run re-reads the last one, unused)
#pragma unroll
            for (int rb = 0; rb < R; ++rb) wq[u][rb] = *(const uint4 *)(w_ptr[rb] + off);
            x0[u] = *(const uint4 *)(x_ptr + off);
            x1[u] = *(const uint4 *)(x_ptr + off + 32);
        }
        // (the table and the zeroed sums are in LDS once every wavefront is here; the loads above stay in flight across
        // this barrier, which waits for LDS operations only)
        if (!table_ready) asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
        table_ready = true;
        // Step tt = word tt % 4 of super-step tt / 4.  The dense operands of step tt + 1 are fetched while the matrix
        // instructions of step tt run (two register sets), so the table reads' latency is covered.
        const uint32_t xa[SPW][4] = {{x0[0].x, x0[0].y, x0[0].z, x0[0].w}, {x0[1].x, x0[1].y, x0[1].z, x0[1].w},
                                     {x0[2].x, x0[2].y, x0[2].z, x0[2].w}, {x0[3].x, x0[3].y, x0[3].z, x0[3].w}};
        const uint32_t xb[SPW][4] = {{x1[0].x, x1[0].y, x1[0].z, x1[0].w}, {x1[1].x, x1[1].y, x1[1].z, x1[1].w},
                                     {x1[2].x, x1[2].y, x1[2].z, x1[2].w}, {x1[3].x, x1[3].y, x1[3].z, x1[3].w}};
        v8i even[2], odd[2];
        dense_columns(s_table, xa[0][0], xb[0][0], pick, even[0], odd[0]);
#pragma unroll
        for (int tt = 0; tt < 4 * SPW; ++tt) {
            const int u = tt / 4, t = tt % 4, cur = tt & 1;
            if (sg + u >= s1) break;                        // (uniform)
            if (tt + 1 < 4 * SPW)                           // (past the run's end: built from re-read words, unused)
                dense_columns(s_table, xa[(tt + 1) / 4][(tt + 1) % 4], xb[(tt + 1) / 4][(tt + 1) % 4], pick, even[cur ^ 1], odd[cur ^ 1]);
#pragma unroll
            for (int rb = 0; rb < R; ++rb) {
                const uint32_t word = t == 0 ? wq[u][rb].x : (t == 1 ? wq[u][rb].y : (t == 2 ? wq[u][rb].z : wq[u][rb].w));
                acc[rb] = __builtin_amdgcn_smfmac_i32_16x16x128_i8(ones_even, even[cur], acc[rb], (int)word, 0, 0);
                acc[rb] = __builtin_amdgcn_smfmac_i32_16x16x128_i8(ones_odd, odd[cur], acc[rb], (int)word, 0, 0);
            }
        }
    }

    if (!table_ready) asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");      // (a wavefront without super-steps)
#pragma unroll
    for (int rb = 0; rb < R; ++rb)
#pragma unroll
        for (int e = 0; e < 4; ++e)
            __hip_atomic_fetch_add(&s_sum[(rb * 4 + e) * 64 + lane], acc[rb][e], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    __syncthreads();
    for (int idx = threadIdx.x; idx < R * 256; idx += blockDim.x) {
        const int rb = idx >> 8, e = (idx >> 6) & 3, l = idx & 63;
        const int m = m0 + 16 * rb + 4 * (l >> 4) + e, n = n0 + (l & 15);
        if (m >= p.M || n >= p.N) continue;
        const int64_t o = (int64_t)m * p.stride_cm + (int64_t)n * p.stride_cn;
        if (p.scale)
            p.Cf[o] = (float)s_sum[idx] * p.scale[m];
        else
            p.C[o] = s_sum[idx];
    }
}

bool fits_int8(const dg_lut *lut) { return lut->min_entry >= -128 && lut->max_entry <= 127; }

}   // namespace

bool dg_fewn_supports(const dg_lut *lut, const DgProblem &p)
{
    if (lut->dtype == DG_LUT_F32 || lut->bits != 2 || !fits_int8(lut)) return false;
    // every activation row is one contiguous run of K codes: a GEMM, or a 1x1 convolution without stride or padding
    if (p.KH != 1 || p.KW != 1 || p.sh != 1 || p.sw != 1 || p.ph != 0 || p.pw != 0) return false;
    if (p.K % 256 != 0 || p.Qp != nullptr) return false;              // whole super-steps; no re-quantising epilogue
    if ((uintptr_t)p.Wp % 16 != 0 || (uintptr_t)p.Xp % 16 != 0) return false;
    return (p.N + 15) / 16 <= 65535 && (p.M + 31) / 32 <= INT32_MAX / 2;
}

// AUTO: one pass of 16 columns streams the weights once; measured against the split-K and the few-columns permute kernels
bool dg_fewn_preferred(const dg_lut *lut, const DgProblem &p)
{
    if (!dg_fewn_supports(lut, p)) return false;
    if (const char *force = dg_override("DG_ONEHOT_PLAN")) return strcmp(force, "fewn") == 0;      // (tests reach it on small shapes)
    // (one column: the permute kernel with K across the lanes is faster, 5.4 against 6.5 us on 8192 x 8192 weights;
    // from 17 columns on the weights would be streamed twice and the split-K matrix-core kernel is faster)
    return p.N >= 2 && p.N <= 16 && p.K >= 2048 && (int64_t)p.M * p.K >= ((int64_t)1 << 22);
}

dg_status dg_launch_fewn(const dg_lut *lut, const DgProblem &p, hipStream_t stream)
{
    FewNArgs a;
    a.p = p;
    a.supersteps = p.K / 256;
    for (int c = 0; c < 4; ++c) {
        a.cols[c] = 0;
        for (int w = 0; w < 4; ++w) a.cols[c] |= (uint32_t)(uint8_t)(int8_t)lut->entry[(w << 2) | c] << (8 * w);
    }
    // as many wavefronts as there are runs of 4 super-steps (what a wavefront loads at a time), up to 8 (measured: 16
    // wavefronts of 2 super-steps each are slower); 32 rows per workgroup while that gives every compute unit a
    // workgroup, else 16
    int waves = (a.supersteps + SPW - 1) / SPW;
    waves = waves < 1 ? 1 : (waves > 8 ? 8 : waves);
    if (const char *e = dg_override("DG_FEWN_WAVES")) waves = atoi(e) >= 1 && atoi(e) <= 16 ? atoi(e) : waves;
    const bool two = (p.M + 31) / 32 >= dg_simd_count() / 4;
    const dim3 grid((unsigned)((p.M + (two ? 31 : 15)) / (two ? 32 : 16)), (unsigned)((p.N + 15) / 16)), block(64 * waves);
    if (two)
        hipLaunchKernelGGL((fewn_kernel<2>), grid, block, 0, stream, a);
    else
        hipLaunchKernelGGL((fewn_kernel<1>), grid, block, 0, stream, a);
    return dg_check_launch("fewn_kernel");
}
