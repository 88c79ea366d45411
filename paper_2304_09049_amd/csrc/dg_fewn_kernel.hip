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

#include "dg_lds_dma.h"
#include "dg_onehot_kernel.h"

namespace {

using dgoh::v4i;
using dgoh::v8i;

struct FewNArgs {
    DgProblem p;
    uint32_t cols[4];            // cols[a] = bytes T[0..3][a]: the table column of activation code a
    int32_t supersteps;          // K / 256
};

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

// R: row blocks of 16 rows per workgroup.  Up to 8 wavefronts.
//
// Loads: a super-step of a row block is 16 rows x 64 bytes.  With the operand layout's lane order (row = lane % 16)
// every lane of a load would touch a cache line of its own -- 60 address cycles per instruction, which made the
// address unit the kernel's longest phase (39 % of its time busy) -- so the loads are staged (dg_lds_dma.h): four
// neighbouring lanes read the 64 bytes of one row, 15 cycles per instruction, straight into LDS, and lane (row, q)
// reads its 16 bytes from there.  Slot j of a staged block (16 bytes, written by loader lane j) holds row j / 4,
// segment (j % 4) ^ (j / 16 % 4): the exchange spreads the 16 rows of one segment over all LDS banks.
template <int R>
__global__ void __launch_bounds__(512, R == 1 ? 2 : 1)
fewn_kernel(FewNArgs a)
{
    constexpr int SS = (R + 1) * 1024;                      // staged bytes of a super-step: R weight blocks, the activations
    __shared__ uint2 s_table[16];                           // entry (c0 | c1 << 2) = {column of code c0, column of code c1}
    __shared__ int32_t s_sum[R * 4 * 64];                   // [row block][sum register][lane]
    __shared__ uint4 s_stage[8][2][SS / 16];                // [wavefront][buffer][block * 64 + slot]
    const DgProblem &p = a.p;
    const int lane = threadIdx.x & 63, wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), waves = blockDim.x >> 6;
    for (int i = threadIdx.x; i < R * 256; i += blockDim.x) s_sum[i] = 0;
    if (threadIdx.x < 16) s_table[threadIdx.x] = make_uint2(a.cols[threadIdx.x & 3], a.cols[threadIdx.x >> 2]);
    const int i16 = lane & 15, q = lane >> 4;
    const int m0 = blockIdx.x * (16 * R), n0 = blockIdx.y * 16;
    const int64_t row_bytes = p.K / 4;
    // as a loader: segment lseg of row lrow of every block (rows beyond M or N re-read the last one: never stored)
    const int lrow = lane >> 2, lseg = (lane & 3) ^ ((lane >> 4) & 3);
    const uint8_t *w_ld[R];
#pragma unroll
    for (int rb = 0; rb < R; ++rb) w_ld[rb] = p.Wp + (int64_t)min(m0 + 16 * rb + lrow, p.M - 1) * row_bytes + 16 * lseg;
    const uint8_t *x_ld = p.Xp + (int64_t)min(n0 + lrow, p.N - 1) * row_bytes + 16 * lseg;
    // as a consumer: of weight row i16 segment q (the sparse operand's index words), of activation row i16 the two
    // segments whose codes this lane's dense registers cover
    auto slot_at = [&](int seg) { return (4 * i16 + (seg ^ ((i16 >> 2) & 3))) * 16; };
    const int w_at = slot_at(q), x0_at = slot_at(q >> 1), x1_at = slot_at(2 + (q >> 1));
    const char *stage = (const char *)s_stage[wv];
    const uint32_t stage_lds = dg_lds_address(s_stage) + wv * (2 * SS);
    const uint32_t pick = dgoh::sparse_pick(q & 1);
    // the kept bytes: (1, 0) per position with the even codes, (0, 1) with the odd; the index of both is the packed word
    // (of a 4-bit field the low half is the first kept byte's index, the high half the second's; the byte that is 0 may
    // pick anything)
    const v4i ones_even = {0x00010001, 0x00010001, 0x00010001, 0x00010001};
    const v4i ones_odd = {0x01000100, 0x01000100, 0x01000100, 0x01000100};

    v4i acc[R];
#pragma unroll
    for (int rb = 0; rb < R; ++rb) acc[rb] = (v4i){0, 0, 0, 0};

    // this wavefront's super-steps: a contiguous run, fetched two ahead into two buffers
    const int per = (a.supersteps + waves - 1) / waves;
    const int s0 = min(wv * per, a.supersteps), s1 = min(s0 + per, a.supersteps);
    int fetched = s0;
    auto fetch = [&]() {                                    // (past the run's end: its last super-step again, unused)
        const int64_t off = (int64_t)min(fetched, s1 - 1) * 64;
        const uint32_t dst = stage_lds + ((fetched - s0) & 1) * SS;
#pragma unroll
        for (int rb = 0; rb < R; ++rb) dg_load16_to_lds(w_ld[rb] + off, dst + rb * 1024);
        dg_load16_to_lds(x_ld + off, dst + R * 1024);
        ++fetched;
    };
    if (s0 < s1) {
        fetch();
        fetch();
    }
    // (the table and the zeroed sums are in LDS once every wavefront is here; the loads above stay in flight across
    // this barrier, which waits for LDS operations only)
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    for (int ss = s0; ss < s1; ++ss) {
        // the older of the two fetches in flight is in (loads complete in order; the newer one is R + 1 instructions)
        dg_wait_for_loads<R + 1>();
        const char *src = stage + ((ss - s0) & 1) * SS;
        uint4 wq[R];
#pragma unroll
        for (int rb = 0; rb < R; ++rb) wq[rb] = *(const uint4 *)(src + rb * 1024 + w_at);
        const uint4 x0 = *(const uint4 *)(src + R * 1024 + x0_at), x1 = *(const uint4 *)(src + R * 1024 + x1_at);
        const uint32_t xa[4] = {x0.x, x0.y, x0.z, x0.w}, xb[4] = {x1.x, x1.y, x1.z, x1.w};
        // Step t = word t of the super-step.  The dense operands of step t + 1 are fetched while the matrix
        // instructions of step t run (two register sets), so the table reads' latency is covered.
        v8i even[2], odd[2];
        dense_columns(s_table, xa[0], xb[0], pick, even[0], odd[0]);
        // (the buffer's words are in registers -- dense_columns used them: the fetch after next may overwrite it)
        fetch();
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int cur = t & 1;
            if (t + 1 < 4) dense_columns(s_table, xa[t + 1], xb[t + 1], pick, even[cur ^ 1], odd[cur ^ 1]);
#pragma unroll
            for (int rb = 0; rb < R; ++rb) {
                const uint32_t word = t == 0 ? wq[rb].x : (t == 1 ? wq[rb].y : (t == 2 ? wq[rb].z : wq[rb].w));
                acc[rb] = __builtin_amdgcn_smfmac_i32_16x16x128_i8(ones_even, even[cur], acc[rb], (int)word, 0, 0);
                acc[rb] = __builtin_amdgcn_smfmac_i32_16x16x128_i8(ones_odd, odd[cur], acc[rb], (int)word, 0, 0);
            }
        }
    }
    dg_wait_for_loads();                                    // (the unused fetches past the end: their LDS writes end before the wavefront does)

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
    // (measured on 8192 x 8192 weights: 5.1 - 5.25 us for 1 to 16 columns, against 5.4 us of the permute kernel with K
    // across the lanes on one column; from 17 columns on the weights would be streamed twice and the tiled kernels
    // are faster)
    return p.N >= 1 && p.N <= 16 && p.K >= 2048 && (int64_t)p.M * p.K >= ((int64_t)1 << 22);
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
    // a wavefront per 4 super-steps, up to 8 (the staging buffers' number); 32 rows per workgroup while that gives
    // every compute unit a workgroup, else 16
    int waves = (a.supersteps + 3) / 4;
    waves = waves < 1 ? 1 : (waves > 8 ? 8 : waves);
    if (const char *e = dg_override("DG_FEWN_WAVES")) waves = atoi(e) >= 1 && atoi(e) <= 8 ? atoi(e) : waves;
    bool two = (p.M + 31) / 32 >= dg_simd_count() / 4;
    if (const char *e = dg_override("DG_FEWN_ROWS")) two = atoi(e) == 32;      // (A/B measurement)
    const dim3 grid((unsigned)((p.M + (two ? 31 : 15)) / (two ? 32 : 16)), (unsigned)((p.N + 15) / 16)), block(64 * waves);
    if (two)
        hipLaunchKernelGGL((fewn_kernel<2>), grid, block, 0, stream, a);
    else
        hipLaunchKernelGGL((fewn_kernel<1>), grid, block, 0, stream, a);
    return dg_check_launch("fewn_kernel");
}
