// LUT-65k on gfx950 (Sec. 3 "LUT-65k"): a table with one entry per (weight byte, activation byte), each entry the
// dot product of the four 2-bit weight codes with the four 2-bit activation codes packed in those bytes.  The index
// is the two packed bytes side by side, so no 2-bit field is ever extracted in the main loop: one table read per
// FOUR products.  The paper keeps the 64 KB table in the CPU's L2 cache; here it lives in LDS (160 KB per compute
// unit on CDNA4), built once per workgroup, and workgroups are persistent (they loop over output tiles).
//
// Table layout: entry[(a << 8) | w], a = activation byte 0..255 or 256, w = weight byte.  Row a = 256 is all zero
// and stands for a filter tap outside the image (and for columns beyond N), so padding needs no branch.
// Entries are int8 when four products always fit (the paper's assumption, here checked), else int16.
// Accumulation is int32 and exact.  Lane tile TM x TN; per packed byte position a lane forms TM*TN indices
// (v_lshl_or_b32), reads TM*TN entries and adds them.
//
// This kernel exists for the register-versus-LDS comparison the method invites; DG_KERNEL_AUTO never selects it.
#include "dg_common.h"

namespace {

constexpr int KB = 16;                 // packed bytes of K per stage (64 codes)
constexpr int TABLE_ROWS = 257;        // 256 activation bytes + the all-zero row

struct Lut65kArgs {
    DgProblem p;
    int16_t entry[16];                 // entry[4*w + a]
    int32_t tiles_m;
    int64_t tiles;
};

template <typename E>
__device__ __forceinline__ int32_t widen(E v)
{
    return (int32_t)v;
}

template <int TM, int TN, typename E>
__global__ void __launch_bounds__(256)
lut65k_kernel(Lut65kArgs a)
{
    constexpr int LM = 16, LN = 16, BM = LM * TM, BN = LN * TN;
    extern __shared__ __align__(16) unsigned char smem[];
    E *s_table = (E *)smem;                                                    // [257][256]
    int16_t *s_pair = (int16_t *)(smem + TABLE_ROWS * 256 * sizeof(E));        // [16 weight nibbles][16 activation nibbles]
    uint32_t *s_w = (uint32_t *)(s_pair + 256);                               // [KB/4 words][BM rows]
    uint16_t *s_a = (uint16_t *)(s_w + (KB / 4) * BM);                        // [KB bytes][BN columns], 0..256

    const DgProblem &p = a.p;
    const int tid = threadIdx.x;
    const int ml = tid % LM, nl = tid / LM;                                   // channel-fastest lanes

    // ---- build the table once per workgroup -----------------------------------------------------
    {
        // two code pairs: nibble x nibble -> sum of two products
        const int wn = tid >> 4, an = tid & 15;
        s_pair[tid] = (int16_t)(a.entry[4 * (wn & 3) + (an & 3)] + a.entry[4 * (wn >> 2) + (an >> 2)]);
        __syncthreads();
        // entry(a, w) = pair[w_lo][a_lo] + pair[w_hi][a_hi]; each lane fills four consecutive w at a time
        for (int idx4 = tid; idx4 < 256 * 64; idx4 += 256) {
            const int ab = idx4 >> 6, wb0 = (idx4 & 63) * 4;
            const int a_lo = ab & 15, a_hi = ab >> 4;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int wb = wb0 + j;
                s_table[(ab << 8) | wb] = (E)(s_pair[((wb & 15) << 4) | a_lo] + s_pair[((wb >> 4) << 4) | a_hi]);
            }
        }
        s_table[(256 << 8) | tid] = (E)0;
        __syncthreads();
    }

    const int cq = p.Cin / 4;
    const int stages = p.K / (4 * KB);
    const int stages_per_tap = p.Cin / (4 * KB);

    for (int64_t tile = blockIdx.x; tile < a.tiles; tile += gridDim.x) {
        const int m_base = (int)(tile % a.tiles_m) * BM;
        const int n_base = (int)(tile / a.tiles_m) * BN;

        // loader roles: lanes 0..BM-1 bring one weight row each, lanes BM..BM+BN-1 one output pixel each
        const bool w_loader = tid < BM, a_loader = tid >= BM && tid < BM + BN;
        const uint8_t *w_src = nullptr;
        int ih0 = 0, iw0 = 0;
        int64_t pix0 = 0;
        bool n_ok = false;
        if (w_loader) {
            int m = m_base + tid;
            if (m >= p.M) m = p.M - 1;
            w_src = p.Wp + (int64_t)m * (p.K / 4);
        } else if (a_loader) {
            const int n = n_base + (tid - BM);
            n_ok = n < p.N;
            const int nn = n_ok ? n : 0;
            const int ow = nn % p.OW, oh = (nn / p.OW) % p.OH, b = nn / (p.OW * p.OH);
            ih0 = oh * p.sh - p.ph;
            iw0 = ow * p.sw - p.pw;
            pix0 = (int64_t)b * p.H * p.W;
        }

        int32_t acc[TM][TN];
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) acc[i][j] = 0;

        for (int s = 0; s < stages; ++s) {
            __syncthreads();                                   // the previous stage's tiles have been consumed
            if (w_loader) {
                const uint4 v = *(const uint4 *)(w_src + (int64_t)s * KB);
                s_w[0 * BM + tid] = v.x;
                s_w[1 * BM + tid] = v.y;
                s_w[2 * BM + tid] = v.z;
                s_w[3 * BM + tid] = v.w;
            } else if (a_loader) {
                const int tap = s / stages_per_tap, ci_b = (s % stages_per_tap) * KB;
                const int kh = tap / p.KW, kw = tap % p.KW;
                const int ih = ih0 + kh, iw = iw0 + kw;
                const bool ok = n_ok && ih >= 0 && ih < p.H && iw >= 0 && iw < p.W;
                uint4 v = make_uint4(0, 0, 0, 0);
                if (ok) v = *(const uint4 *)(p.Xp + (pix0 + (int64_t)ih * p.W + iw) * cq + ci_b);
                const uint32_t words[4] = {v.x, v.y, v.z, v.w};
                const int col = tid - BM;
#pragma unroll
                for (int b = 0; b < KB; ++b)
                    s_a[b * BN + col] = ok ? (uint16_t)((words[b / 4] >> (8 * (b % 4))) & 0xFFu) : (uint16_t)256;
            }
            __syncthreads();

#pragma unroll
            for (int d = 0; d < KB / 4; ++d) {
                uint32_t ww[TM];
#pragma unroll
                for (int i = 0; i < TM; ++i) ww[i] = s_w[d * BM + ml * TM + i];
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    uint32_t av[TN];
#pragma unroll
                    for (int j = 0; j < TN; ++j) av[j] = s_a[(4 * d + b) * BN + nl * TN + j];
#pragma unroll
                    for (int i = 0; i < TM; ++i) {
                        const uint32_t wb = (ww[i] >> (8 * b)) & 0xFFu;
#pragma unroll
                        for (int j = 0; j < TN; ++j) acc[i][j] += widen(s_table[(av[j] << 8) | wb]);
                    }
                }
            }
        }

        // epilogue
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int n = n_base + nl * TN + j;
            if (n >= p.N) continue;
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const int m = m_base + ml * TM + i;
                if (m >= p.M) continue;
                const int64_t o = (int64_t)m * p.stride_cm + (int64_t)n * p.stride_cn;
                if (p.scale)
                    p.Cf[o] = (float)acc[i][j] * p.scale[m];
                else
                    p.C[o] = acc[i][j];
            }
        }
    }
}

template <int TM, int TN, typename E>
dg_status launch(const Lut65kArgs &a, hipStream_t stream)
{
    constexpr int BM = 16 * TM, BN = 16 * TN;
    const size_t lds = TABLE_ROWS * 256 * sizeof(E) + 512 + (KB / 4) * BM * 4 + KB * BN * 2;
    auto kernel = lut65k_kernel<TM, TN, E>;
    static bool ready = false;
    if (!ready) {
        hipError_t e = hipFuncSetAttribute((const void *)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return dg_fail(DG_ERR_HIP, "lut65k kernel LDS attribute: %s", hipGetErrorString(e));
        ready = true;
    }
    // persistent workgroups: as many as stay resident (two per compute unit with the int8 table, one with int16)
    const int64_t resident = 256 * (sizeof(E) == 1 ? 2 : 1);
    const int64_t blocks = a.tiles < resident ? a.tiles : resident;
    hipLaunchKernelGGL(kernel, dim3((unsigned)blocks), dim3(256), lds, stream, a);
    return dg_check_launch("lut65k_kernel");
}

}   // namespace

bool dg_lut65k_supports(const dg_lut *lut, const DgProblem &p)
{
    if (4 * lut->max_entry > 32767 || 4 * lut->min_entry < -32768) return false;   // four products must fit int16
    if (p.Cin % (4 * KB) != 0) return false;                  // a 16-byte stage stays inside one filter tap
    if ((uintptr_t)p.Wp % 16 != 0 || (uintptr_t)p.Xp % 16 != 0) return false;
    return true;
}

dg_status dg_launch_lut65k(const dg_lut *lut, const DgProblem &p, hipStream_t stream)
{
    Lut65kArgs a;
    a.p = p;
    for (int i = 0; i < 16; ++i) a.entry[i] = lut->entry[i];
    constexpr int TM = 4, TN = 4;
    a.tiles_m = (p.M + 16 * TM - 1) / (16 * TM);
    a.tiles = (int64_t)a.tiles_m * (((int64_t)p.N + 16 * TN - 1) / (16 * TN));
    // four products per entry: int8 entries only when every such sum fits (Sec. 3.2 assumes it; here it is checked)
    const bool fits8 = 4 * lut->max_entry <= 127 && 4 * lut->min_entry >= -128;
    if (fits8) return launch<TM, TN, int8_t>(a, stream);
    return launch<TM, TN, int16_t>(a, stream);
}
