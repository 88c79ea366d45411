// The plain table kernel: the table sits in LDS and every product is one indexed LDS read.
// This is Algorithm 1 of the paper mapped one output per lane: for each packed byte pair, for each code slot,
// index = (weight code << bits) | activation code, fetch, add (int32).
// It accepts every shape the library accepts (any K, any stride / pad, any table) and every code width: the
// paper's 2-bit codes (16 entries) and the 3- and 4-bit extension it describes in Sec. 3.3 / Table 2 (64 and 256
// entries; two codes per byte in 4-bit slots).  It is the fallback for shapes the tuned kernels do not cover, and
// the "16-entry table in LDS" side of the register-versus-LDS comparison.
#include <cstring>

#include "dg_common.h"

namespace {

// The table travels in the kernel arguments (512 bytes at most): no device allocation is needed for it.
struct Table256 {
    int16_t e[256];
};

template <int BITS, typename WordT>
__device__ __forceinline__ int32_t lookup_run(const int32_t *lut, const uint8_t *w, const uint8_t *x, int bytes)
{
    // `bytes` packed bytes of one filter tap: both runs are contiguous (channel-fastest layouts)
    constexpr int SLOT = BITS == 2 ? 2 : 4;                  // bits per code slot
    constexpr uint32_t MASK = (1u << BITS) - 1u;
    constexpr int WB = sizeof(WordT);
    constexpr int SLOTS = 8 * WB / SLOT;                     // codes per loaded word
    const WordT *wwords = (const WordT *)w, *xwords = (const WordT *)x;
    int32_t acc = 0;
    for (int j = 0; j < bytes / WB; ++j) {
        // walk the two words from the low slot up: the low fields of the shifted words are the current code pair
        uint32_t wrest = wwords[j], xrest = xwords[j];
#pragma unroll
        for (int slot = 0; slot < SLOTS; ++slot) {
            acc += lut[((wrest & MASK) << BITS) | (xrest & MASK)];     // table address: weight code, then activation code
            wrest >>= SLOT;
            xrest >>= SLOT;
        }
    }
    return acc;
}

template <int BITS, typename WordT>
__global__ void __launch_bounds__(256)
lds_lut_kernel(DgProblem p, Table256 table)
{
    constexpr int ENTRIES = 1 << (2 * BITS);
    constexpr int PER_BYTE = BITS == 2 ? 4 : 2;
    __shared__ int32_t lut[ENTRIES];
    for (int i = threadIdx.x; i < ENTRIES; i += blockDim.x) lut[i] = table.e[i];
    __syncthreads();

    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= (int64_t)p.M * p.N) return;
    const int m = (int)(t % p.M);      // channel fastest: NHWC stores coalesce
    const int n = (int)(t / p.M);
    const int ow = n % p.OW;
    const int oh = (n / p.OW) % p.OH;
    const int b = n / (p.OW * p.OH);

    const int tap_bytes = p.Cin / PER_BYTE;
    const uint8_t *wrow = p.Wp + (int64_t)m * (p.K / PER_BYTE);
    int32_t acc = 0;
    for (int kh = 0; kh < p.KH; ++kh) {
        const int ih = oh * p.sh - p.ph + kh;
        if (ih < 0 || ih >= p.H) continue;            // a tap outside the image adds nothing
        for (int kw = 0; kw < p.KW; ++kw) {
            const int iw = ow * p.sw - p.pw + kw;
            if (iw < 0 || iw >= p.W) continue;
            const uint8_t *x = p.Xp + (((int64_t)b * p.H + ih) * p.W + iw) * tap_bytes;
            const uint8_t *w = wrow + (int64_t)(kh * p.KW + kw) * tap_bytes;
            acc += lookup_run<BITS, WordT>(lut, w, x, tap_bytes);
        }
    }
    const int64_t o = (int64_t)m * p.stride_cm + (int64_t)n * p.stride_cn;
    if (p.scale)
        p.Cf[o] = (float)acc * p.scale[m];
    else
        p.C[o] = acc;
}

// binary32 table: the sum is one binary32 addition per reduction position, in ascending k, starting from +0
// (the compiler does not re-associate floating-point additions, so the source order is the arithmetic order).
struct TableF32 {
    float e[16];
};

template <typename WordT>
__global__ void __launch_bounds__(256)
lds_lut_f32_kernel(DgProblem p, TableF32 table)
{
    __shared__ float lut[16];
    if (threadIdx.x < 16) lut[threadIdx.x] = table.e[threadIdx.x];
    __syncthreads();

    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= (int64_t)p.M * p.N) return;
    const int m = (int)(t % p.M);
    const int n = (int)(t / p.M);
    const int ow = n % p.OW;
    const int oh = (n / p.OW) % p.OH;
    const int b = n / (p.OW * p.OH);

    constexpr int WB = sizeof(WordT);
    const int tap_bytes = p.Cin / 4;
    const uint8_t *wrow = p.Wp + (int64_t)m * (p.K / 4);
    float acc = 0.0f;
    for (int kh = 0; kh < p.KH; ++kh) {
        const int ih = oh * p.sh - p.ph + kh;
        if (ih < 0 || ih >= p.H) continue;
        for (int kw = 0; kw < p.KW; ++kw) {
            const int iw = ow * p.sw - p.pw + kw;
            if (iw < 0 || iw >= p.W) continue;
            const WordT *x = (const WordT *)(p.Xp + (((int64_t)b * p.H + ih) * p.W + iw) * tap_bytes);
            const WordT *w = (const WordT *)(wrow + (int64_t)(kh * p.KW + kw) * tap_bytes);
            for (int j = 0; j < tap_bytes / WB; ++j) {
                const uint32_t vw = w[j], va = x[j];
#pragma unroll
                for (int i = 0; i < 4 * WB; ++i) {
                    const int shift = 2 * i;
                    acc = __fadd_rn(acc, lut[(((vw >> shift) & 3u) << 2) | ((va >> shift) & 3u)]);
                }
            }
        }
    }
    const int64_t o = (int64_t)m * p.stride_cm + (int64_t)n * p.stride_cn;
    p.Cf[o] = p.scale ? __fmul_rn(acc, p.scale[m]) : acc;
}

template <int BITS>
void launch_bits(const DgProblem &p, const Table256 &t, bool words, unsigned blocks, hipStream_t stream)
{
    if (words)
        hipLaunchKernelGGL((lds_lut_kernel<BITS, uint32_t>), dim3(blocks), dim3(256), 0, stream, p, t);
    else
        hipLaunchKernelGGL((lds_lut_kernel<BITS, uint8_t>), dim3(blocks), dim3(256), 0, stream, p, t);
}

}   // namespace

dg_status dg_launch_lds(const dg_lut *lut, const DgProblem &p, hipStream_t stream)
{
    Table256 t;
    memset(&t, 0, sizeof(t));
    const int entries = 1 << (2 * lut->bits);
    for (int i = 0; i < entries; ++i) t.e[i] = lut->entry[i];
    const int64_t total = (int64_t)p.M * p.N;
    const int64_t blocks = (total + 255) / 256;
    if (blocks > INT32_MAX) return dg_fail(DG_ERR_UNSUPPORTED, "lds kernel: M*N too large for one grid");
    // 32-bit reads need every tap run to start on a 4-byte boundary
    const int per_byte = lut->bits == 2 ? 4 : 2;
    const bool words = (p.Cin % (4 * per_byte) == 0) && ((uintptr_t)p.Wp % 4 == 0) && ((uintptr_t)p.Xp % 4 == 0);
    switch (lut->bits) {
    case 2: launch_bits<2>(p, t, words, (unsigned)blocks, stream); break;
    case 3: launch_bits<3>(p, t, words, (unsigned)blocks, stream); break;
    default: launch_bits<4>(p, t, words, (unsigned)blocks, stream); break;
    }
    return dg_check_launch("lds_lut_kernel");
}

dg_status dg_launch_lds_f32(const dg_lut *lut, const DgProblem &p, hipStream_t stream)
{
    TableF32 t;
    for (int i = 0; i < 16; ++i) t.e[i] = lut->fentry[i];
    const int64_t blocks = ((int64_t)p.M * p.N + 255) / 256;
    if (blocks > INT32_MAX) return dg_fail(DG_ERR_UNSUPPORTED, "lds kernel: M*N too large for one grid");
    const bool words = (p.Cin % 16 == 0) && ((uintptr_t)p.Wp % 4 == 0) && ((uintptr_t)p.Xp % 4 == 0);
    if (words)
        hipLaunchKernelGGL(lds_lut_f32_kernel<uint32_t>, dim3((unsigned)blocks), dim3(256), 0, stream, p, t);
    else
        hipLaunchKernelGGL(lds_lut_f32_kernel<uint8_t>, dim3((unsigned)blocks), dim3(256), 0, stream, p, t);
    return dg_check_launch("lds_lut_f32_kernel");
}
