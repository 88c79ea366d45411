// The plain table kernel: the 16-entry table sits in LDS and every product is one indexed LDS read.
// This is Algorithm 1 of the paper mapped one output per lane: for each packed byte pair, for the
// four 2-bit slots, index = (weight code << 2) | activation code, fetch, add (int32).
// It accepts every shape the library accepts (any K % 4 == 0, any stride / pad, any table) and is
// the fallback for shapes the tuned kernels do not cover, and the "table in LDS" side of the
// register-vs-LDS comparison.
#include "dg_common.h"

namespace {

template <typename WordT>
__device__ __forceinline__ int32_t lookup_run(const int32_t *lut, const uint8_t *w, const uint8_t *x, int bytes)
{
    // `bytes` packed bytes of one filter tap: both runs are contiguous (channel-fastest layouts)
    int32_t acc = 0;
    constexpr int WB = sizeof(WordT);
    const WordT *w4 = (const WordT *)w;
    const WordT *x4 = (const WordT *)x;
    for (int j = 0; j < bytes / WB; ++j) {
        const uint32_t vw = w4[j], va = x4[j];
#pragma unroll
        for (int i = 0; i < 4 * WB; ++i) {
            const int shift = 2 * i;
            const uint32_t indx = (((vw >> shift) & 3u) << 2) | ((va >> shift) & 3u);
            acc += lut[indx];
        }
    }
    return acc;
}

template <typename WordT>
__global__ void __launch_bounds__(256)
lds_lut_kernel(DgProblem p, DgTable16 table)
{
    __shared__ int32_t lut[16];
    if (threadIdx.x < 16) lut[threadIdx.x] = table.e[threadIdx.x];
    __syncthreads();

    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= (int64_t)p.M * p.N) return;
    const int m = (int)(t % p.M);      // channel fastest: NHWC stores coalesce
    const int n = (int)(t / p.M);
    const int ow = n % p.OW;
    const int oh = (n / p.OW) % p.OH;
    const int b = n / (p.OW * p.OH);

    const int tap_bytes = p.Cin / 4;
    const uint8_t *wrow = p.Wp + (int64_t)m * (p.K / 4);
    int32_t acc = 0;
    for (int kh = 0; kh < p.KH; ++kh) {
        const int ih = oh * p.sh - p.ph + kh;
        if (ih < 0 || ih >= p.H) continue;            // a tap outside the image adds nothing
        for (int kw = 0; kw < p.KW; ++kw) {
            const int iw = ow * p.sw - p.pw + kw;
            if (iw < 0 || iw >= p.W) continue;
            const uint8_t *x = p.Xp + (((int64_t)b * p.H + ih) * p.W + iw) * tap_bytes;
            const uint8_t *w = wrow + (int64_t)(kh * p.KW + kw) * tap_bytes;
            acc += lookup_run<WordT>(lut, w, x, tap_bytes);
        }
    }
    const int64_t o = (int64_t)m * p.stride_cm + (int64_t)n * p.stride_cn;
    if (p.scale)
        p.Cf[o] = (float)acc * p.scale[m];
    else
        p.C[o] = acc;
}

}   // namespace

dg_status dg_launch_lds(const dg_lut *lut, const DgProblem &p, hipStream_t stream)
{
    DgTable16 t;
    for (int i = 0; i < 16; ++i) t.e[i] = lut->entry[i];
    const int64_t total = (int64_t)p.M * p.N;
    const int64_t blocks = (total + 255) / 256;
    if (blocks > INT32_MAX) return dg_fail(DG_ERR_UNSUPPORTED, "lds kernel: M*N too large for one grid");
    // 32-bit reads need every tap run to start on a 4-byte boundary
    const bool words = (p.Cin % 16 == 0) && ((uintptr_t)p.Wp % 4 == 0) && ((uintptr_t)p.Xp % 4 == 0);
    if (words)
        hipLaunchKernelGGL(lds_lut_kernel<uint32_t>, dim3((unsigned)blocks), dim3(256), 0, stream, p, t);
    else
        hipLaunchKernelGGL(lds_lut_kernel<uint8_t>, dim3((unsigned)blocks), dim3(256), 0, stream, p, t);
    return dg_check_launch("lds_lut_kernel");
}
