// Packing kernels: 2-bit codes, one per byte, to four per byte (Sec. 3.1: packing by shift and OR), and the fused
// quantise + pack of fp32 activations (Sec. 2.1, Eq. 1, then the same packing).
// Code k of a row lands in byte k/4, bits [2*(k%4)+1 : 2*(k%4)].  Rows are contiguous and K % 4 == 0,
// so the whole matrix is one flat run of rows*K codes.  HBM-bound: 1 byte read and 1/4 byte written
// per code; each lane moves 16 codes per 128-bit load and writes one 32-bit word.
#include "dg_common.h"
#include "dg_quant.h"

namespace {

// Four codes held in the four bytes of `d` (low bits of each byte) -> one packed byte.
__device__ __forceinline__ uint32_t pack4(uint32_t d)
{
    uint32_t x = d & 0x03030303u;
    x |= x >> 6;                                  // bytes 0 and 2 now hold two codes each, in bits 3:0
    return (x & 0xFu) | ((x >> 12) & 0xF0u);
}

__global__ void __launch_bounds__(256)
pack_vec16_kernel(const uint4 *__restrict__ codes, uint32_t *__restrict__ packed, int64_t groups16)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; g < groups16; g += stride) {
        const uint4 v = codes[g];
        packed[g] = pack4(v.x) | (pack4(v.y) << 8) | (pack4(v.z) << 16) | (pack4(v.w) << 24);
    }
}

// Large inputs: U independent 128-bit loads per lane are issued before the first is used (more bytes in flight per
// wavefront), each still coalesced across the workgroup.  `groups16` is a multiple of 256*U here.
template <int U>
__global__ void __launch_bounds__(256)
pack_vec16_unrolled_kernel(const uint4 *__restrict__ codes, uint32_t *__restrict__ packed, int64_t groups16)
{
    const int64_t stride = (int64_t)gridDim.x * (256 * U);
    for (int64_t base = (int64_t)blockIdx.x * (256 * U) + threadIdx.x; base < groups16; base += stride) {
        uint4 v[U];
#pragma unroll
        for (int j = 0; j < U; ++j) v[j] = codes[base + 256 * j];
#pragma unroll
        for (int j = 0; j < U; ++j)
            packed[base + 256 * j] = pack4(v[j].x) | (pack4(v[j].y) << 8) | (pack4(v[j].z) << 16) | (pack4(v[j].w) << 24);
    }
}

// Only the pixels a 1x1 convolution with a stride reads: output pixel (b, oh, ow) of the packed tensor [B][OH][OW][Cin/4]
// is input pixel (b, oh * sh, ow * sw).  `groups` 16-code groups per pixel, fewer than 2^31 in all; a lane moves one group.
__global__ void __launch_bounds__(256)
pack_strided_pixels_kernel(const uint4 *__restrict__ codes, uint32_t *__restrict__ packed, uint32_t groups16, uint32_t groups,
                           DgFastDiv div_groups, DgFastDiv div_ow, DgFastDiv div_oh, int32_t OH, int32_t OW, int32_t H, int32_t W,
                           int32_t sh, int32_t sw)
{
    const uint32_t stride = gridDim.x * blockDim.x;
    for (uint32_t g = blockIdx.x * blockDim.x + threadIdx.x; g < groups16; g += stride) {
        const uint32_t pixel = dg_fdiv(g, div_groups), row = dg_fdiv(pixel, div_ow), b = dg_fdiv(row, div_oh);
        const uint32_t within = g - pixel * groups, ow = pixel - row * (uint32_t)OW, oh = row - b * (uint32_t)OH;
        const uint4 v = codes[(((int64_t)b * H + (int64_t)oh * sh) * W + (int64_t)ow * sw) * groups + within];
        packed[g] = pack4(v.x) | (pack4(v.y) << 8) | (pack4(v.z) << 16) | (pack4(v.w) << 24);
    }
}

// Any alignment, any count that is a multiple of 4: one packed byte per lane per step.
__global__ void __launch_bounds__(256)
pack_bytes_kernel(const uint8_t *__restrict__ codes, uint8_t *__restrict__ packed, int64_t first_group,
                  int64_t groups4)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t g = first_group + (int64_t)blockIdx.x * blockDim.x + threadIdx.x; g < groups4; g += stride) {
        const uint8_t *c = codes + 4 * g;
        packed[g] = (uint8_t)((c[0] & 3) | ((c[1] & 3) << 2) | ((c[2] & 3) << 4) | ((c[3] & 3) << 6));
    }
}

// 16 values per lane: four 128-bit loads, one 32-bit store (4.06 bytes of HBM traffic per code).
__global__ void __launch_bounds__(256)
quantize_pack_vec16_kernel(const float4 *__restrict__ x, uint32_t *__restrict__ packed, int64_t groups16, float s,
                           float z, int lo)
{
    const float lo_f = (float)lo, hi_f = (float)(lo + 3);
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; g < groups16; g += stride) {
        uint32_t word = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float4 v = x[4 * g + j];
            const uint32_t byte = dg_quantize_code(v.x, s, z, lo_f, hi_f, lo) | (dg_quantize_code(v.y, s, z, lo_f, hi_f, lo) << 2) |
                                  (dg_quantize_code(v.z, s, z, lo_f, hi_f, lo) << 4) |
                                  (dg_quantize_code(v.w, s, z, lo_f, hi_f, lo) << 6);
            word |= byte << (8 * j);
        }
        packed[g] = word;
    }
}

__global__ void __launch_bounds__(256)
quantize_pack_bytes_kernel(const float *__restrict__ x, uint8_t *__restrict__ packed, int64_t first_group,
                           int64_t groups4, float s, float z, int lo)
{
    const float lo_f = (float)lo, hi_f = (float)(lo + 3);
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t g = first_group + (int64_t)blockIdx.x * blockDim.x + threadIdx.x; g < groups4; g += stride) {
        const float *v = x + 4 * g;
        packed[g] = (uint8_t)(dg_quantize_code(v[0], s, z, lo_f, hi_f, lo) | (dg_quantize_code(v[1], s, z, lo_f, hi_f, lo) << 2) |
                              (dg_quantize_code(v[2], s, z, lo_f, hi_f, lo) << 4) |
                              (dg_quantize_code(v[3], s, z, lo_f, hi_f, lo) << 6));
    }
}

}   // namespace

dg_status dg_launch_quantize_pack(const float *x, int64_t rows, int64_t K, float scale, float zero_point,
                                  int32_t lo, uint8_t *packed, hipStream_t stream)
{
    const int64_t total = rows * K, groups4 = total / 4;
    int64_t done4 = 0;
    if ((uintptr_t)x % 16 == 0 && (uintptr_t)packed % 4 == 0 && total >= 16) {
        const int64_t groups16 = total / 16;
        int64_t blocks = (groups16 + 255) / 256;
        if (blocks > 256 * 32) blocks = 256 * 32;
        hipLaunchKernelGGL(quantize_pack_vec16_kernel, dim3((unsigned)blocks), dim3(256), 0, stream,
                           (const float4 *)x, (uint32_t *)packed, groups16, scale, zero_point, lo);
        dg_status s = dg_check_launch("quantize_pack_vec16_kernel");
        if (s != DG_OK) return s;
        done4 = groups16 * 4;
    }
    if (done4 < groups4) {
        int64_t blocks = (groups4 - done4 + 255) / 256;
        if (blocks > 256 * 32) blocks = 256 * 32;
        hipLaunchKernelGGL(quantize_pack_bytes_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, x, packed,
                           done4, groups4, scale, zero_point, lo);
        return dg_check_launch("quantize_pack_bytes_kernel");
    }
    return DG_OK;
}

namespace {
// 3- and 4-bit codes: two per byte, each in a 4-bit slot (the layout the paper leaves open for Sec. 3.3).
__global__ void __launch_bounds__(256)
pack_slots4_kernel(const uint8_t *__restrict__ codes, uint8_t *__restrict__ packed, int64_t pairs, uint32_t mask)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; g < pairs; g += stride)
        packed[g] = (uint8_t)((codes[2 * g] & mask) | ((codes[2 * g + 1] & mask) << 4));
}
}   // namespace

dg_status dg_launch_pack(const uint8_t *codes, int64_t rows, int64_t K, int bits, uint8_t *packed, hipStream_t stream)
{
    if (bits != 2) {
        const int64_t pairs = rows * K / 2;
        int64_t blocks = (pairs + 255) / 256;
        if (blocks > 256 * 32) blocks = 256 * 32;
        hipLaunchKernelGGL(pack_slots4_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, codes, packed, pairs,
                           (1u << bits) - 1u);
        return dg_check_launch("pack_slots4_kernel");
    }
    const int64_t total = rows * K;           // multiple of 4
    const int64_t groups4 = total / 4;
    int64_t done4 = 0;
    const bool aligned = ((uintptr_t)codes % 16 == 0) && ((uintptr_t)packed % 4 == 0);
    if (aligned && total >= 16) {
        const int64_t groups16 = total / 16;
        constexpr int U = 4;
        const int64_t big = groups16 >= 256 * 1024 ? groups16 / (256 * U) * (256 * U) : 0;   // from 4 Mi codes up
        if (big > 0) {
            int64_t blocks = big / (256 * U);
            if (blocks > 256 * 32) blocks = 256 * 32;
            hipLaunchKernelGGL(pack_vec16_unrolled_kernel<U>, dim3((unsigned)blocks), dim3(256), 0, stream,
                               (const uint4 *)codes, (uint32_t *)packed, big);
            dg_status s = dg_check_launch("pack_vec16_unrolled_kernel");
            if (s != DG_OK) return s;
        }
        if (big < groups16) {
            int64_t blocks = (groups16 - big + 255) / 256;
            if (blocks > 256 * 32) blocks = 256 * 32;   // grid-stride beyond 32 workgroups per CU
            hipLaunchKernelGGL(pack_vec16_kernel, dim3((unsigned)blocks), dim3(256), 0, stream,
                               (const uint4 *)codes + big, (uint32_t *)packed + big, groups16 - big);
            dg_status s = dg_check_launch("pack_vec16_kernel");
            if (s != DG_OK) return s;
        }
        done4 = groups16 * 4;
    }
    if (done4 < groups4) {
        int64_t blocks = (groups4 - done4 + 255) / 256;
        if (blocks > 256 * 32) blocks = 256 * 32;
        hipLaunchKernelGGL(pack_bytes_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, codes, packed,
                           done4, groups4);
        return dg_check_launch("pack_bytes_kernel");
    }
    return DG_OK;
}

dg_status dg_launch_pack_strided_pixels(const uint8_t *codes, int64_t B, int32_t H, int32_t W, int32_t OH, int32_t OW, int32_t sh,
                                        int32_t sw, int32_t Cin, uint8_t *packed, hipStream_t stream)
{
    const int64_t groups16 = B * OH * OW * (Cin / 16);
    if (groups16 >= ((int64_t)1 << 31)) return dg_fail(DG_ERR_UNSUPPORTED, "pack_strided_pixels_kernel: 2^35 codes or more");
    int64_t blocks = (groups16 + 255) / 256;
    if (blocks > 256 * 32) blocks = 256 * 32;
    if (blocks < 1) return DG_OK;
    hipLaunchKernelGGL(pack_strided_pixels_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, (const uint4 *)codes,
                       (uint32_t *)packed, (uint32_t)groups16, (uint32_t)(Cin / 16), dg_make_div((uint32_t)(Cin / 16)),
                       dg_make_div((uint32_t)OW), dg_make_div((uint32_t)OH), OH, OW, H, W, sh, sw);
    return dg_check_launch("pack_strided_pixels_kernel");
}

namespace {
// Dequantise: out = float(acc) * scale[channel].  HBM-bound: 4 bytes read and 4 written per element; 128-bit accesses
// when the row length and the pointers allow (then a lane's four elements are four consecutive channels of one row).
template <bool VEC>
__global__ void __launch_bounds__(256)
dequantize_kernel(const int32_t *acc, const float *__restrict__ scale, float *out, int64_t total, int32_t C)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    if (VEC) {
        const int64_t groups = total / 4;
        for (int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; g < groups; g += stride) {
            const int4 v = ((const int4 *)acc)[g];
            const int c = (int)((4 * g) % C);
            const float4 s = *(const float4 *)(scale + c);
            float4 o;
            o.x = __fmul_rn((float)v.x, s.x), o.y = __fmul_rn((float)v.y, s.y);
            o.z = __fmul_rn((float)v.z, s.z), o.w = __fmul_rn((float)v.w, s.w);
            ((float4 *)out)[g] = o;
        }
    } else {
        for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += stride)
            out[i] = __fmul_rn((float)acc[i], scale[i % C]);
    }
}
}   // namespace

dg_status dg_launch_dequantize(const int32_t *acc, int64_t rows, int64_t C, const float *scale, float *out,
                               hipStream_t stream)
{
    const int64_t total = rows * C;
    const bool vec = C % 4 == 0 && (uintptr_t)acc % 16 == 0 && (uintptr_t)out % 16 == 0 && (uintptr_t)scale % 16 == 0;
    int64_t blocks = ((vec ? total / 4 : total) + 255) / 256;
    if (blocks > 256 * 32) blocks = 256 * 32;
    if (vec)
        hipLaunchKernelGGL(dequantize_kernel<true>, dim3((unsigned)blocks), dim3(256), 0, stream, acc, scale, out, total,
                           (int32_t)C);
    else
        hipLaunchKernelGGL(dequantize_kernel<false>, dim3((unsigned)blocks), dim3(256), 0, stream, acc, scale, out, total,
                           (int32_t)C);
    return dg_check_launch("dequantize_kernel");
}
