// Packing kernel: 2-bit codes, one per byte, to four per byte (Sec. 3.1: packing by shift and OR).
// Code k of a row lands in byte k/4, bits [2*(k%4)+1 : 2*(k%4)].  Rows are contiguous and K % 4 == 0,
// so the whole matrix is one flat run of rows*K codes.  HBM-bound: 1 byte read and 1/4 byte written
// per code; each lane moves 16 codes per 128-bit load and writes one 32-bit word.
#include "dg_common.h"

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

}   // namespace

dg_status dg_launch_pack(const uint8_t *codes, int64_t rows, int64_t K, uint8_t *packed, hipStream_t stream)
{
    const int64_t total = rows * K;           // multiple of 4
    const int64_t groups4 = total / 4;
    int64_t done4 = 0;
    const bool aligned = ((uintptr_t)codes % 16 == 0) && ((uintptr_t)packed % 4 == 0);
    if (aligned && total >= 16) {
        const int64_t groups16 = total / 16;
        int64_t blocks = (groups16 + 255) / 256;
        if (blocks > 256 * 32) blocks = 256 * 32;   // grid-stride beyond 32 workgroups per CU
        hipLaunchKernelGGL(pack_vec16_kernel, dim3((unsigned)blocks), dim3(256), 0, stream,
                           (const uint4 *)codes, (uint32_t *)packed, groups16);
        dg_status s = dg_check_launch("pack_vec16_kernel");
        if (s != DG_OK) return s;
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
