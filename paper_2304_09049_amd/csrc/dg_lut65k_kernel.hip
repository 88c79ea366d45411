// LUT-65k on gfx950 (Sec. 3 "LUT-65k"): a table with one entry per (weight byte, activation byte), each entry the
// dot product of the four 2-bit weight codes with the four 2-bit activation codes packed in those bytes.  The index
// is the two packed bytes side by side, so no 2-bit field is ever extracted in the main loop: one table read per
// FOUR products.  The paper keeps the 64 KB table in the CPU's L2 cache; here it lives in LDS (160 KB per compute
// unit on CDNA4), built once per workgroup, and workgroups are persistent (their wavefronts loop over output tiles).
//
// Table layout: entry[(a << 8) | w], a = activation byte, w = weight byte.  A filter tap outside the image is the same
// for every lane of a wavefront (see below) and is skipped.  Entries are int8 when four products always fit (the paper's assumption, here checked), else int16.
// Accumulation is int32 and exact.
//
// A random byte read by 64 lanes from a 64 KB table is a bank-conflict machine, so the reads are arranged to have
// none: the 64 lanes of a wavefront hold 64 different weight rows m and ALL work on the same output pixel n at a time.
// The activation byte of a read is then the same in every lane -- it lives in a scalar register, and so does the base
// address of its table row -- and the lanes' weight bytes pick entries inside that one 256-byte row, which spans each
// LDS bank exactly once.  Per read: one scalar field extract and shift, one vector add (weight byte + row base), one
// LDS read of the entry's dword, one bit-field extract, one add.  A wavefront owns a tile of 64 rows x TN pixels and keeps TN sums per lane.
//
// This kernel exists for the register-versus-LDS comparison the method invites; DG_KERNEL_AUTO never selects it.
#include "dg_common.h"

namespace {

constexpr int KB = 16;                 // packed bytes of K per stage (64 codes)
constexpr int TABLE_ROWS = 256;        // one row per activation byte
constexpr int TN = 8;                  // output pixels per wavefront tile
constexpr int WAVES = 8;               // wavefronts per workgroup

struct Lut65kArgs {
    DgProblem p;
    int16_t entry[16];                 // entry[4*w + a]
    int32_t tiles_m;
    int64_t tiles;
};

// a wave-uniform value, held in a scalar register
__device__ __forceinline__ uint32_t uniform(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_readfirstlane((int)v);
}

template <typename E>
__global__ void __launch_bounds__(64 * WAVES)
lut65k_kernel(Lut65kArgs a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    E *s_table = (E *)smem;                                                    // [257][256]
    int16_t *s_pair = (int16_t *)(smem + TABLE_ROWS * 256 * sizeof(E));        // [16 weight nibbles][16 activation nibbles]

    const DgProblem &p = a.p;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = (int)uniform((uint32_t)(tid >> 6));

    // ---- build the table once per workgroup -----------------------------------------------------
    {
        // two code pairs: nibble x nibble -> sum of two products
        if (tid < 256) {
            const int wn = tid >> 4, an = tid & 15;
            s_pair[tid] = (int16_t)(a.entry[4 * (wn & 3) + (an & 3)] + a.entry[4 * (wn >> 2) + (an >> 2)]);
        }
        __syncthreads();
        // entry(a, w) = pair[w_lo][a_lo] + pair[w_hi][a_hi]; each lane fills four consecutive w at a time
        for (int idx4 = tid; idx4 < 256 * 64; idx4 += 64 * WAVES) {
            const int ab = idx4 >> 6, wb0 = (idx4 & 63) * 4;
            const int a_lo = ab & 15, a_hi = ab >> 4;
            int v[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int wb = wb0 + j;
                v[j] = s_pair[((wb & 15) << 4) | a_lo] + s_pair[((wb >> 4) << 4) | a_hi];
            }
            // whole dwords at a time (byte stores into one dword from four instructions would queue up)
            uint32_t *dst = (uint32_t *)(s_table + ((ab << 8) | wb0));
            if (sizeof(E) == 1) {
                dst[0] = (uint32_t)(v[0] & 255) | ((uint32_t)(v[1] & 255) << 8) | ((uint32_t)(v[2] & 255) << 16) | ((uint32_t)v[3] << 24);
            } else {
                dst[0] = (uint32_t)(v[0] & 65535) | ((uint32_t)v[1] << 16);
                dst[1] = (uint32_t)(v[2] & 65535) | ((uint32_t)v[3] << 16);
            }
        }
        __syncthreads();
    }

    const int cq = p.Cin / 4;
    const int stages = p.K / (4 * KB);
    const int stages_per_tap = p.Cin / (4 * KB);

    // wavefront tiles: 64 rows x TN pixels, the row tiles of one pixel tile side by side
    for (int64_t tile = (int64_t)blockIdx.x * WAVES + wave; tile < a.tiles; tile += (int64_t)gridDim.x * WAVES) {
        const int m_base = (int)(tile % a.tiles_m) * 64;
        const int n_base = (int)(tile / a.tiles_m) * TN;
        const int m = min(m_base + lane, p.M - 1);             // rows beyond M: a valid row, never stored
        const uint8_t *w_src = p.Wp + (int64_t)m * (p.K / 4);

        // the tile's pixels: image coordinates of their first tap (wave-uniform)
        int ih0[TN], iw0[TN], img[TN];
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int n = min(n_base + j, p.N - 1);            // pixels beyond N: a valid pixel, never stored
            const int ow = n % p.OW, oh = (n / p.OW) % p.OH, b = n / (p.OW * p.OH);
            ih0[j] = (int)uniform((uint32_t)(oh * p.sh - p.ph));
            iw0[j] = (int)uniform((uint32_t)(ow * p.sw - p.pw));
            img[j] = (int)uniform((uint32_t)b);
        }

        int32_t acc[TN];
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[j] = 0;

        uint4 wnext = *(const uint4 *)w_src;
        for (int s = 0; s < stages; ++s) {
            const uint4 wv = wnext;
            wnext = *(const uint4 *)(w_src + (int64_t)min(s + 1, stages - 1) * KB);       // (the last one re-reads, unused)
            const uint32_t ww[4] = {wv.x, wv.y, wv.z, wv.w};
            // this lane's 16 weight bytes as positions in a table row: the dword that holds the entry, and the entry's bit
            // offset in it (a whole-dword read of a 256-byte row touches every LDS bank once, and lanes that want the same
            // dword share it; byte reads of one dword by several lanes would queue up)
            const unsigned char *wdw[KB];                      // (the table's own address goes in here, once, not per read)
            uint32_t wsh[KB];
#pragma unroll
            for (int b = 0; b < KB; ++b) {
                const uint32_t wb = ((ww[b / 4] >> (8 * (b % 4))) & 0xFFu) * (uint32_t)sizeof(E);
                wdw[b] = smem + (wb & ~3u);
                wsh[b] = (wb & 3u) * 8u;
            }

            const int tap = s / stages_per_tap, ci_b = (s % stages_per_tap) * KB;
            const int kh = tap / p.KW, kw = tap % p.KW;
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int ih = ih0[j] + kh, iw = iw0[j] + kw;
                if (!((uint32_t)ih < (uint32_t)p.H && (uint32_t)iw < (uint32_t)p.W)) continue;      // (wave-uniform) adds 0
                // the pixel's 16 activation bytes, the same for every lane: a scalar load (the packed activations are
                // not written while this kernel runs, so the constant address space's rules hold for them)
                const int64_t off = (((int64_t)img[j] * p.H + ih) * p.W + iw) * cq + ci_b;
                const __attribute__((address_space(4))) uint32_t *ap =
                    (const __attribute__((address_space(4))) uint32_t *)(p.Xp + off);
                const uint32_t aw[4] = {ap[0], ap[1], ap[2], ap[3]};
#pragma unroll
                for (int b = 0; b < KB; ++b) {
                    const uint32_t row = ((aw[b / 4] >> (8 * (b % 4))) & 0xFFu) * (256u * (uint32_t)sizeof(E));     // scalar
                    const int32_t dw = *(const int32_t *)(wdw[b] + row);
                    acc[j] += __builtin_amdgcn_sbfe(dw, wsh[b], 8 * (int)sizeof(E));
                }
            }
        }

        // epilogue: lane = row m, its TN pixels
        if (m_base + lane < p.M) {
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int n = n_base + j;
                if (n >= p.N) continue;
                const int64_t o = (int64_t)m * p.stride_cm + (int64_t)n * p.stride_cn;
                if (p.scale)
                    p.Cf[o] = (float)acc[j] * p.scale[m];
                else
                    p.C[o] = acc[j];
            }
        }
    }
}

template <typename E>
dg_status launch(const Lut65kArgs &a, hipStream_t stream)
{
    const size_t lds = TABLE_ROWS * 256 * sizeof(E) + 512;
    auto kernel = lut65k_kernel<E>;
    static bool ready = false;
    if (!ready) {
        hipError_t e = hipFuncSetAttribute((const void *)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return dg_fail(DG_ERR_HIP, "lut65k kernel LDS attribute: %s", hipGetErrorString(e));
        ready = true;
    }
    // persistent workgroups: as many as stay resident (two per compute unit with the int8 table, one with int16)
    const int64_t resident = 256 * (sizeof(E) == 1 ? 2 : 1);
    const int64_t wanted = (a.tiles + WAVES - 1) / WAVES;
    const int64_t blocks = wanted < resident ? wanted : resident;
    hipLaunchKernelGGL(kernel, dim3((unsigned)blocks), dim3(64 * WAVES), lds, stream, a);
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
    a.tiles_m = (p.M + 63) / 64;
    a.tiles = (int64_t)a.tiles_m * (((int64_t)p.N + TN - 1) / TN);
    // four products per entry: int8 entries only when every such sum fits (Sec. 3.2 assumes it; here it is checked)
    const bool fits8 = 4 * lut->max_entry <= 127 && 4 * lut->min_entry >= -128;
    if (fits8) return launch<int8_t>(a, stream);
    return launch<int16_t>(a, stream);
}
