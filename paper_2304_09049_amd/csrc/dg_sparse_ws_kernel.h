// 2-bit table kernel on the sparse matrix instruction with the WEIGHT OPERANDS STATIONARY in registers, for layers
// with a short reduction (1x1 convolutions / GEMMs with K = 64, 128 or 256) whose time is the output's way to memory.
//
// In the tiled sparse-instruction kernel (dg_onehot_kernel.h, BITS = 20) every wavefront rebuilds the dense operand --
// the table rows of its weight codes, 4 bytes per (row, position) -- for every tile it owns: about 23 VALU instructions
// and 8 LDS reads per pair of matrix instructions.  With K <= 256 the dense operand of 32 weight rows over ALL of K is
// at most 128 registers per lane, so here a wavefront builds it once, keeps it, and then only streams pixels: per 32
// pixels it loads their packed words (the index registers of the instruction as they are: no expansion), issues K / 16
// matrix instructions and stores the 32 x 32 sums.  Stores of one block overlap the loads and matrix instructions of the
// next (a store reads its registers when it issues, nothing waits for it), and nothing of the contraction is left on
// the VALU.  Operand layout and the row-pair table in LDS are those of dg_onehot_kernel.h.
//
// Work split: a wavefront owns one block of 32 output channels (its stationary weights) and a contiguous run of
// 32-pixel blocks; the wavefronts of the other channel blocks of the same pixels sit next to it in the workgroup, so
// the pixels' words are fetched from memory once and the halves of an output row are written together.
#pragma once

#include <type_traits>

#include "dg_lds_dma.h"
#include "dg_onehot_kernel.h"

namespace dgoh {

struct WsArgs {
    DgProblem p;
    uint32_t rows[4];            // rows[w] = bytes T[w][0..3]
    int32_t row_blocks;          // ceil(M / 32)
    int32_t streams;             // runs of pixel blocks; wavefronts = row_blocks * streams
    int32_t run, longer;         // the first `longer` runs have run + 1 pixel blocks, the others `run`
    FastDiv div_row_blocks;
    FastDiv div_ow, div_oh;      // STRIDED: output pixel -> (image, row, column)
    int32_t count_stores;        // RAW: 0 = a wait for staged codes also waits for the stores issued so far (A/B measurement)
};

// T = K / 32: matrix-instruction pairs per 32 x 32 block; a lane half reads T words of a pixel (or weight row).
// (T = 16, K = 512, on packed activations: 256 registers of dense operands -- a lone wavefront per SIMD has 512.)
// G: pixel blocks per group (their words are in registers together).
// What was measured on the 56x56x256 -> 64 layer at batch 32 (25.7 MB of output, which alone takes 5.2 us to write in
// HIP-graph replays, whatever the store pattern): the layer's time is the time to the first stores and the drain, so
//   - the words of a whole group of pixel blocks are loaded before the group's first store is issued: a wavefront's
//     vector memory instructions leave the compute unit in issue order, and a load queued behind a burst of stores
//     waits until the memory system has taken them; a wavefront's run is normally one group;
//   - there is no division in the prologue (0.3 us);
//   - blocks are computed and stored one at a time: two blocks sharing the instruction stream (independent sums back to
//     back) store in larger bursts and were 0.7 us slower; so was building the operands interleaved with the first block;
//   - pixel words are asked for before the weight words (0.15 us faster than the other way round).
//
// RAW: the activations are codes one per byte ([pixel][K] bytes at p.Xp) and are packed by the kernel itself, which
// spares a layer the packing kernel (as long as this one on the 56x56x256 -> 64 layer) and the packed tensor's round
// trip through memory.  A lane needs half a pixel's codes, 16 T contiguous bytes -- as direct loads that is a cache
// line of its own per lane and instruction, which the address unit takes a line per cycle -- so the codes of a pixel
// block are staged (dg_lds_dma.h): 2 T neighbouring lanes read the 32 T bytes of one pixel straight into LDS, two
// blocks in flight per wavefront, and lane (pixel, half) reads its 16-byte segments from there and packs each into a
// word.  Slot j of a staged pixel holds its segment j ^ (pixel % 2T): the exchange spreads the 32 pixels' reads of one
// segment over the LDS banks.
// What a timeline of this form showed (timestamps per wavefront, 56x56x256 -> 64 at batch 32): writing the 25.7 MB of
// output takes 5.2 us whatever the store pattern, and the kernel's time is that plus the time to the first stores.  So
// the weight rows are asked for BEFORE the first block's codes (loads complete in issue order, and the weights waited
// behind two blocks of codes), the second block only after the dense operands are built (the address unit serves
// every wavefront's first block first), and a wait for staged codes does not wait for the stores issued since: the
// wavefront counts them (9.5 -> 8.9 us on that layer; the same at batch 8: 5.2 -> 4.7 us).
// STRIDED (packed activations): a 1x1 convolution with a stride and no padding -- output pixel (b, oh, ow) reads the
// row of input pixel (b, oh * sh, ow * sw).
template <int T, int G, bool RAW, bool STRIDED = false>
__global__ void __launch_bounds__(256, (!RAW && T * G > 32 ? 1 : 2))
smfmac_ws_kernel(WsArgs a)
{
    static_assert(T == 2 || T == 4 || T == 8 || (T == 16 && !RAW), "K = 64, 128 or 256; 512 on packed activations");
    static_assert(!(RAW && STRIDED), "the form that packs reads contiguous pixels");
    __shared__ uint2 s_rows[16];                            // the table of row pairs, one for the workgroup
    extern __shared__ uint4 s_codes[];                      // RAW: [wavefront][2][32 pixels x 2 T segments]
    const DgProblem &p = a.p;
    const int lane = threadIdx.x & 63, w4 = threadIdx.x >> 6;
    {
        Pools pl;
#pragma unroll
        for (int i = 0; i < 4; ++i) pl.w[i] = a.rows[i];
        sparse_fill_table(s_rows, pl, threadIdx.x);
    }
    // (no division in the prologue: it is on the way to the first store)
    const uint32_t wave = xcd_contiguous(blockIdx.x, gridDim.x) * 4u + (uint32_t)__builtin_amdgcn_readfirstlane(w4);
    const uint32_t stream = fdiv(wave, a.div_row_blocks);
    const int rb = (int)(wave - stream * (uint32_t)a.row_blocks);
    const bool idle = stream >= (uint32_t)a.streams;        // (a wavefront beyond the last run: it only joins the barrier)
    const int r = lane & 31, h = lane >> 5;
    const int row_bytes = p.K / 4;                          // = 8 * T
    const int m0 = rb * 32;

    // this wavefront's run of pixel blocks
    const int64_t b0 = (int64_t)stream * a.run + min(stream, (uint32_t)a.longer);
    const int64_t b1 = b0 + a.run + (stream < (uint32_t)a.longer ? 1 : 0);
    const int last_row = p.N - 1;
    const uint8_t *x_base = p.Xp + h * (4 * T);
    Words<T> x[G];
    constexpr int SP = 2 * T, BLOCK = 32 * SP;              // RAW: 16-byte segments per pixel, and per staged pixel block
    const int wv = __builtin_amdgcn_readfirstlane(w4);
    const uint32_t codes_lds = dg_lds_address(s_codes) + wv * (2 * BLOCK * 16);
    // RAW, as a loader: instruction j of a block fetches pixels j * (64 / SP) + lp, this lane segment seg_off[j] / 16 of
    // each (slot ls of the staged pixel).  Rows beyond N re-read row N - 1: the pixel is clamped, branch-free.
    uint32_t seg_off[RAW ? T : 1];
    uint32_t lp_bytes = 0;
    if constexpr (RAW) {
        const int lp = lane / SP, ls = lane % SP;
        lp_bytes = (uint32_t)(lp * p.K);
#pragma unroll
        for (int j = 0; j < T; ++j) seg_off[j] = (uint32_t)((ls ^ ((j * (64 / SP) + lp) % SP)) * 16);
    }
    auto stage = [&](int64_t blk, int buf) {                // RAW: pixel block `blk` into buffer `buf`
        const uint32_t dst = codes_lds + buf * BLOCK * 16;
        const uint8_t *base = p.Xp + blk * 32 * p.K;        // (uniform: one base address, the lanes' offsets)
        const uint32_t last = (uint32_t)min((int64_t)31, (int64_t)last_row - blk * 32) * (uint32_t)p.K;
#pragma unroll
        for (int j = 0; j < T; ++j)
            dg_load16_to_lds(base, (int32_t)(min(lp_bytes + (uint32_t)(j * (64 / SP) * p.K), last) + seg_off[j]), dst + j * 64 * 16);
    };
    auto fetch = [&](int64_t blk) {                         // rows beyond N re-read row N - 1 (their sums are not stored)
#pragma unroll
        for (int g = 0; g < G; ++g) {
            int64_t n = min((blk + g) * 32 + r, (int64_t)last_row);
            if constexpr (STRIDED) {
                const uint32_t line = fdiv((uint32_t)n, a.div_ow), image = fdiv(line, a.div_oh);
                const int64_t ow = n - (int64_t)line * p.OW, oh = (int64_t)line - (int64_t)image * p.OH;
                n = ((int64_t)image * p.H + oh * p.sh) * p.W + ow * p.sw;
            }
            if (blk + g < b1) x[g] = load_words_any<T>(x_base + n * row_bytes);
        }
    };
    float sc_cols[1] = {0.0f};
    if constexpr (RAW) {
        // The order in which a wavefront asks: its scale, its weight rows (staged like the codes, into the second
        // buffer), its first block of codes.  Loads complete in that order, so the dense operands are built while the
        // first block is still on its way; the second block is asked for once they are (a compute unit's address unit
        // serves its wavefronts' first blocks first).  These loads are assembly so that the wavefront itself counts
        // what it waits for: the compiler would wait for everything, staged codes included.
        // A wavefront never ends with a staged load in flight -- its LDS could be another workgroup's by the time the
        // data lands: it starts loads for blocks of its run only, and waits for each.
        if (!idle) {
            const float *sc_at = p.scale ? p.scale + min(m0 + r, p.M - 1) : (const float *)p.Wp;      // (no scales: any readable word)
            asm volatile("global_load_dword %0, %1, off" : "=v"(sc_cols[0]) : "v"(sc_at) : "memory");
            constexpr int LPR = T >= 4 ? T / 2 : 1, NWI = T >= 4 ? T / 4 : 1;      // lanes per weight row; instructions
#pragma unroll
            for (int j = 0; j < NWI; ++j) {
                const int row = min(j * (64 / LPR) + lane / LPR, 31);
                dg_load16_to_lds(p.Wp + (int64_t)min(m0 + row, p.M - 1) * row_bytes + (lane % LPR) * 16, codes_lds + BLOCK * 16 + j * 1024);
            }
            stage(b0, 0);
        }
    } else {
        fetch(b0);
    }

    // the stationary dense operands: for word t of either half of the weight row, the even and the odd codes' table rows
    v8i dn[T][2];
    if constexpr (RAW) {
        // (the table is in LDS once every wavefront is here; the loads above stay in flight across this barrier, which
        // waits for LDS operations only)
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
        if (idle) return;
        // the scale and the weight rows are in; the first block's T loads may be under way
        asm volatile("s_waitcnt vmcnt(%1)" : "+v"(sc_cols[0]) : "n"(T) : "memory");
        const uint4 *wsrc = (const uint4 *)((const char *)s_codes + wv * (2 * BLOCK * 16) + BLOCK * 16 + r * row_bytes);
        uint32_t ww[2 * T];
#pragma unroll
        for (int i = 0; i < (T >= 2 ? T / 2 : 1); ++i) {
            const uint4 q = wsrc[i];
            ww[4 * i] = q.x, ww[4 * i + 1] = q.y, ww[4 * i + 2] = q.z, ww[4 * i + 3] = q.w;
        }
        const uint32_t pick = sparse_pick(h);
#pragma unroll
        for (int t = 0; t < T; ++t) sparse_dense_rows_shared(s_rows, ww[t], ww[T + t], pick, dn[t][0], dn[t][1]);
        // (the weight rows are in registers: their buffer takes the second block)
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        if (b0 + 1 < b1) stage(b0 + 1, 1);
    } else {
        const uint8_t *wrow = p.Wp + (int64_t)min(m0 + r, p.M - 1) * row_bytes;
        const Words<T> w0 = load_words_any<T>(wrow), w1 = load_words_any<T>(wrow + 4 * T);
        // (the table is in LDS once every wavefront is here; the loads above stay in flight across this barrier,
        // which waits for LDS operations only)
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
        if (idle) return;
        const uint32_t pick = sparse_pick(h);
#pragma unroll
        for (int t = 0; t < T; ++t) sparse_dense_rows_shared(s_rows, w0.v[t], w1.v[t], pick, dn[t][0], dn[t][1]);
        dg_mfma_column_scales<1, true>(p, m0, lane, sc_cols);
    }
    // the kept bytes: (1, 0) per position with the even codes, (0, 1) with the odd; the index of both is the packed word
    const v4i ones[2] = {{0x00010001, 0x00010001, 0x00010001, 0x00010001}, {0x01000100, 0x01000100, 0x01000100, 0x01000100}};

    if constexpr (RAW) {
        // A block's codes are packed and multiplied while the next block is on its way; the loads of the block after
        // next are issued as soon as the buffer's codes are in registers, ahead of this block's stores.
        // Waiting for a block's loads: the counter counts stores as well, and everything completes in issue order.
        // Issued after block blk's loads were: the stores of block blk - 2, the loads of block blk + 1, the stores of
        // block blk - 1 -- all of which may still be under way.  The stores of a block wholly inside the output are 16
        // instructions (dg_mfma_store_block: one per sum register); of any other block they count as none here, which
        // only waits longer.
        auto stores_of = [&](int64_t blk) -> int {
            const int64_t span = 32 * ((p.stride_cn < 0 ? -p.stride_cn : p.stride_cn) + (p.stride_cm < 0 ? -p.stride_cm : p.stride_cm));
            const bool whole = m0 + 32 <= p.M && (blk + 1) * 32 <= (int64_t)p.N && span < ((int64_t)1 << 30);
            return a.count_stores && p.Qp == nullptr && whole ? 16 : 0;
        };
        int stores1 = 0, stores2 = 0;                       // of the last block, of the one before
        // (the body twice, with and without the loads of the block after next, so that each is straight-line code: the
        // compiler then issues those loads between the matrix instructions, whose chain they do not hold up.  One body
        // with the loads issued behind the block's stores measured the same on some boxes of the pool and 0.65 us
        // slower on others.)
        auto block = [&](int64_t blk, auto ahead) {
            const int buf = (int)(blk - b0) & 1;
            dg_wait_for_loads_at_most(stores2 + (blk + 1 < b1 ? T : 0) + stores1);
            const uint4 *src = s_codes + (wv * 2 + buf) * BLOCK + r * SP;
            uint4 c[T];
#pragma unroll
            for (int i = 0; i < T; ++i) c[i] = src[(h * T + i) ^ (r % SP)];
            Words<T> xw;
#pragma unroll
            for (int i = 0; i < T; ++i) xw.v[i] = dg_pack_codes16(c[i]);
            if constexpr (decltype(ahead)::value) {
                // (the buffer's codes are in registers, not merely asked for, before loads that overwrite it are issued)
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                stage(blk + 2, buf);
            }
            v16i acc;
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[e] = 0;
#pragma unroll
            for (int t = 0; t < T; ++t)
#pragma unroll
                for (int par = 0; par < 2; ++par)
                    acc = __builtin_amdgcn_smfmac_i32_32x32x64_i8(ones[par], dn[t][par], acc, (int)xw.v[t], 0, 0);
            dg_mfma_store_block<true>(p, acc, m0, (int)(blk * 32), lane, sc_cols[0]);
            stores2 = stores1, stores1 = stores_of(blk);
        };
        int64_t blk = b0;
        for (; blk + 2 < b1; ++blk) block(blk, std::true_type{});
        for (; blk < b1; ++blk) block(blk, std::false_type{});
        return;
    }
    for (int64_t blk = b0; blk < b1; blk += G) {
        // one block at a time, so that the first stores go out as early as possible: the layer's time is the time its
        // output takes to drain, counted from the first store (the other wavefront of the SIMD fills the gaps between
        // the dependent matrix instructions)
#pragma unroll
        for (int g = 0; g < G; ++g) {
            if (blk + g >= b1) break;                       // (uniform)
            v16i acc;
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[e] = 0;
#pragma unroll
            for (int t = 0; t < T; ++t)
#pragma unroll
                for (int par = 0; par < 2; ++par)
                    acc = __builtin_amdgcn_smfmac_i32_32x32x64_i8(ones[par], dn[t][par], acc, (int)x[g].v[t], 0, 0);
            dg_mfma_store_block<true>(p, acc, m0, (int)((blk + g) * 32), lane, sc_cols[0]);
        }
        // (only a run longer than one group comes here; these loads do queue behind the group's stores, which is why
        // the host sizes runs to one group where it can)
        if (blk + G < b1) fetch(blk + G);
    }
}

// `raw`: p.Xp holds codes one per byte
inline void launch_sparse_ws(const DgProblem &p, const uint32_t (&rows)[4], int streams, bool raw, hipStream_t stream)
{
    WsArgs a;
    a.p = p;
    for (int w = 0; w < 4; ++w) a.rows[w] = rows[w];
    a.row_blocks = (p.M + 31) / 32;
    const int pixel_blocks = (p.N + 31) / 32;
    a.streams = streams;
    a.run = pixel_blocks / streams;
    a.longer = pixel_blocks % streams;
    a.div_row_blocks = make_div((uint32_t)a.row_blocks);
    a.div_ow = make_div((uint32_t)p.OW), a.div_oh = make_div((uint32_t)p.OH);
    const bool strided = p.sh != 1 || p.sw != 1;           // (the host sends these on packed activations only)
    a.count_stores = 1;
    if (const char *e = dg_override("DG_WS_COUNT_STORES")) a.count_stores = atoi(e) != 0;
    const int64_t waves = (int64_t)a.row_blocks * streams;
    const dim3 grid((unsigned)((waves + 3) / 4));
    // a wavefront's whole run in one group where the registers allow it (up to 8 blocks)
    const int t = p.K / 32;
    const bool wide = a.run + (a.longer ? 1 : 0) > 4;
    // (the staging buffers of the form that packs: 4 wavefronts x 2 blocks x 32 pixels x K bytes, up to 64 KB)
#define DG_WS(T, G)                                                                                                   \
    do {                                                                                                              \
        if (raw) {                                                                                                    \
            const int lds = 4 * 2 * 32 * 32 * T;                                                                      \
            (void)hipFuncSetAttribute((const void *)smfmac_ws_kernel<T, G, true>, hipFuncAttributeMaxDynamicSharedMemorySize, lds); \
            hipLaunchKernelGGL((smfmac_ws_kernel<T, G, true>), grid, dim3(256), lds, stream, a);                      \
        } else if (strided) {                                                                                         \
            hipLaunchKernelGGL((smfmac_ws_kernel<T, G, false, true>), grid, dim3(256), 0, stream, a);                 \
        } else {                                                                                                      \
            hipLaunchKernelGGL((smfmac_ws_kernel<T, G, false>), grid, dim3(256), 0, stream, a);                       \
        }                                                                                                             \
    } while (0)
    if (t == 16) {
        if (strided)
            hipLaunchKernelGGL((smfmac_ws_kernel<16, 4, false, true>), grid, dim3(256), 0, stream, a);
        else
            hipLaunchKernelGGL((smfmac_ws_kernel<16, 4, false>), grid, dim3(256), 0, stream, a);
    } else if (t == 8 && wide) DG_WS(8, 8);
    else if (t == 8) DG_WS(8, 4);
    else if (t == 4 && wide) DG_WS(4, 8);
    else if (t == 4) DG_WS(4, 4);
    else if (wide) DG_WS(2, 8);
    else DG_WS(2, 4);
#undef DG_WS
}

}   // namespace dgoh
