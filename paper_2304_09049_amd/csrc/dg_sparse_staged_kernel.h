// 2-bit table kernel on the sparse matrix instruction (operand layout, index register and row-pair table as in
// dg_onehot_kernel.h, BITS = 20), with the packed operands fetched in WHOLE 32-BYTE RUNS and handed to their lanes
// through LDS.  A wavefront owns a tile of 32 (or 64) channels x 64 ... 224 pixels and walks all of K, or a share of it.
//
// Why: the matrix instruction wants lane (r, half) to hold words of row r, so a direct load has 32 lanes reading 8
// bytes each from 32 different rows.  The address unit of a compute unit takes such a load one cache line per cycle
// (dg_lds_dma.h): 64 cycles and more for 512 or 1024 bytes, and on a GEMM with K = 8192 it was busy 93 % of the
// kernel's time (counters TA_TA_BUSY / TCP_GATE_EN) while the matrix pipe idled -- the loads, not the arithmetic, set
// the time.  Here two neighbouring lanes read the two 16-byte halves of one row's run, so a load instruction covers 32
// rows x 32 bytes, at half the address cycles per byte (26 % busy on the same GEMM).  The loads write LDS directly
// (lane l's 16 bytes land at the instruction's LDS base + 16 l; no registers are held while they are in flight), into
// staging rows of the wavefront's own, from which lane (r, half) reads its 8 bytes per 64 positions of K.  Staging
// rows belong to one wavefront, so no barrier is involved: a wavefront waits for its own loads (vmcnt) before it reads
// a run, and runs alternate between two buffers, fetched two ahead.
// The multiplication is one software pipeline over all of K: the dense operands of a step are made between the matrix
// instructions of the step before, across chunks, runs and filter taps alike.
//
// A run is 128 positions of K inside one filter tap (Cin % 128 == 0; Cin % 128 == 64: HALF below).  A tap outside the image is fetched from a
// clamped address and contributes nothing because the kept bytes of its lanes are zero.
#pragma once

#include "dg_lds_dma.h"
#include "dg_onehot_kernel.h"

namespace dgoh {

// The dense operands of all WM weight blocks for word `t` of `w` (as sparse_dense_rows_shared, but with the opaque
// statement that keeps the indices pre-multiplied NOT volatile, so that the scheduler may move these instructions
// between matrix instructions).
template <int WM, class W>
__device__ __forceinline__ void dense_rows_movable(const uint2 *table, const W &w, int t, uint32_t pick, v8i (&out)[WM][2])
{
#pragma unroll
    for (int u = 0; u < WM; ++u) {
        const uint32_t w0 = t ? w.ca[u].y : w.ca[u].x, w1 = t ? w.ca1[u].y : w.ca1[u].x;
        const uint32_t v = __builtin_amdgcn_perm(w1, w0, pick), s2 = v >> 2;
        uint32_t e = ((v & 0x03030303u) | (s2 & 0x0C0C0C0Cu)) << 3;          // byte b: 8 * (code 4b | code 4b+2 << 2)
        uint32_t o = ((s2 & 0x03030303u) | ((v >> 4) & 0x0C0C0C0Cu)) << 3;   // byte b: 8 * (code 4b+1 | code 4b+3 << 2)
        asm("" : "+v"(e), "+v"(o));
        const char *base = (const char *)table;
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const uint2 x = *(const uint2 *)(base + ((e >> (8 * b)) & 255u)), y = *(const uint2 *)(base + ((o >> (8 * b)) & 255u));
            out[u][0][2 * b] = (int)x.x, out[u][0][2 * b + 1] = (int)x.y;
            out[u][1][2 * b] = (int)y.x, out[u][1][2 * b + 1] = (int)y.y;
        }
    }
}

// SKW = 1: a wavefront walks all of K.  SKW = 2 or 4 (layers whose tiles alone would leave SIMDs idle): SKW wavefronts
// of the workgroup share a tile and split K between them (run by run, or in contiguous shares); their sums meet in LDS by integer atomics
// (exact in any order) and each of them stores a share of the tile's blocks, as in dg_onehot_kernel.h.
//
// HALF (unshared tiles, Cin % 128 == 64): a filter tap is an odd number of
// 64-position chunks, so the two chunks of a run may lie in different taps -- two different pixels for the loader's two
// lanes of a row, two sets of kept bytes for the run's two halves -- and the last run of K may be half a run, whose
// second chunk is fetched from the first's place and multiplied by kept bytes of zero.
template <int WM, int WN, int SKW, bool TURNS, bool HALF>
__global__ void __launch_bounds__(256, 2)
smfmac_staged_kernel(Args a)
{
    static_assert(!HALF || SKW == 1, "taps of half runs: unshared tiles only");
    constexpr int ROWS = (WM + WN) * 32;                    // staged rows of a wavefront: its weight rows, then its pixels
    constexpr int BUF = ROWS * 32;                          // bytes of one wavefront's buffer
    constexpr int TPW = 4 / SKW;                           // tiles per workgroup
    constexpr int NB = WM * WN;                            // 32x32 output blocks per tile
    // A block of 32 rows is 64 slots of 16 bytes, slot j = what loader lane j fetched: row j / 2, segment
    // (j % 2) ^ (j / 16 % 2) of the row's 32 bytes -- the exchange puts rows r and r + 8 of a segment on different
    // LDS banks, which leaves the consumers' reads (32 rows of one segment) two to a bank instead of four.
    __shared__ uint2 s_rows[16];                            // the table of row pairs, one for the workgroup
    // staging rows [wavefront][buffer][block * 64 + slot]; once the walk over K is over, the same memory holds the
    // shared tiles' sums [tile][block][sum register][lane]
    constexpr int STAGE_BYTES = 4 * 2 * BUF, SUM_BYTES = SKW > 1 ? TPW * NB * 4096 : 0;
    __shared__ uint4 s_mem[(STAGE_BYTES > SUM_BYTES ? STAGE_BYTES : SUM_BYTES) / 16];
    static_assert(sizeof(s_mem) <= 80 * 1024 - 256, "two workgroups per compute unit (160 KB of LDS)");
    int32_t *s_acc = (int32_t *)s_mem;
    // the narrower tiles have the registers for a second set of kept bytes, (0, 1), which spares the odd codes' shift
    constexpr bool SHIFT_ODD = WM * WN >= 7;
    const DgProblem &p = a.p;
    const int lane = threadIdx.x & 63, w4 = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int ks = w4 % SKW, tw = w4 / SKW;                 // this wavefront's share of K, and its tile within the workgroup
    const int64_t my_tile = (int64_t)xcd_contiguous(blockIdx.x, gridDim.x) * TPW + tw;
    const bool active = my_tile < a.wave_tiles;
    sparse_fill_table(s_rows, a.pools, threadIdx.x);
    __syncthreads();                                       // (every wavefront of the workgroup, also one without a tile)
    if (SKW == 1 && !active) return;                       // whole wavefronts leave; no barrier follows on this path
    const int64_t wave_tile = active ? my_tile : 0;        // (an idle wavefront of a shared workgroup adds nothing)
    const int r = lane & 31, h = lane >> 5;
    // Tiles are numbered in bands of 2^band_log2 pixel tiles; inside a band groups of 2^m_log2 channel tiles (the four
    // wavefronts of a workgroup, which then share their pixels' loads) follow each other along the pixels first.  The
    // tiles in flight on an XCD at one time (consecutive numbers, see xcd_contiguous) then form a patch about as high
    // as it is wide, whose weight rows and pixels that XCD's L2 fetches once (numbered along the channels first, every
    // column of tiles streamed all of the weights through the L2 again: 4.3 times the operands' bytes on an 8192-cube).
    int m_tile, n_tile;
    {
        const uint32_t t = (uint32_t)wave_tile, band = fdiv(t, a.div_band), t_in = t - band * a.band_tiles;
        const uint32_t g = t_in >> a.m_log2, mi = t_in & ((1u << a.m_log2) - 1u);
        const int first = (int)band << a.band_log2, width = min(1 << a.band_log2, a.tiles_n - first);
        uint32_t mg;
        if (width == 1 << a.band_log2)
            mg = g >> a.band_log2;
        else
            mg = fdiv(g, a.div_last);                       // (the last band, narrower)
        n_tile = first + (int)(g - mg * (uint32_t)width);
        m_tile = (int)((mg << a.m_log2) + mi);
    }
    const int m0 = m_tile * (WM * 32), n0 = n_tile * (WN * 32);
    const int cq = p.Cin / 4;                               // packed bytes per pixel
    // This wavefront's runs of K: g0, g0 + stride, ... below g1.  TURNS (layers without a filter window): wavefronts sharing
    // a tile take turns run by run (stride SKW), so that at any time the four of them read the four 32-byte runs of the SAME
    // cache lines -- one fetch into the compute unit's cache serves all; with a contiguous quarter of K each, every
    // wavefront streamed lines of its own, which the cache lost before their next run came up (66 address cycles per
    // load against 34; 8192 x 256 x 8192: 28.7 -> 24.4 us).  With a window they keep contiguous shares: taking turns
    // puts every run of a wavefront in another filter tap, and the kept bytes made anew per run cost more than the
    // cache gives (3x3 layers 7 - 14 % slower).
    static_assert(!TURNS || SKW > 1, "taking turns is for wavefronts that share a tile");
    constexpr int stride = TURNS ? SKW : 1;
    const int runs = HALF ? (p.K + 127) / 128 : p.K / 128, share = (runs + SKW - 1) / SKW;
    const int chunks = p.K / 64, cpt = p.Cin / 64;          // HALF: 64-position chunks in all, and per filter tap
    const int g0 = min(TURNS ? ks : ks * share, runs), g1 = !active ? g0 : (TURNS ? runs : min(g0 + share, runs));
    const int runs_per_tap = cq / 32;
    const int tap0 = (int)fdiv((uint32_t)g0, a.div_runs), rt0 = g0 - tap0 * runs_per_tap;

    // as a loader, this lane fetches 16-byte segment lseg of row lrow of every 32-row block
    const int lrow = lane >> 1, lseg = (lane & 1) ^ ((lane >> 4) & 1);
    const uint8_t *w_ld[WM];
#pragma unroll
    for (int bm = 0; bm < WM; ++bm)
        w_ld[bm] = p.Wp + (int64_t)min(m0 + bm * 32 + lrow, p.M - 1) * (p.K / 4) + (HALF ? 0 : lseg * 16);
    int32_t x_ld[WN];                                       // (32-bit offsets: the host sends inputs below 2^31 bytes)
#pragma unroll
    for (int bn = 0; bn < WN; ++bn)
        x_ld[bn] = (int32_t)make_column(p, a.div_ow, a.div_oh, n0 + bn * 32 + lrow, cq, HALF ? 0 : lseg * 16).off0;
    const int images = (int)fdiv(fdiv((uint32_t)p.N, a.div_ow), a.div_oh);
    const int32_t x_last = images * p.H * p.W * cq - 16;    // the last 16 bytes of the packed activations
    // as a consumer, it is row / pixel r (lane half h) of every block: its slot of segment s is slot0 ^ s
    const int slot0 = 2 * r + ((r >> 3) & 1);
    Column col[WN];
#pragma unroll
    for (int bn = 0; bn < WN; ++bn) col[bn] = make_column(p, a.div_ow, a.div_oh, n0 + bn * 32 + r, cq, 0);

    v16i acc[WM][WN];
#pragma unroll
    for (int bm = 0; bm < WM; ++bm)
#pragma unroll
        for (int bn = 0; bn < WN; ++bn)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[bm][bn][e] = 0;
    float sc_cols[WM];
    dg_mfma_column_scales<WM, true>(p, m0, lane, sc_cols);

    // ---- the loader's side: runs are fetched two ahead of the one being multiplied
    const char *stage = (const char *)s_mem + w4 * (2 * BUF);
    const uint32_t stage_lds = dg_lds_address(s_mem) + w4 * (2 * BUF);
    // filter tap and byte within the pixel of the run fetched next
    int kh = (int)fdiv((uint32_t)tap0, a.div_kw), kw = tap0 - kh * p.KW, cib = rt0 * 32, fetched = g0, fetches = 0;
    auto fetch = [&]() {                                    // this wavefront's next run, into the buffer of its parity
        const int g = min(fetched, runs - 1);               // (past the end: a run inside the tensors, unused)
        const uint32_t dst = stage_lds + ((TURNS ? fetches : fetched) & 1) * BUF;
        if constexpr (HALF) {
            // this lane's chunk of the run: 2 g + lseg (past the end of K: the chunk before), its tap and place in it
            const int c0 = 2 * g, c1 = min(2 * g + 1, chunks - 1);
            auto pixel_offset = [&](int c) {
                const int tap = (int)fdiv((uint32_t)c, a.div_cpt), th = (int)fdiv((uint32_t)tap, a.div_kw);
                return (int32_t)((th * p.W + (tap - th * p.KW)) * cq + (c - tap * cpt) * 16);
            };
            const int32_t off0 = pixel_offset(c0), off1 = pixel_offset(c1);
            const int32_t w_off = (lseg ? c1 : c0) * 16, x_off = lseg ? off1 : off0;
#pragma unroll
            for (int bm = 0; bm < WM; ++bm) dg_load16_to_lds(w_ld[bm] + w_off, dst + bm * 1024);
#pragma unroll
            for (int bn = 0; bn < WN; ++bn) dg_load16_to_lds(p.Xp, max(0, min(x_ld[bn] + x_off, x_last)), dst + (WM + bn) * 1024);
            ++fetches, ++fetched;
            return;
        }
#pragma unroll
        for (int bm = 0; bm < WM; ++bm) dg_load16_to_lds(w_ld[bm] + g * 32, dst + bm * 1024);
        const int32_t tap_off = (kh * p.W + kw) * cq + cib;
#pragma unroll
        for (int bn = 0; bn < WN; ++bn) {
            // (a tap outside the image or past the end: any address inside the tensor will do; the kept bytes of a
            // lane outside the image are zero)
            const int32_t off = max(0, min(x_ld[bn] + tap_off, x_last));
            dg_load16_to_lds(p.Xp, off, dst + (WM + bn) * 1024);
        }
        ++fetches;
        fetched += stride;
        cib += 32 * stride;
        if constexpr (TURNS) {
            while (cib >= cq) cib -= cq;                    // (uniform; no filter window: the tap stays)
        } else if (cib == cq) {                             // (uniform)
            cib = 0;
            if (++kw == p.KW) {
                kw = 0;
                ++kh;
            }
        }
    };

    // ---- the consumer's side.  Words of a chunk (64 positions): of weight row r both halves' 8 bytes, of pixel r its
    // own half's.  Lane offsets into a buffer, for the run's two chunks:
    const int w_at[2] = {slot0 * 16, (slot0 ^ 1) * 16}, x_at[2] = {slot0 * 16 + h * 8, (slot0 ^ 1) * 16 + h * 8};
    struct Words2 {
        uint2 ca[WM], ca1[WM], cb[WN];
    };
    auto read_words = [&](Words2 &w, int buf, int s) {
        const char *src = stage + buf * BUF;
#pragma unroll
        for (int bm = 0; bm < WM; ++bm) {
            const uint4 q = *(const uint4 *)(src + bm * 1024 + w_at[s]);
            w.ca[bm] = make_uint2(q.x, q.y), w.ca1[bm] = make_uint2(q.z, q.w);
        }
#pragma unroll
        for (int bn = 0; bn < WN; ++bn) w.cb[bn] = *(const uint2 *)(src + (WM + bn) * 1024 + x_at[s]);
    };
    const uint32_t pick = sparse_pick(h);
    auto word = [](const uint2 &v, int t) { return t ? v.y : v.x; };
    // One step = one word of the chunk: two instructions (even codes, odd codes) per block of the tile, with the dense
    // operands `next` of the following step -- per weight block a unit of table reads -- made between them.
    // (see dg_onehot_kernel.h for the index register and the kept bytes)
    v4i ones[WN], ones_odd[SHIFT_ODD ? 1 : WN];
    // which of this lane's pixels see a filter tap: the kept bytes, (1, 0) per position (and (0, 1) for the odd codes),
    // or zeros outside the image (or for a chunk past the end of K)
    auto kept_bytes = [&](int tap, bool live, v4i (&on)[WN], v4i (&on_odd)[SHIFT_ODD ? 1 : WN]) {
        const int khc = (int)fdiv((uint32_t)tap, a.div_kw), kwc = tap - khc * p.KW;
#pragma unroll
        for (int bn = 0; bn < WN; ++bn) {
            const int ih = col[bn].ih0 + khc, iw = col[bn].iw0 + kwc;
            const bool v = live & col[bn].ok & ((uint32_t)ih < (uint32_t)p.H) & ((uint32_t)iw < (uint32_t)p.W);
            const int x = v ? 0x00010001 : 0;
            on[bn] = (v4i){x, x, x, x};
            if constexpr (!SHIFT_ODD) {
                const int y = v ? 0x01000100 : 0;
                on_odd[bn] = (v4i){y, y, y, y};
            }
        }
    };
    auto step = [&](const v8i (&dn)[WM][2], const Words2 &w, int t, v8i (&next)[WM][2], const Words2 &nw, int nt,
                    const v4i (&ones)[WN], const v4i (&ones_odd)[SHIFT_ODD ? 1 : WN]) {
        constexpr int MN = WM * WN;
        // the next step's dense operands: written here, spread by the scheduling groups below a few instructions at a
        // time between this step's matrix instructions, in whose shadow they then issue
        dense_rows_movable(s_rows, nw, nt, pick, next);
        int odd_ix[SHIFT_ODD ? WN : 1];
        if constexpr (SHIFT_ODD) {
#pragma unroll
            for (int bn = 0; bn < WN; ++bn) odd_ix[bn] = (int)(word(w.cb[bn], t) >> 2);
        }
        constexpr int PER = (31 * WM + (SHIFT_ODD ? WN : 0) + 2 * MN - 1) / (2 * MN);      // other instructions per matrix instruction
#pragma unroll
        for (int i = 0; i < 2 * MN; ++i) {
            const int par = i / MN, bm = (i % MN) / WN, bn = i % WN;
            if (par && !SHIFT_ODD)
                acc[bm][bn] = __builtin_amdgcn_smfmac_i32_32x32x64_i8(ones_odd[SHIFT_ODD ? 0 : bn], dn[bm][1], acc[bm][bn], (int)word(w.cb[bn], t), 0, 0);
            else
                acc[bm][bn] = __builtin_amdgcn_smfmac_i32_32x32x64_i8(ones[bn], dn[bm][par], acc[bm][bn],
                                                                      par ? odd_ix[SHIFT_ODD ? bn : 0] : (int)word(w.cb[bn], t), 0, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x102, PER, 0);
        }
    };

    if (g0 < g1) {                                          // (uniform; a wavefront without a share of K only joins the barrier)
        fetch();
        fetch();
        // The sums start at zero, or -- the table's entries having been raised by a.bias to make them all small and
        // non-negative (launch_sparse_staged says why) -- at minus the bias for every position of K the pixel really
        // sees: Cin per filter tap inside the image.  Lane (r, .) works that out for pixel r of a block; sum register
        // e of a lane belongs to pixel 8 (e / 4) + 4 h + e % 4 and takes it from that lane.  Of the wavefronts sharing
        // a tile the first one does this (it always has a share of K).  Done here, while the first runs are on their way.
        if (a.bias != 0 && ks == 0) {                       // (uniform)
#pragma unroll
            for (int bn = 0; bn < WN; ++bn) {
                const int ih0 = col[bn].ih0, iw0 = col[bn].iw0;
                const int taps_h = max(0, min(p.KH, p.H - ih0) - max(0, -ih0)), taps_w = max(0, min(p.KW, p.W - iw0) - max(0, -iw0));
                const int start = col[bn].ok ? -a.bias * p.Cin * taps_h * taps_w : 0;
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int v = __builtin_amdgcn_ds_bpermute(4 * (8 * (e / 4) + 4 * h + e % 4), start);
#pragma unroll
                    for (int bm = 0; bm < WM; ++bm) acc[bm][bn][e] = v;
                }
            }
        }
        Words2 wa, wb;
        v8i dn0[WM][2], dn1[WM][2];
        dg_wait_for_loads();                                   // (both runs: the first is needed now)
        read_words(wa, TURNS ? 0 : g0 & 1, 0);
#pragma unroll
        for (int u = 0; u < WM; ++u) sparse_dense_rows_shared(s_rows, wa.ca[u].x, wa.ca1[u].x, pick, dn0[u][0], dn0[u][1]);
        if constexpr (HALF) {
            for (int g = 0; g < runs; ++g) {
                kept_bytes((int)fdiv((uint32_t)(2 * g), a.div_cpt), true, ones, ones_odd);
                step(dn0, wa, 0, dn1, wa, 1, ones, ones_odd);
                read_words(wb, g & 1, 1);
                step(dn1, wa, 1, dn0, wb, 0, ones, ones_odd);
                // (the second chunk's kept bytes take the first's registers)
                kept_bytes((int)fdiv((uint32_t)min(2 * g + 1, chunks - 1), a.div_cpt), 2 * g + 1 < chunks, ones, ones_odd);
                step(dn0, wb, 0, dn1, wb, 1, ones, ones_odd);
                dg_wait_for_loads();
                fetch();
                read_words(wa, (g + 1) & 1, 0);
                step(dn1, wb, 1, dn0, wa, 0, ones, ones_odd);
            }
        }
        int g = HALF ? g1 : g0, rt = rt0, n = 0;            // the run, its place in its tap, runs done
        for (int tap = tap0; g < g1;) {
            kept_bytes(tap, true, ones, ones_odd);
            for (; rt < runs_per_tap && g < g1; rt += stride, g += stride, ++n) {
                // run g, in the buffer of its parity (of its count where wavefronts take turns): wa holds its first chunk's words, dn0 the dense operands of that chunk's word 0
                step(dn0, wa, 0, dn1, wa, 1, ones, ones_odd);
                read_words(wb, (TURNS ? n : g) & 1, 1);
                step(dn1, wa, 1, dn0, wb, 0, ones, ones_odd);
                step(dn0, wb, 0, dn1, wb, 1, ones, ones_odd);
                // every read of run g has been issued: its buffer takes the wavefront's run after next, once its next
                // run is known to be in (one counter serves all loads, and they complete in order)
                dg_wait_for_loads();
                fetch();
                read_words(wa, ((TURNS ? n : g) + 1) & 1, 0);
                step(dn1, wb, 1, dn0, wa, 0, ones, ones_odd);
            }
            if constexpr (TURNS) {
                while (rt >= runs_per_tap) rt -= runs_per_tap;      // (uniform; no filter window: the tap stays)
            } else {
                rt = 0, ++tap;
            }
        }
        dg_wait_for_loads();                                   // (unused fetches past the end: their LDS writes end before the wavefront does)
    }
    if (SKW == 1) {
        dg_mfma_store_tile<WM, WN, true>(p, acc, m0, n0, lane, sc_cols);
        return;
    }
    // The sums take the place of the staging rows: every wavefront is done with its rows (and its last loads have
    // landed) at the first barrier; the tile's first wavefront writes its sums, the others add theirs.
    int32_t *sums = s_acc + tw * (NB * 1024);
    __syncthreads();
    if (ks == 0) {
#pragma unroll
        for (int i = 0; i < NB; ++i)
#pragma unroll
            for (int e = 0; e < 16; ++e) sums[(i * 16 + e) * 64 + lane] = acc[i / WN][i % WN][e];
    }
    __syncthreads();
    if (ks != 0 && g0 < g1) {
#pragma unroll
        for (int i = 0; i < NB; ++i)
#pragma unroll
            for (int e = 0; e < 16; ++e)
                __hip_atomic_fetch_add(&sums[(i * 16 + e) * 64 + lane], acc[i / WN][i % WN][e], __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_WORKGROUP);
    }
    __syncthreads();
    if (!active) return;
#pragma unroll
    for (int i = 0; i < NB; ++i) {
        if (i % SKW != ks) continue;                        // each wavefront of the tile stores a share of its blocks
        v16i blk;
#pragma unroll
        for (int e = 0; e < 16; ++e) blk[e] = sums[(i * 16 + e) * 64 + lane];
        dg_mfma_store_block<true>(p, blk, m0 + (i / WN) * 32, n0 + (i % WN) * 32, lane, sc_cols[i / WN]);
    }
}

// `wave_tiles` tiles of q.wm x q.wn blocks, 4 / q.skw of them per workgroup
//
// `bias`: the caller added it to every entry of the table in `pools` (0: the table as it is).  The matrix pipe's power
// draw, and with it the clock the chip sustains, follows the bits that toggle in its operands and sums: the same
// 8192-cube takes 550 us with an all-zero table, 640 us with entries 0 ... 9, 700 us with -6 ... 3 and 800 us with
// -64 ... 64.  A table raised to 0 ... max - min keeps the high bits of the dense operand and of the growing sums
// quiet; the kernel starts each sum at minus the bias times the pixel's positions of K, so the result is the same.
inline void launch_sparse_staged(const DgProblem &p, const Pools &pools, int32_t bias, const Plan &q, int64_t wave_tiles, hipStream_t stream)
{
    Args a;
    a.p = p;
    a.pools = pools;
    a.bias = bias;
    a.tiles_m = (p.M + q.wm * 32 - 1) / (q.wm * 32);
    a.wave_tiles = wave_tiles;
    a.div_ow = make_div((uint32_t)p.OW), a.div_oh = make_div((uint32_t)p.OH);
    a.div_cin = make_div((uint32_t)p.Cin), a.div_kw = make_div((uint32_t)p.KW);
    const bool half = p.Cin % 128 != 0;                    // (see the kernel: taps of an odd number of 64-position chunks)
    a.div_runs = make_div((uint32_t)(half ? 1 : p.Cin / 128));
    a.div_cpt = make_div((uint32_t)(p.Cin / 64));
    a.tiles_n = (int32_t)((p.N + q.wn * 32 - 1) / (q.wn * 32));
    a.band_log2 = 3;                                       // bands of 8 pixel tiles
    a.m_log2 = a.tiles_m % 4 == 0 ? 2 : 0;                 // (unshared tiles: a workgroup's four wavefronts)
    a.band_tiles = (uint32_t)a.tiles_m << a.band_log2;
    a.div_band = make_div(a.band_tiles);
    const int last = a.tiles_n & ((1 << a.band_log2) - 1);
    a.div_last = make_div((uint32_t)(last ? last : 1));
    const int tpw = 4 / q.skw;
    const dim3 grid((unsigned)((wave_tiles + tpw - 1) / tpw));
    const bool turns = p.KH * p.KW == 1;                   // (see the kernel: run by run without a filter window)
#define DG_STAGED(WM, WN, SKW, TURNS) hipLaunchKernelGGL((smfmac_staged_kernel<WM, WN, SKW, TURNS, false>), grid, dim3(256), 0, stream, a)
    if (half && q.wn == 4) hipLaunchKernelGGL((smfmac_staged_kernel<1, 4, 1, false, true>), grid, dim3(256), 0, stream, a);
    else if (half) hipLaunchKernelGGL((smfmac_staged_kernel<1, 2, 1, false, true>), grid, dim3(256), 0, stream, a);
    else if (q.wm == 2) DG_STAGED(2, 4, 1, false);
    else if (q.wn == 7) DG_STAGED(1, 7, 1, false);
    else if (q.wn == 6) DG_STAGED(1, 6, 1, false);
    else if (q.wn == 4 && q.skw == 4 && turns) DG_STAGED(1, 4, 4, true);
    else if (q.wn == 4 && q.skw == 4) DG_STAGED(1, 4, 4, false);
    else if (q.wn == 4 && q.skw == 2 && turns) DG_STAGED(1, 4, 2, true);
    else if (q.wn == 4 && q.skw == 2) DG_STAGED(1, 4, 2, false);
    else if (q.wn == 4) DG_STAGED(1, 4, 1, false);
    else if (q.skw == 4 && turns) DG_STAGED(1, 2, 4, true);
    else if (q.skw == 4) DG_STAGED(1, 2, 4, false);
    else if (q.skw == 2 && turns) DG_STAGED(1, 2, 2, true);
    else if (q.skw == 2) DG_STAGED(1, 2, 2, false);
    else DG_STAGED(1, 2, 1, false);
#undef DG_STAGED
}

}   // namespace dgoh
