// Host side of the one-hot matrix-core kernels (dense and sparse instruction) and of the decode-and-multiply comparison
// built in the same frame (dg_onehot_kernel.h): which problems they take, which of their shapes runs a given problem,
// and the launch.
#include <cstdlib>
#include <cstring>

#include "dg_onehot_kernel.h"

namespace {

using dgoh::Plan;

enum Mode { TABLE, DECODE, SPARSE };      // one-hot selection by the dense MFMA; decode-and-multiply; selection by the sparse MFMA

int per_byte(const dg_lut *lut) { return lut->bits == 2 ? 4 : 2; }

// VALU and matrix-pipe cycles of one step of a decoding wavefront's tile, whichever is more: each operand costs about
// 11 (weights) or 15 (activations, with the padding mask) instructions of 4 cycles, each MFMA 32 cycles
double decode_step_cycles(int wm, int wn)
{
    const double valu = 4.0 * (11 * wm + 15 * wn), mfma = 32.0 * wm * wn;
    return 1.08 * (valu > mfma ? valu : mfma);
}

int64_t tile_count(const DgProblem &p, int wm, int wn)
{
    return ((int64_t)(p.M + wm * 32 - 1) / (wm * 32)) * (((int64_t)p.N + wn * 32 - 1) / (wn * 32));
}

bool fits_int8(const dg_lut *lut) { return lut->min_entry >= -128 && lut->max_entry <= 127; }

// the tiled kernels address the packed activations with 32-bit byte offsets
bool offsets_fit(const DgProblem &p, int codes_per_byte)
{
    const int64_t images = (int64_t)p.N / ((int64_t)p.OH * p.OW);
    return images * p.H * p.W * (p.Cin / codes_per_byte) < ((int64_t)1 << 31);
}

// `tile` > 0 fixes an unshared tile of that many blocks' width instead of modelling (see sparse_plan)
Plan plan_for(const dg_lut *lut, const DgProblem &p, Mode mode, int tile = 0)
{
    const bool decode = mode == DECODE;
    Plan q;
    q.staged = false;
    q.decode = decode;
    q.two = mode == TABLE && !fits_int8(lut);              // two int8 planes; a tile is then 32 rows high, not 64
    const int wm = q.two ? 1 : 2;
    q.wm = wm;
    // a lane half reads 4*ch packed bytes of one filter tap per chunk
    const int tap_bytes = p.Cin / per_byte(lut);
    q.ch = tap_bytes % 32 == 0 ? 4 : (tap_bytes % 16 == 0 ? 2 : 1);
    if (lut->bits == 4 && q.ch == 4) q.ch = 2;             // (a 4-word chunk of 4-bit codes would be 32 MFMA steps)
    if (mode == SPARSE && q.ch == 4) q.ch = 2;             // (the sparse instruction's widest tile has no registers for 4)
    q.chunks = (p.K / per_byte(lut)) / (8 * q.ch);
    q.wn = 1, q.skw = 1, q.S = 1, q.cpw = q.chunks;
    q.split = false;
    // the split-K kernel's shape: about 2048 wavefronts in all (3072 for K = 2304 ... 4608), at most 16 per workgroup, whole chunks each
    const int64_t blocks11 = tile_count(p, 1, 1);
    // (3072 from K = 2304: a wavefront's share of a long K is a chain of load latencies, and 12 wavefronts per block
    // instead of 9 measured 5.6 -> 5.2 us on 14x14x256 -> 256 3x3 at batch 4 and 8.4 -> 7.1 us on 7x7x512 -> 512 3x3 at
    // batch 8; with K = 2048 and below the larger target was slower, 4.65 -> 5.15 us, and so it was on the 8192 x 1 x 8192
    // GEMM, whose weights stream from memory: 10.5 -> 11.6 us)
    int64_t target = p.K >= 2304 && p.K <= 4608 ? 3072 : 2048;
    if (const char *e = dg_override("DG_ONEHOT_WAVES")) target = atoi(e) > 0 ? atoi(e) : target;   // tuning override
    int S = (int)((target + blocks11 - 1) / blocks11);
    S = S < 1 ? 1 : (S > 16 ? 16 : S);
    const int S_wanted = S;
    if (S > q.chunks) S = q.chunks;
    const int split_cpw = (q.chunks + S - 1) / S, split_S = (q.chunks + split_cpw - 1) / split_cpw;

    // Which kernel and shape: the one with the least modelled time on the busiest SIMD, in cycles.  A SIMD's wavefronts
    // share its matrix pipe, so the time of a plan is (wavefronts per SIMD, rounded up) x (32x32 blocks per tile) x
    // (MFMA steps of a wavefront's share of K) x (cycles per MFMA), plus what no other wavefront hides: a prologue, the
    // last tile's stores, and the LDS exchange where wavefronts share a tile.  Sharing a tile (2 or 4 wavefronts
    // splitting K) fills SIMDs that the tiles alone would leave idle; 7 blocks wide fits the 56 x 56 and 28 x 28 images
    // of ImageNet networks (N = 49 * 2^k) where 4 wide leaves the last round of tiles half empty.  The constants are a
    // least-regret fit to timings of 78 layer shapes x 12 plans with 2-bit codes (the plan chosen is within 14 % of
    // the best measured one on each, 1.3 % on average); ties go to the wider, less shared plan.
    static const int widths[4] = {7, 4, 2, 1};
    const int64_t simds = dg_simd_count();
    const bool can_share = lut->bits == 2 && !q.two;       // (the comparison takes 2-bit codes only)
    // (the wider codes and two-plane tables, with 2 to 4 times the MFMA work per load, keep the constants of an earlier
    // fit without sharing, under which their measured times are better: 32 cycles per MFMA, 33 and 42 for the two
    // narrowest tiles, 3000 + 600 per block for prologue and stores)
    static const double fitted_cycles[4] = {37.7, 28.9, 29.5, 34.0}, plain_cycles[4] = {32.0, 32.0, 33.0, 42.0};
    const double *mfma_cycles = can_share ? fitted_cycles : plain_cycles;
    // matrix instructions per 32 x 32 block: one per 32 positions decoding, per 32 / L selecting, per 16 on the sparse one
    const double steps = decode ? p.K / 32.0 : (mode == SPARSE ? p.K / 16.0 : (double)p.K * (1 << lut->bits) / 32.0);
    // Sharing fills SIMDs that tiles alone would leave idle.  With two or more tiles of a width per SIMD there is nothing
    // to fill, and what the model then sees in sharing is the rounding of its own queue lengths (6.125 tiles per SIMD
    // count as 7, 24.5 quarter tiles as 6.25): measured without it on the layers where the model had chosen it,
    // 56x56x512 -> 1024 at batch 64 379 -> 246 us, 56x56x128 -> 256 3x3 at batch 32 79 -> 58 us, 224x224x64 -> 64 3x3 at
    // batch 8 55 -> 40 us, 56x56x256 -> 256 3x3 at batch 32 112 -> 94 us.  DG_ONEHOT_SHARE_BELOW: tiles per SIMD from
    // which a tile width is not shared (default 2).
    int64_t share_below = 2;
    if (const char *e = dg_override("DG_ONEHOT_SHARE_BELOW")) share_below = atoi(e) > 0 ? atoi(e) : share_below;
    double best = 0.0;
    bool first = true;
    for (int i = 0; i < 4; ++i)
        for (int skw = 1; skw <= (can_share ? 4 : 1); skw *= 2) {
            const int wn = widths[i];
            if (skw > q.chunks || (wn == 7 && skw == 2)) continue;      // (two 64x224 tiles of sums exceed 64 KB of LDS)
            if (skw > 1 && tile_count(p, wm, wn) >= share_below * simds) continue;
            if (wn == 7 && mode == SPARSE) continue;                    // (14 blocks of sparse-instruction sums exceed the VGPRs)
            if (wn == 7 && decode) continue;                            // (measured slower than 64x128 when decoding, shared or not)
            const int64_t per_simd = (tile_count(p, wm, wn) * skw + simds - 1) / simds;
            const double lone = !can_share ? 1.0 : (per_simd == 1 ? 0.84 : (per_simd == 2 ? 0.78 : 1.0));   // (rounding up overstates short queues)
            double cost = (double)per_simd * 2 * wn * (steps / skw) * mfma_cycles[i] * lone;
            if (decode) cost = (double)per_simd * (steps / skw) * decode_step_cycles(2, wn) * lone;
            cost += can_share ? 2670.0 + 350.0 * 2 * wn / skw : 3000.0 + 600.0 * 2 * wn;
            if (skw > 1) cost += 955.0 + 147.0 * 2 * wn;
            if (first || cost < best * 0.999) best = cost, q.wn = wn, q.skw = skw, first = false;
        }
    // the comparison's own 128 x 128 tile, one wavefront per SIMD with 64 KB of sums to store at the end: for long
    // reductions without a filter window (8192-cube 500 against 528 us for 64 x 128, 4096-cube 69.7 against 70.9).  With a
    // 3x3 window it measured 1.2 - 2.7 times the 64 x 128 tile's time on six layers, with K = 512 and 1024 1.2 - 2.5
    // times on five, none of which the model sees.
    if (decode && p.M > 64 && p.KH * p.KW == 1 && p.K >= 4096) {
        const int64_t per_simd = (tile_count(p, 4, 4) + simds - 1) / simds;
        const double cost = (double)per_simd * steps * decode_step_cycles(4, 4) + 2670.0 + 350.0 * 16;
        if (cost < best * 0.999) best = cost, q.wm = 4, q.wn = 4, q.skw = 1;
    }
    if (can_share) {
        const int64_t per_simd = (blocks11 * split_S + simds - 1) / simds;
        const double cost = (double)per_simd * (steps * split_cpw / q.chunks) * (decode ? decode_step_cycles(1, 1) : 50.6) + 3370.0;
        q.split = q.chunks > 1 && cost < best;
    } else {
        // other code widths and two-plane tables (not in the fit): split K when there are too few 64 x 32 tiles to give
        // every SIMD a wavefront, or barely enough and a long K to walk
        const int64_t t21 = tile_count(p, wm, 1);
        q.split = (t21 < simds / 2 || (t21 < simds && q.chunks >= 32)) && q.chunks > 1;
    }
    if (tile > 0) q.split = false, q.wm = wm, q.wn = tile, q.skw = 1;
    // DG_ONEHOT_PLAN = split | <wn> | <wn>k<skw> (wn = 1, 2, 4, 7; skw = 1, 2, 4) | 44 (the comparison's 128 x 128 tile)
    // overrides the choice (tuning, and tests that must reach every plan)
    if (const char *force = dg_override("DG_ONEHOT_PLAN")) {
        const int v = atoi(force);
        if (force[0] == 's') q.split = true;
        else if (v == 44 && decode) q.split = false, q.wm = 4, q.wn = 4, q.skw = 1;
        else if (v == 1 || v == 2 || v == 4 || (v == 7 && mode != SPARSE)) {
            int k = 1;
            if (const char *at = strchr(force, 'k')) k = atoi(at + 1);
            q.split = false;
            q.wm = wm;
            q.wn = v;
            q.skw = (can_share && (k == 2 || k == 4) && k <= q.chunks && !(v == 7 && k == 2)) ? k : 1;
        }
    }
    if (q.split) q.cpw = split_cpw, q.S = split_S, q.wm = wm;
    // The dense instruction's chunks of 128 positions cap the wavefronts per tile at K / 128 and make their shares of K
    // coarse.  It walks K in chunks of 64 instead: up to K = 512 where at least twice as many wavefronts are wanted
    // (measured at batch 1: K = 256, four wavefronts instead of two, 3.8 -> 3.1 us on five layers of ResNet-50; K = 384
    // 3.6 -> 3.1; K = 512, eight instead of four, 3.3 -> 3.1), and where the finer shares give more wavefronts, up to 12
    // (K = 2304, 12 of 3 chunks instead of 9 of 2: 5.5 -> 5.1 us, the one-call step 7.1 -> 6.2; K = 768, 12 instead of
    // 6: the step 4.5 -> 4.05).  More than 12 were slower (K = 1024, 16 for 8: 3.5 -> 3.9; K = 4608, 15 for 12: 6.9 -> 8.0).
    // DG_ONEHOT_CH2_MAX, DG_ONEHOT_CH2_SMAX: the most 128-position chunks for the first rule (default 4; 0: never),
    // the most wavefronts for the second (default 12; 0: never).
    int ch2_max = 4, s_max = 12;
    if (const char *e = dg_override("DG_ONEHOT_CH2_MAX")) ch2_max = atoi(e);
    if (const char *e = dg_override("DG_ONEHOT_CH2_SMAX")) s_max = atoi(e);
    if (q.split && mode != SPARSE && can_share && q.ch == 4) {
        const int chunks2 = 2 * q.chunks, S2 = S_wanted > chunks2 ? chunks2 : S_wanted;
        const int cpw2 = (chunks2 + S2 - 1) / S2, waves2 = (chunks2 + cpw2 - 1) / cpw2;
        if ((q.chunks <= ch2_max && S_wanted >= 2 * q.chunks) || (waves2 > q.S && waves2 <= s_max))
            q.ch = 2, q.chunks = chunks2, q.cpw = cpw2, q.S = waves2;
    }
    if (lut->bits == 4 && q.wn == 7) q.ch = 1;             // (the 2-word kernel of this tile is not built: see launch_ch)
    // (the sparse instruction's narrower unshared tiles do have the registers for 4-word chunks)
    if (mode == SPARSE && !q.split && q.skw == 1 && q.wn <= 2 && tap_bytes % 32 == 0) q.ch = 4, q.chunks /= 2;
    return q;
}

}   // namespace

bool dg_onehot_supports(const dg_lut *lut, const DgProblem &p)
{
    if (lut->dtype == DG_LUT_F32) return false;
    // MFMA operands are int8: wider entries take two planes, T = 256 * hi + lo (2-bit codes only, hi within int8)
    if (!fits_int8(lut) && (lut->bits != 2 || lut->max_entry > 127 * 256 + 127)) return false;
    if (p.Cin % (8 * per_byte(lut)) != 0) return false;                // a lane half reads whole words of one tap
    if (!offsets_fit(p, per_byte(lut))) return false;
    const Plan q = plan_for(lut, p, TABLE);
    if ((uintptr_t)p.Wp % (4 * q.ch) != 0 || (uintptr_t)p.Xp % (4 * q.ch) != 0) return false;
    return true;
}

namespace {

// The sparse instruction's one-hot operand is its row operand, so the activations sit on the MFMA rows and the channel
// axis m on its columns: right for outputs whose stride-1 axis is m (NHWC).  A plain GEMM with n contiguous is the
// same problem transposed -- activations as "weights", the table transposed -- and is run that way.
bool sparse_transposes(const DgProblem &p)
{
    return p.stride_cn == 1 && p.stride_cm != 1;
}

bool sparse_can_transpose(const DgProblem &p)
{
    return p.H == 1 && p.W == 1 && p.KH == 1 && p.KW == 1 && p.sh == 1 && p.sw == 1 && p.ph == 0 && p.pw == 0 &&
           p.scale == nullptr && p.Qp == nullptr;
}

DgProblem sparse_problem(const DgProblem &p)
{
    if (!sparse_transposes(p)) return p;
    DgProblem t = p;
    t.M = p.N, t.N = p.M;
    t.Wp = p.Xp, t.Xp = p.Wp;
    t.stride_cm = p.stride_cn, t.stride_cn = p.stride_cm;
    return t;
}

// Measured on 29 layer shapes: where the dense-instruction planner picks an unshared tile at least 64 columns wide, the
// sparse instruction with the same tile (at most 128 wide: its sums must stay in the vector registers) is 2 - 24 %
// faster; on 64 x 32 tiles, shared tiles and the split-K kernel it is not (its weight operand costs more VALU and LDS
// work per matrix instruction, which narrow tiles do not amortise).  `t` is the problem as the sparse kernel runs it.
int sparse_tile_hint(const dg_lut *lut, const DgProblem &t)
{
    if (!fits_int8(lut) || lut->bits != 2) return 0;
    const Plan dense = plan_for(lut, t, TABLE);
    if (dense.split || dense.skw != 1 || dense.wn < 2) return 0;
    return dense.wn > 4 ? 4 : dense.wn;
}

// The tiled kernel with operands staged through LDS (dg_sparse_staged_kernel.h) takes the unshared tiles of layers
// whose filter taps are whole 32-byte runs of packed codes, or -- its two narrow tiles, unshared -- whole 16-byte chunks.
// DG_ONEHOT_STAGED=0 keeps the direct loads (A/B measurement).
bool staged_takes(const DgProblem &t)
{
    if (t.Cin % 64 != 0 || (uintptr_t)t.Wp % 16 != 0 || (uintptr_t)t.Xp % 16 != 0) return false;
    if (const char *e = dg_override("DG_ONEHOT_STAGED")) return atoi(e) != 0;
    return true;
}

// The staged kernel's tiles are one block of 32 channels high -- the weight operand of a block, the expensive one,
// then serves every pixel block of the tile -- and 64, 128 or 192 pixels wide; at equal area they were measured 3 - 20 %
// faster than the 64-row tiles on every layer tried, so a plan made for the 64-row tiles is run on the tile of the
// same area (64 x 32 -> 32 x 64, 64 x 64 -> 32 x 128, with the same sharing of K).  Beside 64 x 128 there are 32 x 192
// and 32 x 224, taken where they leave the busiest SIMD fewer blocks to do (the 1568 pixel blocks x 8 channel blocks of
// the 56x56x256 -> 256 layer at batch 16: 1568 tiles of 64 x 128 are two per SIMD for half the SIMDs, 16 blocks; 1792
// tiles of 32 x 224 are 14; measured 54.6 and 49.2 us).
// DG_ONEHOT_PLAN = 12 | 14 [k2 | k4] | 16 | 17 | 24 forces a staged tile (32 x 64, 32 x 128, 32 x 192, 32 x 224,
// 64 x 128); the other values of that override force the direct-load kernels.
Plan sparse_plan(const dg_lut *lut, const DgProblem &t)
{
    Plan q = plan_for(lut, t, SPARSE, sparse_tile_hint(lut, t));
    q.staged = false;
    if (!staged_takes(t)) return q;
    const bool half = t.Cin % 128 != 0;                     // only the unshared 32 x 64 and 32 x 128 tiles
    if (const char *force = dg_override("DG_ONEHOT_PLAN")) {
        const int v = atoi(force), k = strstr(force, "k4") ? 4 : (strstr(force, "k2") ? 2 : 1);
        if (half && ((v != 12 && v != 14) || k != 1)) return q;
        if (v == 12 || v == 14) q.staged = true, q.split = false, q.wm = 1, q.wn = v == 12 ? 2 : 4, q.skw = k, q.ch = 2;
        if (v == 16 || v == 24) q.staged = true, q.split = false, q.wm = v == 16 ? 1 : 2, q.wn = v == 16 ? 6 : 4, q.skw = 1, q.ch = 2;
        if (v == 17) q.staged = true, q.split = false, q.wm = 1, q.wn = 7, q.skw = 1, q.ch = 2;
        return q;
    }
    if (q.split || q.wm != 2) return q;
    // Wavefronts that share a tile need two runs of K each: with one (K = 512 shared by four), the 28x28x512 -> 128 and
    // 7x7x512 -> 2048 layers at batch 8 measured 8 and 11 % slower than the dense instruction's direct-load kernel;
    // with two (K = 1024 by four) from equal to 6 % faster.
    if (q.skw > 1 && t.K / 128 < 2 * q.skw) return q;
    if (half) {
        // Layers with a filter window and three or more chunks per tap, where the planner does not share tiles or
        // there are so many tiles that sharing is not needed to fill the chip: the wider of the two tiles that leaves
        // every SIMD more than one tile.  Measured against the direct loads, batch 32: 28x28x192 -> 96 3x3 18.4
        // against 20.9 us, 28x28x320 -> 320 3x3 43.4 against 50.0, 56x56x192 -> 192 3x3 67.4 against 82.7 (shared
        // 64 x 64 tiles; unshared 70.3).  Elsewhere the direct loads stay: with 64 channels (seven 3x3 layers) the
        // staged tiles measured within +-2 %, on GEMMs and 1x1 layers from 13 % slower to 6 % faster, with the few
        // tiles of the planner's shared plans 6 - 40 % slower.
        const int64_t simds = dg_simd_count();
        if (t.KH * t.KW == 1 || t.Cin < 192) return q;
        if (q.skw != 1 && tile_count(t, 1, 4) <= 4 * simds) return q;
        if (tile_count(t, 1, 4) > simds) q.staged = true, q.wm = 1, q.wn = 4, q.skw = 1, q.ch = 2;
        else if (q.skw == 1 && tile_count(t, 1, 2) > simds) q.staged = true, q.wm = 1, q.wn = 2, q.ch = 2;
    } else if (q.wn <= 2) {
        q.staged = true, q.wm = 1, q.wn *= 2, q.ch = 2;
        // 32 x 224 in place of 32 x 128 on layers with a filter window and two or more such tiles per SIMD, where it leaves
        // the busiest SIMD no more blocks: 5 - 7 % faster on four 3x3 layers (56x56x256 -> 256 at batch 32 93.4 -> 88.4 us,
        // 112x112x128 -> 128 at batch 16 56.8 -> 53.6); with one tile per SIMD or less it was 8 % slower, without a
        // window no different.
        const int64_t simds = dg_simd_count();
        if (q.wn == 4 && q.skw == 1 && t.KH * t.KW > 1 && tile_count(t, 1, 7) >= 2 * simds &&
            (tile_count(t, 1, 7) + simds - 1) / simds * 7 <= (tile_count(t, 1, 4) + simds - 1) / simds * 4)
            q.wn = 7;
    } else if (q.wn == 4 && q.skw == 1) {
        // 64 x 128, 32 x 192 or 32 x 224: the one that leaves the busiest SIMD the fewest blocks (ties: 32 x 192, which
        // at equal work per SIMD measured 2 % faster than the others, then 64 x 128)
        const int64_t simds = dg_simd_count();
        const int64_t blocks_24 = (tile_count(t, 2, 4) + simds - 1) / simds * 8;
        const int64_t blocks_16 = (tile_count(t, 1, 6) + simds - 1) / simds * 6;
        const int64_t blocks_17 = (tile_count(t, 1, 7) + simds - 1) / simds * 7;
        q.staged = true, q.ch = 2;
        if (blocks_16 <= blocks_24 && blocks_16 <= blocks_17) q.wm = 1, q.wn = 6;
        else if (blocks_17 < blocks_24) q.wm = 1, q.wn = 7;
    }
    return q;
}

bool sparse_staged(const DgProblem &, const Plan &q) { return q.staged; }

}   // namespace

bool dg_sparse_preferred(const dg_lut *lut, const DgProblem &p)
{
    if (!dg_sparse_supports(lut, p) || dg_override("DG_ONEHOT_PLAN") != nullptr) return false;
    const DgProblem t = sparse_problem(p);
    if (sparse_tile_hint(lut, t) > 0) return true;
    // the staged kernel, where the layer is its case and large enough for tiles, was faster than the dense
    // instruction's kernels on all 9 such layers measured (by 7 - 25 %)
    const Plan sparse = sparse_plan(lut, t);
    if (sparse.staged) return true;
    // Also where the dense-instruction planner shares tiles at least 64 columns wide and there are 384 of them or more:
    // the sparse kernel in the shape its own planner picks was 1 - 15 % faster on all 9 such layers measured (it lost
    // on shared 64 x 32 tiles, on 200 shared 64 x 64 tiles, and with one-word chunks, Cin % 64 != 0).
    const Plan dense = plan_for(lut, t, TABLE);
    if (fits_int8(lut) && t.Cin % 64 == 0 && !dense.split && dense.skw > 1 && dense.wn >= 2 && tile_count(t, 2, dense.wn) >= 384)
        return true;
    // And on unshared 64 x 32 tiles where there is more than one per SIMD: 8 - 13 % faster on eight layers measured (3x3
    // layers with 64 channels at 1568 tiles, 1x1 layers and GEMMs with K = 320 and 576 at 1764 and 2048); at 1024 and
    // 784 tiles the two were within 2 % of each other either way.
    return fits_int8(lut) && t.Cin % 64 == 0 && !dense.split && dense.skw == 1 && dense.wn == 1 &&
           tile_count(t, 2, 1) > dg_simd_count();
}

bool dg_sparse_supports(const dg_lut *lut, const DgProblem &p)
{
    if (lut->dtype == DG_LUT_F32 || lut->bits != 2 || !fits_int8(lut)) return false;
    if (p.Cin % 32 != 0) return false;                                 // a lane half reads whole words of one tap
    if (sparse_transposes(p) && !sparse_can_transpose(p)) return false;
    const DgProblem t = sparse_problem(p);
    if (!offsets_fit(t, 4)) return false;
    const Plan q = sparse_plan(lut, t);
    if ((uintptr_t)t.Wp % (4 * q.ch) != 0 || (uintptr_t)t.Xp % (4 * q.ch) != 0) return false;
    return true;
}

const char *dg_sparse_config_name(const dg_lut *lut, const DgProblem &p)
{
    static const char *const split_names[17] = {
        "", "onehot_smfmac_splitk_s1", "onehot_smfmac_splitk_s2", "onehot_smfmac_splitk_s3", "onehot_smfmac_splitk_s4",
        "onehot_smfmac_splitk_s5", "onehot_smfmac_splitk_s6", "onehot_smfmac_splitk_s7", "onehot_smfmac_splitk_s8",
        "onehot_smfmac_splitk_s9", "onehot_smfmac_splitk_s10", "onehot_smfmac_splitk_s11", "onehot_smfmac_splitk_s12",
        "onehot_smfmac_splitk_s13", "onehot_smfmac_splitk_s14", "onehot_smfmac_splitk_s15", "onehot_smfmac_splitk_s16"};
    static const char *const tile_names[3][4] = {
        {"onehot_smfmac_64x224", "onehot_smfmac_64x128", "onehot_smfmac_64x64", "onehot_smfmac_64x32"},
        {"", "onehot_smfmac_64x128_k2", "onehot_smfmac_64x64_k2", "onehot_smfmac_64x32_k2"},
        {"onehot_smfmac_64x224_k4", "onehot_smfmac_64x128_k4", "onehot_smfmac_64x64_k4", "onehot_smfmac_64x32_k4"}};
    const DgProblem t = sparse_problem(p);
    const Plan q = sparse_plan(lut, t);
    if (q.split) return split_names[q.S];
    if (q.staged) {
        static const char *const staged_names[3][2] = {
            {"onehot_smfmac_staged_32x64", "onehot_smfmac_staged_32x128"},
            {"onehot_smfmac_staged_32x64_k2", "onehot_smfmac_staged_32x128_k2"},
            {"onehot_smfmac_staged_32x64_k4", "onehot_smfmac_staged_32x128_k4"}};
        if (q.wm == 2) return "onehot_smfmac_staged_64x128";
        if (q.wn == 7) return "onehot_smfmac_staged_32x224";
        if (q.wn == 6) return "onehot_smfmac_staged_32x192";
        return staged_names[q.skw == 4 ? 2 : (q.skw == 2 ? 1 : 0)][q.wn == 4 ? 1 : 0];
    }
    return tile_names[q.skw == 4 ? 2 : (q.skw == 2 ? 1 : 0)][q.wn == 7 ? 0 : (q.wn == 4 ? 1 : (q.wn == 2 ? 2 : 3))];
}

dg_status dg_launch_sparse(const dg_lut *lut, const DgProblem &p0, hipStream_t stream)
{
    const bool transposed = sparse_transposes(p0);
    const DgProblem p = sparse_problem(p0);
    const Plan q = sparse_plan(lut, p);
    // pool word w = the table row of "weight" code w, bytes over the "activation" code (the transposed problem swaps them)
    dgoh::Pools pools;
    for (int i = 0; i < 64; ++i) pools.w[i] = 0;
    for (int w = 0; w < 4; ++w)
        for (int v = 0; v < 4; ++v) {
            const int T = transposed ? lut->entry[(v << 2) | w] : lut->entry[(w << 2) | v];
            pools.w[w] |= (uint32_t)(uint8_t)(int8_t)T << (8 * v);
        }
    const int64_t blocks11 = tile_count(p, 1, 1), wave_tiles = tile_count(p, q.wm, q.wn);
    if ((q.split ? blocks11 : wave_tiles) > INT32_MAX)
        return dg_fail(DG_ERR_UNSUPPORTED, "sparse one-hot kernel: too many tiles for one grid");
    using namespace dgoh;
    if (q.split) {
        unit_split_b20_t1(p, pools, q, blocks11, stream);
        return dg_check_launch("onehot_splitk_kernel<20>");
    }
    if (sparse_staged(p, q)) {
        // The staged kernel takes the table raised to 0 ... max - min where that fits a signed byte and the raised sums
        // fit 32 bits (dg_sparse_staged_kernel.h: fewer toggling bits, a higher sustained clock) -- on problems large
        // enough to heat the chip; shorter kernels only pay the longer start.  DG_STAGED_BIAS: 0 keeps the table as it
        // is, 1 raises it whatever the size (tests, A/B measurement).
        const int lo = lut->min_entry, hi = lut->max_entry;
        const bool fits = hi - lo <= 127 && (int64_t)(hi - lo > abs(lo) ? hi - lo : abs(lo)) * p.K <= INT32_MAX;
        bool raise = 2.0 * (double)p.M * (double)p.N * (double)p.K >= 2e10;
        if (const char *e = dg_override("DG_STAGED_BIAS")) raise = atoi(e) != 0;
        const int32_t bias = fits && raise ? -lo : 0;
        if (bias != 0)
            for (int w = 0; w < 4; ++w) {
                uint32_t word = 0;
                for (int v = 0; v < 4; ++v) word |= (uint32_t)(uint8_t)(int8_t)((int8_t)(pools.w[w] >> (8 * v)) + bias) << (8 * v);
                pools.w[w] = word;
            }
        unit_sparse_staged(p, pools, bias, q, wave_tiles, stream);
        return dg_check_launch("smfmac_staged_kernel");
    }
    static const MainFn main_units[3] = {unit_main_b20_t1_k1, unit_main_b20_t1_k2, unit_main_b20_t1_k4};
    main_units[q.skw == 4 ? 2 : (q.skw == 2 ? 1 : 0)](p, pools, q, wave_tiles, stream);
    return dg_check_launch("onehot_mfma_kernel<20>");
}

// ---- weights stationary in registers on the sparse instruction (dg_sparse_ws_kernel.h): short reductions without filter window

namespace {

// `packed`: the activations are packed (then a 1x1 convolution may have a stride: a lane works out its pixel's row)
bool sparse_ws_takes(const dg_lut *lut, const DgProblem &p, bool packed = true)
{
    if (lut->dtype == DG_LUT_F32 || lut->bits != 2 || !fits_int8(lut)) return false;
    // the whole dense operand of 32 rows stays in registers (K = 512: all 512 of a lone wavefront's, packed activations only)
    if (p.K != 64 && p.K != 128 && p.K != 256 && !(p.K == 512 && packed)) return false;
    // every "pixel" is one contiguous row of K codes: a GEMM, or a 1x1 convolution without padding
    if (p.KH != 1 || p.KW != 1 || p.ph != 0 || p.pw != 0) return false;
    if ((p.sh != 1 || p.sw != 1) && (!packed || sparse_transposes(p))) return false;
    if (sparse_transposes(p) && !sparse_can_transpose(p)) return false;
    const DgProblem t = sparse_problem(p);
    if (t.stride_cm != 1) return false;                               // the 32 channels of a lane half are stored side by side
    if ((uintptr_t)t.Wp % 16 != 0 || (uintptr_t)t.Xp % 16 != 0) return false;
    return ((int64_t)(t.M + 31) / 32) * (((int64_t)t.N + 31) / 32) <= INT32_MAX;
}

// runs of pixel blocks: about one wavefront per SIMD in all (measured on seven 1x1 layers: as fast as two or faster, and
// runs of up to 8 blocks are loaded whole before the first store), each with at least one block.  `raw` (the form that
// packs the codes itself, block by block): two per SIMD, whose packing and stores overlap (four layers measured: 9.5
// against 10.9 us on 56x56x256 -> 64, 4 - 10 % on two others; the layer with K = 128 was 6 % slower and keeps one)
int sparse_ws_streams(const DgProblem &t, bool raw)
{
    const int64_t row_blocks = (t.M + 31) / 32, pixel_blocks = ((int64_t)t.N + 31) / 32;
    // K = 64 on packed codes: three per SIMD -- a block is then 8 matrix instructions against 16 stores, and one
    // wavefront's stores in flight do not fill the write path (56x56x64 -> 64 at batch 32: 6.2 against 6.8 us, -> 256:
    // 21.1 against 22.0, the same at batch 8: 6.4 against 6.8; four per SIMD were slower again)
    int64_t waves = (int64_t)dg_simd_count() * (raw ? (t.K != 128 ? 2 : 1) : (t.K == 64 ? 3 : 1));
    if (const char *e = dg_override("DG_WS_WAVES")) waves = atoi(e) > 0 ? atoi(e) : waves;
    int64_t streams = waves / row_blocks;
    if (streams < 1) streams = 1;
    if (streams > pixel_blocks) streams = pixel_blocks;
    return (int)streams;
}

}   // namespace

bool dg_sparse_ws_supports(const dg_lut *lut, const DgProblem &p) { return sparse_ws_takes(lut, p); }

// AUTO: layers with enough 32 x 32 blocks that every wavefront streams several (measured against the tiled kernels)
bool dg_sparse_ws_preferred(const dg_lut *lut, const DgProblem &p)
{
    if (!sparse_ws_takes(lut, p)) return false;
    if (const char *force = dg_override("DG_ONEHOT_PLAN")) return strcmp(force, "ws") == 0;     // (tests reach it on small shapes)
    const DgProblem t = sparse_problem(p);
    const int64_t blocks = ((int64_t)(t.M + 31) / 32) * (((int64_t)t.N + 31) / 32);
    if (p.sh != 1 || p.sw != 1) {
        // With a stride a pixel's row is a part of a cache line whose rest is not read.  Measured against AUTO's other
        // choices on 60 layers with stride 2 (K = 64, 128, 256; 64 to 1024 output channels; batch 4 to 64): ahead only
        // with K = 256 from about 12 blocks per SIMD up (8 - 13 % at 12544 blocks, 40 % from 25088), 0 - 10 % behind
        // on most others.  DG_WS_STRIDED: 0 never, 1 always.
        if (const char *e = dg_override("DG_WS_STRIDED")) return atoi(e) != 0;
        return t.K == 256 && blocks >= 12 * (int64_t)dg_simd_count();
    }
    // K = 512: the operands are all of a lone wavefront's registers and take 1.5 us to build, which pays from about 12
    // blocks per SIMD (28x28x512 -> 512 at batch 32 17.7 against 19.7 us for the staged tiles, at batch 64 29.0 against
    // 34.1; at 6272 blocks and below 10 - 25 % slower)
    if (t.K == 512) return blocks >= 12 * (int64_t)dg_simd_count();
    return blocks >= (int64_t)dg_simd_count() / 2;
}

namespace {

dg_status launch_ws(const dg_lut *lut, const DgProblem &p0, bool raw, hipStream_t stream)
{
    const bool transposed = sparse_transposes(p0);
    const DgProblem p = sparse_problem(p0);
    uint32_t rows[4];                                      // rows[w] = T[w][0..3] (the transposed problem swaps the codes)
    for (int w = 0; w < 4; ++w) {
        rows[w] = 0;
        for (int v = 0; v < 4; ++v) {
            const int T = transposed ? lut->entry[(v << 2) | w] : lut->entry[(w << 2) | v];
            rows[w] |= (uint32_t)(uint8_t)(int8_t)T << (8 * v);
        }
    }
    dgoh::unit_sparse_ws(p, rows, sparse_ws_streams(p, raw), raw, stream);
    return dg_check_launch("smfmac_ws_kernel");
}

}   // namespace

dg_status dg_launch_sparse_ws(const dg_lut *lut, const DgProblem &p0, hipStream_t stream) { return launch_ws(lut, p0, false, stream); }

// The same on activations still one code per byte (p.Xp: [N][K] bytes): where the kernel runs the problem as it is
// (the activations are its pixels, not, as in a transposed GEMM, its stationary operand).
bool dg_sparse_ws_codes_supports(const dg_lut *lut, const DgProblem &p)
{
    return sparse_ws_takes(lut, p, false) && !sparse_transposes(p);
}

dg_status dg_launch_sparse_ws_codes(const dg_lut *lut, const DgProblem &p, hipStream_t stream) { return launch_ws(lut, p, true, stream); }

// ---- 4-bit codes on the sparse instruction (dg_sparse4_kernel.h): 64 x 128 tiles only, so large layers only

namespace {

int sparse4_ch(const DgProblem &t) { return (t.Cin / 2) % 16 == 0 ? 2 : 1; }

bool sparse4_takes(const dg_lut *lut, const DgProblem &p)
{
    if (lut->dtype == DG_LUT_F32 || lut->bits != 4 || !fits_int8(lut)) return false;
    if (p.Cin % 16 != 0) return false;                                 // a lane half reads whole words of one tap
    if (sparse_transposes(p) && !sparse_can_transpose(p)) return false;
    const DgProblem t = sparse_problem(p);
    const int ch = sparse4_ch(t);
    if ((uintptr_t)t.Wp % (4 * ch) != 0 || (uintptr_t)t.Xp % (4 * ch) != 0) return false;
    return tile_count(t, 2, 4) <= INT32_MAX;
}

}   // namespace

bool dg_sparse4_supports(const dg_lut *lut, const DgProblem &p) { return sparse4_takes(lut, p); }

// AUTO: where the 64 x 128 tiles give at least every second SIMD a wavefront and K is not too short for such a tile
// (measured on 14 layers: 784 tiles and more 22 - 41 % faster than the dense-instruction kernel, 392 tiles even, 196
// tiles 12 % slower, K = 64 at 784 tiles 13 % slower; that kernel's narrower tiles and split-K form serve the rest)
bool dg_sparse4_preferred(const dg_lut *lut, const DgProblem &p)
{
    return sparse4_takes(lut, p) && tile_count(sparse_problem(p), 2, 4) >= 512 && p.K >= 256 &&
           dg_override("DG_ONEHOT_PLAN") == nullptr;
}

dg_status dg_launch_sparse4(const dg_lut *lut, const DgProblem &p0, hipStream_t stream)
{
    const bool transposed = sparse_transposes(p0);
    const DgProblem p = sparse_problem(p0);
    uint32_t rows[16][4];                                  // rows[w] = T[w][0..15] (the transposed problem swaps the codes)
    for (int w = 0; w < 16; ++w)
        for (int i = 0; i < 4; ++i) {
            rows[w][i] = 0;
            for (int b = 0; b < 4; ++b) {
                const int v = 4 * i + b, T = transposed ? lut->entry[(v << 4) | w] : lut->entry[(w << 4) | v];
                rows[w][i] |= (uint32_t)(uint8_t)(int8_t)T << (8 * b);
            }
        }
    dgoh::unit_sparse4(p, rows, sparse4_ch(p), stream);
    return dg_check_launch("sparse4_kernel");
}

// ---- 2-bit codes with entries beyond int8 on the sparse instruction (dg_sparse2p_kernel.h): 32 x 128 tiles only

namespace {

int sparse2p_ch(const DgProblem &t) { return (t.Cin / 4) % 16 == 0 ? 2 : 1; }    // (4 words per chunk would spill)

bool sparse2p_takes(const dg_lut *lut, const DgProblem &p)
{
    if (lut->dtype == DG_LUT_F32 || lut->bits != 2 || fits_int8(lut) || lut->max_entry > 127 * 256 + 127) return false;
    if (p.Cin % 32 != 0) return false;                                 // a lane half reads whole words of one tap
    if (sparse_transposes(p) && !sparse_can_transpose(p)) return false;
    const DgProblem t = sparse_problem(p);
    const int ch = sparse2p_ch(t);
    if ((uintptr_t)t.Wp % (4 * ch) != 0 || (uintptr_t)t.Xp % (4 * ch) != 0) return false;
    return tile_count(t, 1, 4) <= INT32_MAX;
}

}   // namespace

bool dg_sparse2p_supports(const dg_lut *lut, const DgProblem &p) { return sparse2p_takes(lut, p); }

// AUTO: where the 32 x 128 tiles give every SIMD a wavefront and K is long enough to amortise the tile's stores
// (measured: 20 - 27 % faster than the dense-instruction kernel from 1568 tiles with K >= 576, even at 784 tiles, 23 %
// slower at K = 64; that kernel's narrower tiles and split-K form serve the smaller layers)
bool dg_sparse2p_preferred(const dg_lut *lut, const DgProblem &p)
{
    return sparse2p_takes(lut, p) && tile_count(sparse_problem(p), 1, 4) >= 1024 && p.K >= 512 &&
           dg_override("DG_ONEHOT_PLAN") == nullptr;
}

dg_status dg_launch_sparse2p(const dg_lut *lut, const DgProblem &p0, hipStream_t stream)
{
    const bool transposed = sparse_transposes(p0);
    const DgProblem p = sparse_problem(p0);
    uint32_t rows[2][4];                                   // rows[plane][w] = plane(T[w][0..3]) (transposed: codes swapped)
    for (int w = 0; w < 4; ++w) {
        rows[0][w] = rows[1][w] = 0;
        for (int v = 0; v < 4; ++v) {
            const int T = transposed ? lut->entry[(v << 2) | w] : lut->entry[(w << 2) | v];
            const int lo = ((T + 128) & 255) - 128, hi = (T - lo) / 256;
            rows[0][w] |= (uint32_t)(uint8_t)(int8_t)lo << (8 * v);
            rows[1][w] |= (uint32_t)(uint8_t)(int8_t)hi << (8 * v);
        }
    }
    dgoh::unit_sparse2p(p, rows, sparse2p_ch(p), stream);
    return dg_check_launch("sparse2p_kernel");
}

bool dg_decode_supports(const dg_lut *lut, const DgProblem &p)
{
    // the levels themselves are the MFMA operands: the table must be their outer product, with 2-bit codes
    if (lut->dtype == DG_LUT_F32 || !lut->separable || lut->bits != 2) return false;
    if (p.Cin % 32 != 0) return false;                                 // a lane half reads whole words of one tap
    if (!offsets_fit(p, 4)) return false;
    const Plan q = plan_for(lut, p, DECODE);
    if ((uintptr_t)p.Wp % (4 * q.ch) != 0 || (uintptr_t)p.Xp % (4 * q.ch) != 0) return false;
    return true;
}

const char *dg_onehot_config_name(const dg_lut *lut, const DgProblem &p)
{
    static const char *const split_names[2][17] = {
        {"", "onehot_mfma_splitk_s1", "onehot_mfma_splitk_s2", "onehot_mfma_splitk_s3", "onehot_mfma_splitk_s4",
         "onehot_mfma_splitk_s5", "onehot_mfma_splitk_s6", "onehot_mfma_splitk_s7", "onehot_mfma_splitk_s8",
         "onehot_mfma_splitk_s9", "onehot_mfma_splitk_s10", "onehot_mfma_splitk_s11", "onehot_mfma_splitk_s12",
         "onehot_mfma_splitk_s13", "onehot_mfma_splitk_s14", "onehot_mfma_splitk_s15", "onehot_mfma_splitk_s16"},
        {"", "onehot_mfma_2p_splitk_s1", "onehot_mfma_2p_splitk_s2", "onehot_mfma_2p_splitk_s3", "onehot_mfma_2p_splitk_s4",
         "onehot_mfma_2p_splitk_s5", "onehot_mfma_2p_splitk_s6", "onehot_mfma_2p_splitk_s7", "onehot_mfma_2p_splitk_s8",
         "onehot_mfma_2p_splitk_s9", "onehot_mfma_2p_splitk_s10", "onehot_mfma_2p_splitk_s11", "onehot_mfma_2p_splitk_s12",
         "onehot_mfma_2p_splitk_s13", "onehot_mfma_2p_splitk_s14", "onehot_mfma_2p_splitk_s15", "onehot_mfma_2p_splitk_s16"}};
    static const char *const tile_names[2][3][4] = {
        {{"onehot_mfma_64x224", "onehot_mfma_64x128", "onehot_mfma_64x64", "onehot_mfma_64x32"},
         {"", "onehot_mfma_64x128_k2", "onehot_mfma_64x64_k2", "onehot_mfma_64x32_k2"},
         {"onehot_mfma_64x224_k4", "onehot_mfma_64x128_k4", "onehot_mfma_64x64_k4", "onehot_mfma_64x32_k4"}},
        {{"onehot_mfma_2p_32x224", "onehot_mfma_2p_32x128", "onehot_mfma_2p_32x64", "onehot_mfma_2p_32x32"},
         {"", "", "", ""}, {"", "", "", ""}}};
    const Plan q = plan_for(lut, p, TABLE);
    if (q.split) return split_names[q.two][q.S];
    return tile_names[q.two][q.skw == 4 ? 2 : (q.skw == 2 ? 1 : 0)][q.wn == 7 ? 0 : (q.wn == 4 ? 1 : (q.wn == 2 ? 2 : 3))];
}

const char *dg_decode_config_name(const dg_lut *lut, const DgProblem &p)
{
    static const char *const split_names[17] = {
        "", "mfma_i8_splitk_s1", "mfma_i8_splitk_s2", "mfma_i8_splitk_s3", "mfma_i8_splitk_s4", "mfma_i8_splitk_s5",
        "mfma_i8_splitk_s6", "mfma_i8_splitk_s7", "mfma_i8_splitk_s8", "mfma_i8_splitk_s9", "mfma_i8_splitk_s10",
        "mfma_i8_splitk_s11", "mfma_i8_splitk_s12", "mfma_i8_splitk_s13", "mfma_i8_splitk_s14", "mfma_i8_splitk_s15",
        "mfma_i8_splitk_s16"};
    static const char *const tile_names[3][4] = {
        {"mfma_i8_64x224", "mfma_i8_64x128", "mfma_i8_64x64", "mfma_i8_64x32"},
        {"", "mfma_i8_64x128_k2", "mfma_i8_64x64_k2", "mfma_i8_64x32_k2"},
        {"mfma_i8_64x224_k4", "mfma_i8_64x128_k4", "mfma_i8_64x64_k4", "mfma_i8_64x32_k4"}};
    const Plan q = plan_for(lut, p, DECODE);
    if (q.split) return split_names[q.S];
    if (q.wm == 4) return "mfma_i8_128x128";
    return tile_names[q.skw == 4 ? 2 : (q.skw == 2 ? 1 : 0)][q.wn == 7 ? 0 : (q.wn == 4 ? 1 : (q.wn == 2 ? 2 : 3))];
}

dg_status dg_launch_decode(const dg_lut *lut, const DgProblem &p, hipStream_t stream)
{
    const Plan q = plan_for(lut, p, DECODE);
    dgoh::Pools pools;
    for (int i = 0; i < 64; ++i) pools.w[i] = 0;
    for (int c = 0; c < 4; ++c) {                          // the two level vectors as byte-permute pools
        pools.w[0] |= (uint32_t)(uint8_t)lut->levels_w[c] << (8 * c);
        pools.w[1] |= (uint32_t)(uint8_t)lut->levels_a[c] << (8 * c);
    }
    const int64_t blocks11 = tile_count(p, 1, 1), wave_tiles = tile_count(p, q.wm, q.wn);
    if ((q.split ? blocks11 : wave_tiles) > INT32_MAX)
        return dg_fail(DG_ERR_UNSUPPORTED, "decode-and-multiply kernel: too many tiles for one grid");
    const int tr = (p.stride_cm == 1 && p.stride_cn != 1) ? 1 : 0;
    using namespace dgoh;
    static const MainFn split_units[2] = {unit_split_b0_t0, unit_split_b0_t1};
    static const MainFn main_units[3][2] = {{unit_main_b0_t0_k1, unit_main_b0_t1_k1}, {unit_main_b0_t0_k2, unit_main_b0_t1_k2},
                                            {unit_main_b0_t0_k4, unit_main_b0_t1_k4}};
    if (q.split) {
        split_units[tr](p, pools, q, blocks11, stream);
        return dg_check_launch("onehot_splitk_kernel<0>");
    }
    main_units[q.skw == 4 ? 2 : (q.skw == 2 ? 1 : 0)][tr](p, pools, q, wave_tiles, stream);
    return dg_check_launch("onehot_mfma_kernel<0>");
}

namespace {

dg_status launch_onehot(const dg_lut *lut, const DgProblem &p, hipStream_t stream, bool codes, bool sparse_tiles = false);

}   // namespace

dg_status dg_launch_onehot(const dg_lut *lut, const DgProblem &p, hipStream_t stream)
{
    return launch_onehot(lut, p, stream, false);
}

// ---- activations still one code per byte (p.Xp = [pixel][Cin] bytes): the split-K kernel packs them as it loads them

bool dg_onehot_codes_supports(const dg_lut *lut, const DgProblem &p)
{
    if (lut->dtype == DG_LUT_F32 || lut->bits != 2) return false;
    if (!fits_int8(lut) && lut->max_entry > 127 * 256 + 127) return false;
    if (p.Cin % 32 != 0) return false;                                 // a lane half reads whole words of one tap
    const Plan q = plan_for(lut, p, TABLE);
    return q.split && (uintptr_t)p.Wp % (4 * q.ch) == 0 && (uintptr_t)p.Xp % 16 == 0;
}

// Every 32-row block of the output packs the activation codes it reads for itself, so the packing is done
// ceil(M / 32) times over (and per filter tap): 14 VALU instructions per 16 codes and 64 lanes.  Worth a saved launch
// (1.6 us) while that stays well under a microsecond of the chip's VALU time -- measured: 0.2 us on a 64 x 3136 x 576
// layer (2 row blocks), but 3 us on the 8192 x 16 x 8192 GEMM (256 row blocks), which is faster as two kernels.
bool dg_onehot_codes_pays(const DgProblem &p)
{
    const double row_blocks = (p.M + 31) / 32, columns = 32.0 * ((p.N + 31) / 32);
    // (and not with the longest reductions: 3x3 windows over 512 channels, K = 4608, measured 9.4 - 9.7 us in one call
    // against 8.6 - 8.8 us as two kernels on 7x7 and 14x14 images; K = 2304 and 2048 6.1 - 6.2 against 6.4 - 6.7)
    return row_blocks * columns * p.K <= 2.0e7 && p.K <= 3072;
}

// The plan of the tiled kernel on unpacked codes: the dense instruction's, in 2-word chunks.
static bool codes_tiled_plan(const dg_lut *lut, const DgProblem &p, Plan *out)
{
    if (lut->dtype == DG_LUT_F32 || lut->bits != 2 || !fits_int8(lut)) return false;
    if (p.Cin % 64 != 0 || !offsets_fit(p, 1)) return false;
    Plan q = plan_for(lut, p, TABLE);
    if (q.split || q.two || q.wm != 2 || q.wn > 2) return false;
    if (q.ch == 4) q.ch = 2, q.chunks *= 2;
    if (q.ch != 2 || (uintptr_t)p.Wp % 8 != 0 || (uintptr_t)p.Xp % 16 != 0) return false;
    *out = q;
    return true;
}

// On the sparse instruction where the output's channel axis has stride 1 (the activations are then the instruction's row
// operand as they stand) and the caller has not named the dense instruction's variant.  DG_ONEHOT_CODES_SPARSE: 0 / 1
// (A/B measurement).
bool dg_onehot_codes_tiled_sparse(const dg_lut *, const DgProblem &p)
{
    if (p.stride_cm != 1) return false;
    if (const char *e = dg_override("DG_ONEHOT_CODES_SPARSE")) return atoi(e) != 0;
    return true;                                           // (3 - 17 % shorter than the dense instruction's on 30 layer shapes)
}

bool dg_onehot_codes_tiled_supports(const dg_lut *lut, const DgProblem &p)
{
    Plan q;
    return codes_tiled_plan(lut, p, &q);
}

// Measured on 44 layer shapes (ResNet-50 and ResNet-18 layers at batch 4 to 32): over the best kernel on packed codes,
// packing in this kernel costs about 0.9 us per 10^9 table operations (2MNK) on the sparse instruction where the best
// kernel is the staged one (Cin % 128 == 0), 0.35 us where it is this kernel's own direct-load form, and 1.6 us on
// the dense instruction (outputs whose channel axis is not the contiguous one) -- narrow tiles, loads of 16 bytes per
// 16 codes, the packing repeated per 64-row tile; the packing kernel costs 1.8 us plus 0.17 us per MB of codes it
// packs (all the input's, except that of a 1x1 layer with a stride only the pixels read).  So: layers up to about
// 2 * 10^9 operations (14x14x1024 -> 256 at batch 8: 5.5 against 6.7 us; 56x56x64 -> 64 3x3 at batch 8: 8.2 against 9.6),
// and further up where there is much to pack or the channels are not whole 128s (56x56x64 -> 64 3x3 at batch 32: 14.8
// against 15.2).  Total regret of this rule against the better of the two on 40 shapes: 1.5 us, 0.6 at most.
// DG_ONEHOT_CODES_TILED: 0 never, 1 always (A/B measurement).
bool dg_onehot_codes_tiled_pays(const dg_lut *, const DgProblem &p, bool sparse_tiles)
{
    if (const char *e = dg_override("DG_ONEHOT_CODES_TILED")) return atoi(e) != 0;
    const double ops = 2.0 * (double)p.M * (double)p.N * (double)p.K;
    const bool strided_1x1 = p.KH == 1 && p.KW == 1 && p.ph == 0 && p.pw == 0;     // (packed pixel by pixel: only those read)
    const double images = (double)p.N / ((double)p.OH * p.OW);
    const double code_bytes = strided_1x1 ? (double)p.N * p.Cin : images * p.H * p.W * p.Cin;
    const double per_op = !sparse_tiles ? 1.6e-9 : (p.Cin % 128 == 0 ? 0.9e-9 : 0.35e-9);
    return per_op * ops + 0.2 < 1.8 + 0.17e-6 * code_bytes;
}

const char *dg_onehot_codes_config_name(const dg_lut *lut, const DgProblem &p, bool sparse_tiles)
{
    Plan t;
    if (!plan_for(lut, p, TABLE).split && codes_tiled_plan(lut, p, &t)) {
        static const char *const tiled[2][3][2] = {{{"codes_onehot_mfma_64x32", "codes_onehot_mfma_64x64"},
                                                    {"codes_onehot_mfma_64x32_k2", "codes_onehot_mfma_64x64_k2"},
                                                    {"codes_onehot_mfma_64x32_k4", "codes_onehot_mfma_64x64_k4"}},
                                                   {{"codes_onehot_smfmac_64x32", "codes_onehot_smfmac_64x64"},
                                                    {"codes_onehot_smfmac_64x32_k2", "codes_onehot_smfmac_64x64_k2"},
                                                    {"codes_onehot_smfmac_64x32_k4", "codes_onehot_smfmac_64x64_k4"}}};
        return tiled[sparse_tiles ? 1 : 0][t.skw == 4 ? 2 : (t.skw == 2 ? 1 : 0)][t.wn == 2 ? 1 : 0];
    }
    static const char *const names[2][17] = {
        {"", "codes_onehot_mfma_splitk_s1", "codes_onehot_mfma_splitk_s2", "codes_onehot_mfma_splitk_s3",
         "codes_onehot_mfma_splitk_s4", "codes_onehot_mfma_splitk_s5", "codes_onehot_mfma_splitk_s6",
         "codes_onehot_mfma_splitk_s7", "codes_onehot_mfma_splitk_s8", "codes_onehot_mfma_splitk_s9",
         "codes_onehot_mfma_splitk_s10", "codes_onehot_mfma_splitk_s11", "codes_onehot_mfma_splitk_s12",
         "codes_onehot_mfma_splitk_s13", "codes_onehot_mfma_splitk_s14", "codes_onehot_mfma_splitk_s15",
         "codes_onehot_mfma_splitk_s16"},
        {"", "codes_onehot_mfma_2p_splitk_s1", "codes_onehot_mfma_2p_splitk_s2", "codes_onehot_mfma_2p_splitk_s3",
         "codes_onehot_mfma_2p_splitk_s4", "codes_onehot_mfma_2p_splitk_s5", "codes_onehot_mfma_2p_splitk_s6",
         "codes_onehot_mfma_2p_splitk_s7", "codes_onehot_mfma_2p_splitk_s8", "codes_onehot_mfma_2p_splitk_s9",
         "codes_onehot_mfma_2p_splitk_s10", "codes_onehot_mfma_2p_splitk_s11", "codes_onehot_mfma_2p_splitk_s12",
         "codes_onehot_mfma_2p_splitk_s13", "codes_onehot_mfma_2p_splitk_s14", "codes_onehot_mfma_2p_splitk_s15",
         "codes_onehot_mfma_2p_splitk_s16"}};
    const Plan q = plan_for(lut, p, TABLE);
    return names[q.two][q.S];
}

dg_status dg_launch_onehot_codes(const dg_lut *lut, const DgProblem &p, hipStream_t stream, bool sparse_tiles)
{
    return launch_onehot(lut, p, stream, true, sparse_tiles);
}

namespace {

dg_status launch_onehot(const dg_lut *lut, const DgProblem &p, hipStream_t stream, bool codes, bool sparse_tiles)
{
    // column v of the table, 4 weight codes per word: the permute pools.  Entries beyond int8 go in two planes,
    // T = 256 * hi + lo with lo in [-128, 127] (so hi is within [-128, 128) for every int16 T).
    Plan q = plan_for(lut, p, TABLE);
    // On unpacked codes the same wavefronts walk their shares of K in chunks of 64 positions, not 128: four 16-byte loads
    // of codes and their packing per chunk instead of eight (measured on nine small layers: the one-call step 0.1 - 0.7 us
    // shorter, 7x7x2048 -> 512 at batch 1 6.85 -> 6.13 us).
    if (codes && q.split && q.ch == 4) q.ch = 2, q.chunks *= 2, q.cpw *= 2;
    dgoh::Pools pools;
    const int L = 1 << lut->bits, qw = L / 4;
    for (int i = 0; i < 64; ++i) pools.w[i] = 0;
    for (int v = 0; v < L; ++v)
        for (int w = 0; w < L; ++w) {
            const int T = lut->entry[(w << lut->bits) | v];
            const int lo = q.two ? ((T + 128) & 255) - 128 : T, hi = (T - lo) / 256;
            pools.w[v * qw + w / 4] |= (uint32_t)(uint8_t)(int8_t)lo << (8 * (w % 4));
            if (q.two) pools.w[32 + v * qw + w / 4] |= (uint32_t)(uint8_t)(int8_t)hi << (8 * (w % 4));
        }
    const int64_t blocks11 = tile_count(p, 1, 1), wave_tiles = tile_count(p, q.two ? 1 : 2, q.wn);
    if ((q.split ? blocks11 : wave_tiles) > INT32_MAX)
        return dg_fail(DG_ERR_UNSUPPORTED, "one-hot kernel: too many tiles for one grid");
    const int tr = (p.stride_cm == 1 && p.stride_cn != 1) ? 1 : 0;   // the output axis with stride 1 goes on the MFMA columns
    using namespace dgoh;
    // [code width: 2, 3, 4, 2 in two planes][layout]
    static const MainFn split_units[4][2] = {{unit_split_b2_t0, unit_split_b2_t1}, {unit_split_b3_t0, unit_split_b3_t1},
                                             {unit_split_b4_t0, unit_split_b4_t1}, {unit_split_b22_t0, unit_split_b22_t1}};
    static const MainFn main_units[4][2] = {{unit_main_b2_t0_k1, unit_main_b2_t1_k1}, {unit_main_b3_t0_k1, unit_main_b3_t1_k1},
                                            {unit_main_b4_t0_k1, unit_main_b4_t1_k1}, {unit_main_b22_t0_k1, unit_main_b22_t1_k1}};
    static const MainFn shared_units[2][2] = {{unit_main_b2_t0_k2, unit_main_b2_t1_k2}, {unit_main_b2_t0_k4, unit_main_b2_t1_k4}};
    const int width = q.two ? 3 : lut->bits - 2;
    if (codes && !q.split) {
        Plan t;
        if (!codes_tiled_plan(lut, p, &t))
            return dg_fail(DG_ERR_UNSUPPORTED, "one-hot kernel on unpacked codes: this layer's plan has no such form");
        const int64_t tiles = tile_count(p, 2, t.wn);
        if (tiles > INT32_MAX) return dg_fail(DG_ERR_UNSUPPORTED, "one-hot kernel: too many tiles for one grid");
        if (sparse_tiles) {
            // (the sparse instruction's pools: word w = the table row of weight code w, bytes over the activation code)
            dgoh::Pools sp;
            for (int i = 0; i < 64; ++i) sp.w[i] = 0;
            for (int w = 0; w < 4; ++w)
                for (int v = 0; v < 4; ++v) sp.w[w] |= (uint32_t)(uint8_t)(int8_t)lut->entry[(w << 2) | v] << (8 * v);
            unit_main_codes(p, sp, t, true, true, tiles, stream);
            return dg_check_launch("onehot_mfma_kernel<20> (unpacked codes)");
        }
        unit_main_codes(p, pools, t, tr != 0, false, tiles, stream);
        return dg_check_launch("onehot_mfma_kernel (unpacked codes)");
    }
    if (codes) {
        if (lut->bits != 2)
            return dg_fail(DG_ERR_UNSUPPORTED, "one-hot kernel on unpacked codes: 2-bit codes only");
        unit_split_codes(p, pools, q, q.two, tr != 0, blocks11, stream);
        return dg_check_launch("onehot_splitk_kernel (unpacked codes)");
    }
    if (q.split) {
        split_units[width][tr](p, pools, q, blocks11, stream);
        return dg_check_launch("onehot_splitk_kernel");
    }
    if (q.skw > 1)
        shared_units[q.skw == 4][tr](p, pools, q, wave_tiles, stream);      // (planned for 2-bit one-plane tables only)
    else
        main_units[width][tr](p, pools, q, wave_tiles, stream);
    return dg_check_launch("onehot_mfma_kernel");
}

}   // namespace
