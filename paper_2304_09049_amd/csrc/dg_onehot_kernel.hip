// Host side of the one-hot matrix-core kernels (dg_onehot_kernel.h): which problems they take, which of their
// shapes runs a given problem, and the launch.
#include <cstdlib>

#include "dg_onehot_kernel.h"

namespace {

using dgoh::Plan;

int per_byte(const dg_lut *lut) { return lut->bits == 2 ? 4 : 2; }

int64_t tile_count(const DgProblem &p, int wm, int wn)
{
    return ((int64_t)(p.M + wm * 32 - 1) / (wm * 32)) * (((int64_t)p.N + wn * 32 - 1) / (wn * 32));
}

bool fits_int8(const dg_lut *lut) { return lut->min_entry >= -128 && lut->max_entry <= 127; }

Plan plan_for(const dg_lut *lut, const DgProblem &p)
{
    Plan q;
    q.two = !fits_int8(lut);                               // two int8 planes; a tile is then 32 rows high, not 64
    const int wm = q.two ? 1 : 2;
    // a lane half reads 4*ch packed bytes of one filter tap per chunk
    const int tap_bytes = p.Cin / per_byte(lut);
    q.ch = tap_bytes % 32 == 0 ? 4 : (tap_bytes % 16 == 0 ? 2 : 1);
    if (lut->bits == 4 && q.ch == 4) q.ch = 2;             // (a 4-word chunk of 4-bit codes would be 32 MFMA steps)
    q.chunks = (p.K / per_byte(lut)) / (8 * q.ch);
    q.wn = 1, q.S = 1, q.cpw = q.chunks;
    // too few 64 x 32 tiles to give every SIMD a wavefront (or barely enough, and a long K to walk): split K
    const int64_t t21 = tile_count(p, wm, 1);
    const bool few_tiles = t21 < 512 || (t21 < 1024 && q.chunks >= 32);
    q.split = few_tiles && q.chunks > 1;
    // DG_ONEHOT_PLAN = split | 1 | 2 | 4 | 7 overrides the choice (tuning, and tests that must reach every plan)
    const char *force = getenv("DG_ONEHOT_PLAN");
    int force_wn = 0;
    if (force) {
        const int v = atoi(force);
        if (force[0] == 's') q.split = true;
        else if (v == 1 || v == 2 || v == 4 || v == 7) force_wn = v, q.split = false;
    }
    if (q.split) {
        // about 2048 wavefronts in all, at most 16 per workgroup, whole chunks each
        const int64_t blocks = tile_count(p, 1, 1);
        int64_t target = 2048;
        if (const char *e = getenv("DG_ONEHOT_WAVES")) target = atoi(e) > 0 ? atoi(e) : target;   // tuning override
        int S = (int)((target + blocks - 1) / blocks);
        S = S < 1 ? 1 : (S > 16 ? 16 : S);
        if (S > q.chunks) S = q.chunks;
        q.cpw = (q.chunks + S - 1) / S;
        q.S = (q.chunks + q.cpw - 1) / q.cpw;
        return q;
    }
    // Wave tile 64 x (32*wn): the one with the least modelled time on the busiest SIMD, in cycles.  A SIMD's
    // wavefronts share its matrix pipe, so its time is (tiles per SIMD, rounded up) x (32x32 blocks per tile) x (MFMA
    // steps of K) x (cycles per MFMA: 32, more where the VALU work of building operands or the operand loads show --
    // measured 42 for one block column, 33 for two), plus what no other wavefront hides: one prologue (~3000 cycles)
    // and the last tile's stores (~600 cycles per block).  7 blocks wide fits the 56 x 56 and 28 x 28 images of
    // ImageNet networks (N = 49 * 2^k) where 4 wide leaves the last round of tiles half empty.  The constants are
    // fitted to timings of 48 layer shapes with 2-bit codes; ties go to the wider tile (fewer operand loads).
    static const int widths[4] = {7, 4, 2, 1};
    static const double mfma_cycles[4] = {32.0, 32.0, 33.0, 42.0};
    const double steps = (double)p.K * (1 << lut->bits) / 32.0;
    double best = 0.0;
    for (int i = 0; i < 4; ++i) {
        const int wn = widths[i];
        const double per_simd = (double)((tile_count(p, wm, wn) + 1023) / 1024);
        const double cost = per_simd * 2 * wn * steps * mfma_cycles[i] + 3000.0 + 600.0 * 2 * wn;
        if (i == 0 || cost < best * 0.999) best = cost, q.wn = wn;
    }
    if (force_wn) q.wn = force_wn;
    if (lut->bits == 4 && q.wn == 7) q.ch = 1;             // (the 2-word kernel of this tile is not built: see launch_ch)
    return q;
}

}   // namespace

bool dg_onehot_supports(const dg_lut *lut, const DgProblem &p)
{
    if (lut->dtype == DG_LUT_F32) return false;
    // MFMA operands are int8: wider entries take two planes, T = 256 * hi + lo (2-bit codes only, hi within int8)
    if (!fits_int8(lut) && (lut->bits != 2 || lut->max_entry > 127 * 256 + 127)) return false;
    if (p.Cin % (8 * per_byte(lut)) != 0) return false;                // a lane half reads whole words of one tap
    const Plan q = plan_for(lut, p);
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
    static const char *const tile_names[2][4] = {
        {"onehot_mfma_64x224", "onehot_mfma_64x128", "onehot_mfma_64x64", "onehot_mfma_64x32"},
        {"onehot_mfma_2p_32x224", "onehot_mfma_2p_32x128", "onehot_mfma_2p_32x64", "onehot_mfma_2p_32x32"}};
    const Plan q = plan_for(lut, p);
    if (q.split) return split_names[q.two][q.S];
    return tile_names[q.two][q.wn == 7 ? 0 : (q.wn == 4 ? 1 : (q.wn == 2 ? 2 : 3))];
}

dg_status dg_launch_onehot(const dg_lut *lut, const DgProblem &p, hipStream_t stream)
{
    // column v of the table, 4 weight codes per word: the permute pools.  Entries beyond int8 go in two planes,
    // T = 256 * hi + lo with lo in [-128, 127] (so hi is within [-128, 128) for every int16 T).
    const Plan q = plan_for(lut, p);
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
    if ((q.split ? blocks11 : (wave_tiles + 3) / 4) > INT32_MAX)
        return dg_fail(DG_ERR_UNSUPPORTED, "one-hot kernel: too many tiles for one grid");
    const bool tr = p.stride_cm == 1 && p.stride_cn != 1;   // the output axis with stride 1 goes on the MFMA columns
    if (q.two) {
        (tr ? dgoh::launch_bits2_two_tr1 : dgoh::launch_bits2_two_tr0)(p, pools, q, blocks11, wave_tiles, stream);
        return dg_check_launch(q.split ? "onehot_splitk_kernel" : "onehot_mfma_kernel");
    }
    switch (lut->bits) {
    case 2: (tr ? dgoh::launch_bits2_tr1 : dgoh::launch_bits2_tr0)(p, pools, q, blocks11, wave_tiles, stream); break;
    case 3: (tr ? dgoh::launch_bits3_tr1 : dgoh::launch_bits3_tr0)(p, pools, q, blocks11, wave_tiles, stream); break;
    default: (tr ? dgoh::launch_bits4_tr1 : dgoh::launch_bits4_tr0)(p, pools, q, blocks11, wave_tiles, stream); break;
    }
    return dg_check_launch(q.split ? "onehot_splitk_kernel" : "onehot_mfma_kernel");
}
