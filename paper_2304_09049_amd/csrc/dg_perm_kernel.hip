// Host side of the permute table kernel: which tables and shapes it accepts, which tile shape runs, the launch.
#include <cstdlib>
#include <cstring>

#include "dg_perm_kernel.h"

namespace {
using dgperm::PermArgs;

struct PermPlan {
    int TM, TN, LM, LN, KS, SK, NBUF, MODE, OCC;   // OCC: workgroups of this shape that fit one compute unit
    const char *name;
    dg_status (*launch_mfast)(const PermArgs &, dim3, hipStream_t);   // output channel-fastest (NHWC)
    dg_status (*launch_nfast)(const PermArgs &, dim3, hipStream_t);   // output column-fastest ([M][N])
    int BM() const { return LM * TM; }
    int BN() const { return LN * TN; }
};

#define DG_PLAN(TM, TN, LM, LN, KS, SK, NBUF, MODE, OCC)                                                  \
    {TM, TN, LM, LN, KS, SK, NBUF, MODE, OCC,                                                             \
     "perm_" #TM "x" #TN "_" #LM "x" #LN "_k" #KS "_s" #SK "_b" #NBUF "_m" #MODE,                         \
     dgperm::perm_launch<TM, TN, LM, LN, KS, SK, NBUF, MODE, true>,                                      \
     dgperm::perm_launch<TM, TN, LM, LN, KS, SK, NBUF, MODE, false>},

const PermPlan kPlans[] = {
#include "dg_perm_plans.inc"
};
constexpr int kNumPlans = sizeof(kPlans) / sizeof(kPlans[0]);
constexpr int kComputeUnits = 256;

// 0: byte lanes (four products per permute), 1: 16-bit lanes (two per permute), -1: not a permute table
int mode_for(const dg_lut *lut)
{
    const int range = lut->max_entry - lut->min_entry;
    if (range <= 31) return 0;      // byte lanes take >= 8 carry-free adds
    if (range <= 255) return 1;     // a biased entry still fits the byte a permute fetches
    return -1;
}

const PermPlan *find(int TM, int TN, int KS, int SK, int mode)
{
    for (int i = 0; i < kNumPlans; ++i) {
        const PermPlan &c = kPlans[i];
        if (c.TM == TM && c.TN == TN && c.KS == KS && c.SK == SK && c.MODE == mode) return &c;
    }
    return nullptr;
}

const PermPlan *plan_for(const dg_lut *lut, const DgProblem &p)
{
    const int mode = mode_for(lut);
    if (mode < 0) return nullptr;
    // DG_PERM_PLAN=<index> forces a tile shape of the right mode (A/B measurement only)
    if (const char *e = dg_override("DG_PERM_PLAN")) {
        const int i = atoi(e);
        if (i >= 0 && i < kNumPlans && kPlans[i].MODE == mode) return &kPlans[i];
    }
    auto tiles = [&](const PermPlan *c) {
        return ((int64_t)(p.M + c->BM() - 1) / c->BM()) * (((int64_t)p.N + c->BN() - 1) / c->BN());
    };
    // Whole-tile shapes: estimate the time of the busiest compute unit.  It holds ceil(tiles / CUs) workgroups,
    // OCC at a time; n workgroups sharing a CU issue at rate[n] of its peak (one wave per SIMD cannot hide LDS
    // latency), and a lane tile with fewer outputs spends more of its instructions outside the permute loop.
    static const double rate[5] = {0.0, 0.55, 0.84, 0.92, 1.0};
    const PermPlan *best = nullptr;
    double best_time = 0.0;
    for (int i = 0; i < kNumPlans; ++i) {
        const PermPlan *c = &kPlans[i];
        if (c->MODE != mode || c->SK != 1) continue;
        if (c->BM() > 64 && p.M <= 64) continue;                       // half-empty tiles: never better
        const int64_t per_cu = (tiles(c) + kComputeUnits - 1) / kComputeUnits;
        const double shape_eff = c->TM * c->TN >= 64 ? 1.0 : (c->TM * c->TN >= 56 ? 0.95 : 0.82);
        const double work = (double)c->BM() * c->BN() / shape_eff;
        const int64_t full_rounds = per_cu / c->OCC, rest = per_cu % c->OCC;
        double time = full_rounds * (c->OCC * work / rate[c->OCC > 4 ? 4 : c->OCC]);
        if (rest) time += rest * work / rate[rest];
        // prefer the stage length that divides K among otherwise equal shapes
        if (p.K % c->KS != 0) time *= 1.0 + (double)(c->KS - p.K % c->KS) / p.K;
        if (!best || time < best_time) best = c, best_time = time;
    }
    const PermPlan *one_stage = find(2, 4, 96, 6, mode), *split = find(4, 4, 48, 4, mode);
    // fewer tiles than compute units: split K inside the workgroup instead
    if (best && tiles(best) >= kComputeUnits) return best;
    if (one_stage && p.K <= one_stage->KS * one_stage->SK) return one_stage;
    if (split) return split;
    return best;
}

dgperm::FastDiv make_div(uint32_t d) { return dg_make_div(d); }

}   // namespace

bool dg_perm_supports(const dg_lut *lut, const DgProblem &p)
{
    if (mode_for(lut) < 0) return false;
    if (p.Cin % 16 != 0) return false;                           // a 32-bit packed word never straddles taps
    if ((uintptr_t)p.Wp % 4 != 0 || (uintptr_t)p.Xp % 4 != 0) return false;
    // the loader keeps 32-bit byte offsets into the activation tensor
    if ((int64_t)p.N / (p.OH * p.OW) * p.H * p.W * (p.Cin / 4) >= ((int64_t)1 << 31)) return false;
    return plan_for(lut, p) != nullptr;
}

const char *dg_perm_config_name(const dg_lut *lut, const DgProblem &p)
{
    const PermPlan *plan = plan_for(lut, p);
    return plan ? plan->name : "unsupported";
}

dg_status dg_launch_perm(const dg_lut *lut, const DgProblem &p, hipStream_t stream)
{
    const PermPlan *plan = plan_for(lut, p);
    if (!plan) return dg_fail(DG_ERR_UNSUPPORTED, "perm kernel: table range %d exceeds 255", lut->max_entry - lut->min_entry);
    PermArgs a;
    a.p = p;
    a.min_entry = lut->min_entry;
    const int range = lut->max_entry - lut->min_entry;
    for (int w = 0; w < 4; ++w) {
        uint32_t r = 0;
        for (int c = 0; c < 4; ++c) r |= (uint32_t)(lut->entry[4 * w + c] - lut->min_entry) << (8 * c);
        a.rows[w] = r;
    }
    // a 16-code group adds 8 entries to each byte lane (mode 0) or 16 entries to each 16-bit lane (mode 1)
    const int lane_max = plan->MODE == 0 ? 255 : 65535, per_group = plan->MODE == 0 ? 8 : 16;
    int fd = range > 0 ? lane_max / range / per_group : 1 << 20;
    if (fd > 1 << 20) fd = 1 << 20;
    a.flush_dwords = fd;
    a.tiles_m = (p.M + plan->BM() - 1) / plan->BM();
    const int64_t tiles_n = ((int64_t)p.N + plan->BN() - 1) / plan->BN();
    const int64_t blocks = tiles_n * a.tiles_m;
    if (blocks > INT32_MAX) return dg_fail(DG_ERR_UNSUPPORTED, "perm kernel: too many tiles for one grid");
    a.div_ow = make_div((uint32_t)p.OW);
    a.div_oh = make_div((uint32_t)p.OH);
    a.div_cin = make_div((uint32_t)p.Cin);
    a.div_kw = make_div((uint32_t)p.KW);
    const int step = plan->KS * plan->SK, step_taps = step / p.Cin;
    a.step_ci = step % p.Cin;
    a.step_kh = step_taps / p.KW;
    a.step_kw = step_taps % p.KW;
    return (p.stride_cm == 1 ? plan->launch_mfast : plan->launch_nfast)(a, dim3((unsigned)blocks), stream);
}
