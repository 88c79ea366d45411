// One-hot split-K kernel on activations still one code per byte (the packing stage done in its load stage).
// (One translation unit per variant keeps build times even.)
#include "dg_onehot_kernel.h"

namespace dgoh {
void unit_split_codes(const DgProblem &p, const Pools &pools, const Plan &q, bool two, bool tr, int64_t blocks11,
                      hipStream_t stream)
{
    if (two) {
        if (tr)
            launch_split<2, true, true, true>(p, pools, q, blocks11, stream);
        else
            launch_split<2, false, true, true>(p, pools, q, blocks11, stream);
    } else {
        if (tr)
            launch_split<2, true, false, true>(p, pools, q, blocks11, stream);
        else
            launch_split<2, false, false, true>(p, pools, q, blocks11, stream);
    }
}

namespace {
template <int WN>
void launch_codes_tile_sparse(const Args &a, int skw, int64_t wave_tiles, hipStream_t stream)
{
    const dim3 grid((unsigned)((wave_tiles + 4 / skw - 1) / (4 / skw)));
    if (skw == 4)
        hipLaunchKernelGGL((onehot_mfma_kernel<20, 2, WN, 2, true, false, 4, true>), grid, dim3(256), (main_lds_bytes<2, WN, false, 4>()), stream, a);
    else if (skw == 2)
        hipLaunchKernelGGL((onehot_mfma_kernel<20, 2, WN, 2, true, false, 2, true>), grid, dim3(256), (main_lds_bytes<2, WN, false, 2>()), stream, a);
    else
        hipLaunchKernelGGL((onehot_mfma_kernel<20, 2, WN, 2, true, false, 1, true>), grid, dim3(256), 0, stream, a);
}

template <int WN, bool TR>
void launch_codes_tile(const Args &a, int skw, int64_t wave_tiles, hipStream_t stream)
{
    const dim3 grid((unsigned)((wave_tiles + 4 / skw - 1) / (4 / skw)));
    if (skw == 4)
        hipLaunchKernelGGL((onehot_mfma_kernel<2, 2, WN, 2, TR, false, 4, true>), grid, dim3(256), (main_lds_bytes<2, WN, false, 4>()), stream, a);
    else if (skw == 2)
        hipLaunchKernelGGL((onehot_mfma_kernel<2, 2, WN, 2, TR, false, 2, true>), grid, dim3(256), (main_lds_bytes<2, WN, false, 2>()), stream, a);
    else
        hipLaunchKernelGGL((onehot_mfma_kernel<2, 2, WN, 2, TR, false, 1, true>), grid, dim3(256), 0, stream, a);
}
}   // namespace

void unit_main_codes(const DgProblem &p, const Pools &pools, const Plan &q, bool tr, bool sparse, int64_t wave_tiles, hipStream_t stream)
{
    Args a{};
    a.p = p;
    a.pools = pools;
    a.tiles_m = (p.M + 63) / 64;
    a.wave_tiles = wave_tiles;
    a.div_ow = make_div((uint32_t)p.OW), a.div_oh = make_div((uint32_t)p.OH);
    a.div_cin = make_div((uint32_t)p.Cin), a.div_kw = make_div((uint32_t)p.KW);
    if (sparse) {
        if (q.wn == 2)
            launch_codes_tile_sparse<2>(a, q.skw, wave_tiles, stream);
        else
            launch_codes_tile_sparse<1>(a, q.skw, wave_tiles, stream);
        return;
    }
    if (q.wn == 2) {
        if (tr)
            launch_codes_tile<2, true>(a, q.skw, wave_tiles, stream);
        else
            launch_codes_tile<2, false>(a, q.skw, wave_tiles, stream);
    } else {
        if (tr)
            launch_codes_tile<1, true>(a, q.skw, wave_tiles, stream);
        else
            launch_codes_tile<1, false>(a, q.skw, wave_tiles, stream);
    }
}
}   // namespace dgoh
