// 2-bit table kernels on the sparse matrix instruction (activations on the MFMA rows: output stride-1 axis = m), 2 wavefronts sharing a tile.
// (One translation unit per variant keeps build times even.)
#include "dg_onehot_kernel.h"

namespace dgoh {
void unit_main_b20_t1_k2(const DgProblem &p, const Pools &pools, const Plan &q, int64_t wave_tiles, hipStream_t stream)
{
    launch_main<20, true, false, 2>(p, pools, q, wave_tiles, stream);
}
}   // namespace dgoh
