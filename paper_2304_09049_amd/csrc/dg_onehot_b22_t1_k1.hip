// One-hot matrix-core kernels: 2-bit codes with entries beyond int8 (two int8 planes), output stride-1 axis = m (NHWC convolution).
// (One translation unit per variant keeps build times even.)
#include "dg_onehot_kernel.h"

namespace dgoh {
void unit_main_b22_t1_k1(const DgProblem &p, const Pools &pools, const Plan &q, int64_t wave_tiles, hipStream_t stream)
{
    launch_main<2, true, true, 1>(p, pools, q, wave_tiles, stream);
}

void unit_split_b22_t1(const DgProblem &p, const Pools &pools, const Plan &q, int64_t blocks11, hipStream_t stream)
{
    launch_split<2, true, true>(p, pools, q, blocks11, stream);
}
}   // namespace dgoh
