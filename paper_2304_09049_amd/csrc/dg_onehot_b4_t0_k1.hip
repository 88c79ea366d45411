// One-hot matrix-core kernels: 4-bit codes, output stride-1 axis = n (row-major GEMM) or neither.
// (One translation unit per variant keeps build times even.)
#include "dg_onehot_kernel.h"

namespace dgoh {
void unit_main_b4_t0_k1(const DgProblem &p, const Pools &pools, const Plan &q, int64_t wave_tiles, hipStream_t stream)
{
    launch_main<4, false, false, 1>(p, pools, q, wave_tiles, stream);
}

void unit_split_b4_t0(const DgProblem &p, const Pools &pools, const Plan &q, int64_t blocks11, hipStream_t stream)
{
    launch_split<4, false, false>(p, pools, q, blocks11, stream);
}
}   // namespace dgoh
