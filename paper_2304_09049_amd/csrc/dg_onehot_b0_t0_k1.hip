// Decode-and-multiply comparison kernels (2-bit codes to int8 levels, int8 MFMA), output stride-1 axis = n (row-major GEMM) or neither.
// (One translation unit per variant keeps build times even.)
#include "dg_onehot_kernel.h"

namespace dgoh {
void unit_main_b0_t0_k1(const DgProblem &p, const Pools &pools, const Plan &q, int64_t wave_tiles, hipStream_t stream)
{
    launch_main<0, false, false, 1>(p, pools, q, wave_tiles, stream);
}

void unit_split_b0_t0(const DgProblem &p, const Pools &pools, const Plan &q, int64_t blocks11, hipStream_t stream)
{
    launch_split<0, false, false>(p, pools, q, blocks11, stream);
}
}   // namespace dgoh
