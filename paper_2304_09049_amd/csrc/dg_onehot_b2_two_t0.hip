// The one-hot matrix-core kernels for 2-bit codes with entries beyond int8 (two int8 planes), output stride-1 axis =
// n (row-major GEMM) or neither (one translation unit per variant keeps build times even).
#include "dg_onehot_kernel.h"

namespace dgoh {
void launch_bits2_two_tr0(const DgProblem &p, const Pools &pools, const Plan &q, int64_t blocks11, int64_t wave_tiles,
                          hipStream_t stream)
{
    launch_tr<2, false, true>(p, pools, q, blocks11, wave_tiles, stream);
}
}   // namespace dgoh
