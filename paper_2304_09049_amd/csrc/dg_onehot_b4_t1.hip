// The one-hot matrix-core kernels for 4-bit codes, output stride-1 axis = m (NHWC convolution)
// (one translation unit per code width and layout keeps build times even).
#include "dg_onehot_kernel.h"

namespace dgoh {
void launch_bits4_tr1(const DgProblem &p, const Pools &pools, const Plan &q, int64_t blocks11, int64_t wave_tiles,
                        hipStream_t stream)
{
    launch_tr<4, true, false>(p, pools, q, blocks11, wave_tiles, stream);
}
}   // namespace dgoh
