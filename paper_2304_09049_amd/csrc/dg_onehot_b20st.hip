// 2-bit table kernel on the sparse matrix instruction with the operands staged through LDS in whole 32-byte runs.
// (One translation unit per variant keeps build times even.)
#include "dg_sparse_staged_kernel.h"

namespace dgoh {
void unit_sparse_staged(const DgProblem &p, const Pools &pools, int32_t bias, const Plan &q, int64_t wave_tiles, hipStream_t stream)
{
    launch_sparse_staged(p, pools, bias, q, wave_tiles, stream);
}
}   // namespace dgoh
