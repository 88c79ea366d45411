// 2-bit table kernel on the sparse matrix instruction with the weight operands stationary in registers.
// (One translation unit per variant keeps build times even.)
#include "dg_sparse_ws_kernel.h"

namespace dgoh {
void unit_sparse_ws(const DgProblem &p, const uint32_t (&rows)[4], int streams, bool raw, hipStream_t stream)
{
    launch_sparse_ws(p, rows, streams, raw, stream);
}
}   // namespace dgoh
