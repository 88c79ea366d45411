// Two-plane 2-bit table kernel on the sparse matrix instruction.
// (One translation unit per variant keeps build times even.)
#include "dg_sparse2p_kernel.h"

namespace dgoh {
void unit_sparse2p(const DgProblem &p, const uint32_t (&rows)[2][4], int ch, hipStream_t stream)
{
    launch_sparse2p(p, rows, ch, stream);
}
}   // namespace dgoh
