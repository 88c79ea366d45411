// 4-bit table kernel on the sparse matrix instruction.
// (One translation unit per variant keeps build times even.)
#include "dg_sparse4_kernel.h"

namespace dgoh {
void unit_sparse4(const DgProblem &p, const uint32_t (&rows)[16][4], int ch, hipStream_t stream)
{
    launch_sparse4(p, rows, ch, stream);
}
}   // namespace dgoh
