// One-hot split-K kernel on activations still one code per byte (the packing stage done in its load stage).
// (One translation unit per variant keeps build times even.)
#include "dg_onehot_kernel.h"

namespace dgoh {
void unit_split_codes(const DgProblem &p, const Pools &pools, const Plan &q, bool two, bool tr, int64_t blocks11,
                      hipStream_t stream)
{
    if (two) {
        if (tr)
            launch_split<2, true, true, true>(p, pools, q, blocks11, stream);
        else
            launch_split<2, false, true, true>(p, pools, q, blocks11, stream);
    } else {
        if (tr)
            launch_split<2, true, false, true>(p, pools, q, blocks11, stream);
        else
            launch_split<2, false, false, true>(p, pools, q, blocks11, stream);
    }
}
}   // namespace dgoh
