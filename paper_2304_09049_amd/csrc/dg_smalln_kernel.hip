#include "dg_common.h"
bool dg_smalln_supports(const dg_lut *, const DgProblem &) { return false; }
dg_status dg_launch_smalln(const dg_lut *, const DgProblem &, hipStream_t) { return dg_fail(DG_ERR_UNSUPPORTED, "smalln kernel not built"); }
