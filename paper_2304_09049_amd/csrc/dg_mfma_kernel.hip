#include "dg_common.h"
bool dg_mfma_supports(const dg_lut *, const DgProblem &) { return false; }
dg_status dg_launch_mfma(const dg_lut *, const DgProblem &, hipStream_t) { return dg_fail(DG_ERR_UNSUPPORTED, "mfma kernel not built"); }
