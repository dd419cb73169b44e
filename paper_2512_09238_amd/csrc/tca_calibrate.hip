// Offline head-specific sparsity determination (Alg. 1).  Not implemented yet.
#include <hip/hip_runtime.h>

#include "tca_common.h"

using namespace tca;

extern "C" size_t tca_calibrate_workspace_bytes(const tca_params*, int64_t, int) { return 0; }

extern "C" int tca_calibrate_budgets(const tca_params*, const void*, const void*, int64_t, int, double, double,
                                     double*, int32_t*, double*, int64_t*, int32_t*, void*, size_t, void*) {
  return fail(TCA_ERR_UNSUPPORTED, "tca_calibrate_budgets: not implemented");
}
