// bf16 prefill attention (Eq. 2).  Placeholder dispatch: the row kernel.
#include <hip/hip_runtime.h>

#include "tca_prefill.h"

namespace tca {

size_t prefill_mfma_workspace_bytes(const tca_params*, int64_t) { return 0; }

int launch_prefill_mfma(const tca_params* prm, const bf16_t* Q, int64_t q_pos0, int64_t n_queries,
                        const bf16_t* K, const bf16_t* V, int64_t kv_stride, const int32_t* idx,
                        const bf16_t* Kg, const bf16_t* Vg, const int64_t* offs, const int32_t* n_rows,
                        bf16_t* O, float* lse, void*, hipStream_t st) {
  return launch_prefill_rows<bf16_t>(prm, Q, q_pos0, n_queries, K, V, kv_stride, idx, Kg, Vg, offs, n_rows,
                                     O, lse, st);
}

}  // namespace tca
