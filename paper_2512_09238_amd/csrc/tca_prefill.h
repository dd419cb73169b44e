// Internal launchers of the two prefill kernels (Eq. 2).
#pragma once

#include <hip/hip_runtime.h>

#include "tca_common.h"
#include "tca_device.h"

namespace tca {

// One wavefront per query, fp32 arithmetic; any storage type.
template <typename T>
int launch_prefill_rows(const tca_params* prm, const T* Q, int64_t q_pos0, int64_t n_queries, const T* K,
                        const T* V, int64_t kv_stride, const int32_t* idx, const T* Kg, const T* Vg,
                        const int64_t* offs, const int32_t* n_rows, T* O, float* lse, hipStream_t st, int part);

// bf16 MFMA flash kernel.
size_t prefill_mfma_workspace_bytes(const tca_params* prm, int64_t n_queries, int64_t cap_rows);
int launch_prefill_mfma(const tca_params* prm, const bf16_t* Q, int64_t q_pos0, int64_t n_queries,
                        const bf16_t* K, const bf16_t* V, int64_t kv_stride, const int32_t* idx,
                        const bf16_t* Kg, const bf16_t* Vg, const int64_t* offs, const int32_t* n_rows,
                        bf16_t* O, float* lse, void* ws, hipStream_t st, int part);
// The ranges of the (head, query tile) sequence the eight XCDs work through for such a call
// (start_out[9]); returns the number of workgroups launched, -1 if the head count is not a multiple of 8.
int64_t prefill_mfma_xcd_plan(const tca_params* prm, const int64_t* offs, int64_t q_pos0, int64_t n_queries, int part,
                              bool gather, int32_t* start_out);

}  // namespace tca
