// tca_prefill entry point (Eq. 2; Alg. 2 line 7): argument checks and dispatch.
#include <hip/hip_runtime.h>

#include "tca_common.h"
#include "tca_device.h"
#include "tca_prefill.h"

using namespace tca;

extern "C" size_t tca_prefill_workspace_bytes(const tca_params* prm, int64_t n_queries, int64_t cap_rows) {
  if (check_params(prm) != TCA_OK || n_queries < 0 || cap_rows < 0) return 0;
  if (prm->dtype != TCA_BF16) return 0;
  return prefill_mfma_workspace_bytes(prm, n_queries, cap_rows);
}

extern "C" int tca_prefill(const tca_params* prm, const void* Q, int64_t q_pos0, int64_t n_queries,
                           const void* K, const void* V, int64_t kv_stride, const int32_t* idx,
                           const void* Kg, const void* Vg, const int64_t* offs, const int32_t* n_rows,
                           void* O, float* lse, void* ws, size_t ws_bytes, void* stream) {
  int rc = check_params(prm);
  if (rc) return rc;
  if (!Q || !K || !V || !idx || !offs || !n_rows || !O)
    return fail(TCA_ERR_INVALID, "tca_prefill: NULL pointer argument");
  if ((Kg == nullptr) != (Vg == nullptr))
    return fail(TCA_ERR_INVALID, "tca_prefill: Kg and Vg must both be given, or both be NULL (gather-free call)");
  if (n_queries < 0 || q_pos0 < 0 || q_pos0 + n_queries > kv_stride)
    return fail(TCA_ERR_INVALID, "tca_prefill: q_pos0=%lld n_queries=%lld kv_stride=%lld",
                (long long)q_pos0, (long long)n_queries, (long long)kv_stride);
  if (q_pos0 + n_queries > INT32_MAX) return fail(TCA_ERR_UNSUPPORTED, "positions beyond int32");
  if (offs[0] != 0) return fail(TCA_ERR_INVALID, "tca_prefill: offs[0] must be 0");
  for (int h = 0; h < sel_heads(prm); ++h)
    if (offs[h + 1] < offs[h]) return fail(TCA_ERR_INVALID, "tca_prefill: offs not ascending at %d", h);
  const size_t need = tca_prefill_workspace_bytes(prm, n_queries, offs[sel_heads(prm)]);
  if (need && (!ws || ws_bytes < need || ((uintptr_t)ws & 255)))
    return fail(TCA_ERR_WORKSPACE, "tca_prefill: workspace needs %zu bytes, 256-byte aligned", need);
  if (n_queries == 0) return TCA_OK;
  hipStream_t st = (hipStream_t)stream;
  if (prm->dtype == TCA_F32) {
    rc = launch_prefill_rows<float>(prm, (const float*)Q, q_pos0, n_queries, (const float*)K,
                                    (const float*)V, kv_stride, idx, (const float*)Kg, (const float*)Vg,
                                    offs, n_rows, (float*)O, lse, st);
  } else {
    rc = launch_prefill_mfma(prm, (const bf16_t*)Q, q_pos0, n_queries, (const bf16_t*)K, (const bf16_t*)V,
                             kv_stride, idx, (const bf16_t*)Kg, (const bf16_t*)Vg, offs, n_rows,
                             (bf16_t*)O, lse, ws, st);
  }
  if (rc) return rc;
  TCA_HIP_CHECK(hipGetLastError());
  return TCA_OK;
}
