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

namespace tca {

// Merge of two attention results over disjoint key sets, each normalised by itself, through their
// log-sum-exp (Eq. 2 is one softmax over the union): O = (e^{lse_a} O_a + e^{lse_b} O_b) / (e^{lse_a} + e^{lse_b}).
// grid (ceil(rows/4)); block 256: one wave per row, each lane D/64 columns.  O_a is overwritten.
template <typename T>
__global__ __launch_bounds__(256) void merge_parts_kernel(T* __restrict__ Oa, const float* __restrict__ lse_a,
                                                          const T* __restrict__ Ob, const float* __restrict__ lse_b,
                                                          float* __restrict__ lse_out, int64_t rows, int D) {
  const int64_t r = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= rows) return;
  const int lane = threadIdx.x & 63;
  const float la = lse_a[r], lb = lse_b[r];
  const float mx = fmaxf(la, lb);
  const float wa = la == -INFINITY ? 0.f : expf(la - mx), wb = lb == -INFINITY ? 0.f : expf(lb - mx);
  const float inv = 1.f / (wa + wb);                   // every query sees itself: at least one part is not empty
  for (int e = lane; e < D; e += 64) {
    const float a = wa > 0.f ? load_f32(Oa + r * D + e) * wa : 0.f;
    const float b = wb > 0.f ? load_f32(Ob + r * D + e) * wb : 0.f;
    store_f32(Oa + r * D + e, (a + b) * inv);
  }
  if (lse_out && lane == 0) lse_out[r] = mx + logf(wa + wb);
}

static int prefill_checked(const tca_params* prm, const void* Q, int64_t q_pos0, int64_t n_queries, const void* K,
                           const void* V, int64_t kv_stride, const int32_t* idx, const void* Kg, const void* Vg,
                           const int64_t* offs, const int32_t* n_rows, void* O, float* lse, void* ws,
                           size_t ws_bytes, void* stream, int part, const char* who) {
  int rc = check_params(prm);
  if (rc) return rc;
  if (!Q || !K || !V || !idx || !offs || !n_rows || !O)
    return fail(TCA_ERR_INVALID, "%s: NULL pointer argument", who);
  if ((Kg == nullptr) != (Vg == nullptr))
    return fail(TCA_ERR_INVALID, "%s: Kg and Vg must both be given, or both be NULL (gather-free call)", who);
  if (part != TCA_PART_ALL && part != TCA_PART_WINDOW && part != TCA_PART_GLOBAL)
    return fail(TCA_ERR_INVALID, "%s: part=%d", who, part);
  if (part != TCA_PART_ALL && !lse) return fail(TCA_ERR_INVALID, "%s: a part needs lse to be merged", who);
  if (n_queries < 0 || q_pos0 < 0 || q_pos0 + n_queries > kv_stride)
    return fail(TCA_ERR_INVALID, "%s: q_pos0=%lld n_queries=%lld kv_stride=%lld", who, (long long)q_pos0,
                (long long)n_queries, (long long)kv_stride);
  if (q_pos0 + n_queries > INT32_MAX) return fail(TCA_ERR_UNSUPPORTED, "positions beyond int32");
  if (offs[0] != 0) return fail(TCA_ERR_INVALID, "%s: offs[0] must be 0", who);
  for (int h = 0; h < sel_heads(prm); ++h)
    if (offs[h + 1] < offs[h]) return fail(TCA_ERR_INVALID, "%s: offs not ascending at %d", who, h);
  const size_t need = tca_prefill_workspace_bytes(prm, n_queries, offs[sel_heads(prm)]);
  if (need && (!ws || ws_bytes < need || ((uintptr_t)ws & 255)))
    return fail(TCA_ERR_WORKSPACE, "%s: workspace needs %zu bytes, 256-byte aligned", who, need);
  if (n_queries == 0) return TCA_OK;
  hipStream_t st = (hipStream_t)stream;
  if (prm->dtype == TCA_F32) {
    rc = launch_prefill_rows<float>(prm, (const float*)Q, q_pos0, n_queries, (const float*)K,
                                    (const float*)V, kv_stride, idx, (const float*)Kg, (const float*)Vg,
                                    offs, n_rows, (float*)O, lse, st, part);
  } else {
    rc = launch_prefill_mfma(prm, (const bf16_t*)Q, q_pos0, n_queries, (const bf16_t*)K, (const bf16_t*)V,
                             kv_stride, idx, (const bf16_t*)Kg, (const bf16_t*)Vg, offs, n_rows,
                             (bf16_t*)O, lse, ws, st, part);
  }
  if (rc) return rc;
  TCA_HIP_CHECK(hipGetLastError());
  return TCA_OK;
}

}  // namespace tca

extern "C" int tca_prefill(const tca_params* prm, const void* Q, int64_t q_pos0, int64_t n_queries,
                           const void* K, const void* V, int64_t kv_stride, const int32_t* idx,
                           const void* Kg, const void* Vg, const int64_t* offs, const int32_t* n_rows,
                           void* O, float* lse, void* ws, size_t ws_bytes, void* stream) {
  return prefill_checked(prm, Q, q_pos0, n_queries, K, V, kv_stride, idx, Kg, Vg, offs, n_rows, O, lse, ws, ws_bytes,
                         stream, TCA_PART_ALL, "tca_prefill");
}

extern "C" int tca_prefill_part(const tca_params* prm, int part, const void* Q, int64_t q_pos0, int64_t n_queries,
                                const void* K, const void* V, int64_t kv_stride, const int32_t* idx,
                                const void* Kg, const void* Vg, const int64_t* offs, const int32_t* n_rows,
                                void* O, float* lse, void* ws, size_t ws_bytes, void* stream) {
  return prefill_checked(prm, Q, q_pos0, n_queries, K, V, kv_stride, idx, Kg, Vg, offs, n_rows, O, lse, ws, ws_bytes,
                         stream, part, "tca_prefill_part");
}

extern "C" int tca_prefill_merge(const tca_params* prm, int64_t n_queries, void* O_a, const float* lse_a,
                                 const void* O_b, const float* lse_b, float* lse_out, void* stream) {
  int rc = check_params(prm);
  if (rc) return rc;
  if (!O_a || !lse_a || !O_b || !lse_b || n_queries < 0)
    return fail(TCA_ERR_INVALID, "tca_prefill_merge: NULL pointer argument or n_queries=%lld", (long long)n_queries);
  const int64_t rows = (int64_t)prm->n_q_heads * n_queries;
  if (rows == 0) return TCA_OK;
  hipStream_t st = (hipStream_t)stream;
  const dim3 grid((unsigned)((rows + 3) / 4));
  if (prm->dtype == TCA_BF16)
    hipLaunchKernelGGL((merge_parts_kernel<bf16_t>), grid, dim3(256), 0, st, (bf16_t*)O_a, lse_a, (const bf16_t*)O_b,
                       lse_b, lse_out, rows, prm->head_dim);
  else
    hipLaunchKernelGGL((merge_parts_kernel<float>), grid, dim3(256), 0, st, (float*)O_a, lse_a, (const float*)O_b, lse_b,
                       lse_out, rows, prm->head_dim);
  TCA_HIP_CHECK(hipGetLastError());
  return TCA_OK;
}

// Alg. 2 with the window part of the attention started before the selection (App. C, the
// overlap named there as a further optimisation): on `side_stream` the attention of every query
// over its window alone, which needs nothing the selection produces; on `stream` the selection,
// then the attention over the selected rows alone; then the merge of the two through their lse.
extern "C" int tca_select_prefill_overlapped(const tca_params* prm, const void* q_last, const void* Q,
                                             const void* K, const void* V, int64_t kv_stride, int64_t pos0,
                                             int64_t n_tokens, const double* p, const int64_t* offs,
                                             int32_t* n_rows, int32_t* idx, void* Kg, void* Vg, void* O,
                                             void* O_part, float* lse_parts, void* ws_select,
                                             size_t ws_select_bytes, void* ws_prefill, size_t ws_prefill_bytes,
                                             void* stream, void* side_stream) {
  int rc = check_params(prm);
  if (rc) return rc;
  if (!O_part || !lse_parts || !side_stream || side_stream == stream)
    return fail(TCA_ERR_INVALID, "tca_select_prefill_overlapped: needs O_part, lse_parts and a second stream");
  const int64_t n_lse = (int64_t)prm->n_q_heads * n_tokens;
  hipStream_t st = (hipStream_t)stream, side = (hipStream_t)side_stream;
  hipEvent_t ready = nullptr, window_done = nullptr;
  auto finish = [&](int code) {                   // the events go on every way out
    if (ready) (void)hipEventDestroy(ready);
    if (window_done) (void)hipEventDestroy(window_done);
    return code;
  };
  auto hip_ok = [&](hipError_t e, const char* what) {
    return e == hipSuccess ? TCA_OK : fail(TCA_ERR_HIP, "tca_select_prefill_overlapped: %s: %s", what, hipGetErrorString(e));
  };
  if ((rc = hip_ok(hipEventCreateWithFlags(&ready, hipEventDisableTiming), "event"))) return finish(rc);
  if ((rc = hip_ok(hipEventCreateWithFlags(&window_done, hipEventDisableTiming), "event"))) return finish(rc);
  // the inputs are ready where `stream` stands now
  if ((rc = hip_ok(hipEventRecord(ready, st), "record"))) return finish(rc);
  if ((rc = hip_ok(hipStreamWaitEvent(side, ready, 0), "wait"))) return finish(rc);
  rc = prefill_checked(prm, Q, pos0, n_tokens, K, V, kv_stride, idx, Kg, Vg, offs, n_rows, O_part, lse_parts,
                       ws_prefill, ws_prefill_bytes, side, TCA_PART_WINDOW, "tca_select_prefill_overlapped (window)");
  if (rc) return finish(rc);
  if ((rc = hip_ok(hipEventRecord(window_done, side), "record"))) return finish(rc);
  rc = tca_select(prm, q_last, K, V, kv_stride, pos0, n_tokens, p, offs, n_rows, idx, Kg, Vg, ws_select,
                  ws_select_bytes, stream);
  if (rc) return finish(rc);
  rc = prefill_checked(prm, Q, pos0, n_tokens, K, V, kv_stride, idx, Kg, Vg, offs, n_rows, O, lse_parts + n_lse,
                       ws_prefill, ws_prefill_bytes, stream, TCA_PART_GLOBAL, "tca_select_prefill_overlapped (global)");
  if (rc) return finish(rc);
  if ((rc = hip_ok(hipStreamWaitEvent(st, window_done, 0), "wait"))) return finish(rc);
  rc = tca_prefill_merge(prm, n_tokens, O, lse_parts + n_lse, O_part, lse_parts, nullptr, stream);
  return finish(rc);
}
