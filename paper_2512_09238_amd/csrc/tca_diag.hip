// Diagnostics (declared in tca_diag.h; not part of the method's boundary).
//
// What this board sustains on the matrix pipe.  A register-only loop
// of v_mfma_f32_32x32x16_bf16 (four independent accumulators per wave, four
// waves per SIMD), timed with events, plus the shader clock it ran at
// (cycle counter against the constant 100 MHz counter).  With operands of
// random sign and magnitude the board is power-limited well below its nominal
// clock, which is the ceiling the attention kernel works under.
#include <hip/hip_runtime.h>

#include <atomic>

#include "tca_common.h"
#include "tca_diag.h"
#include "tca_device.h"
#include "tca_prefill.h"

namespace tca {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 probe_bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float probe_f32x16_t;

constexpr int kProbeBlocks = 1024;     // x 4 waves = 4 waves per SIMD on 256 CUs
constexpr int kProbeMfmaPerIter = 16;

__global__ __launch_bounds__(256) void probe_mfma_kernel(int iters, float rnd, unsigned long long* out) {
  probe_bf16x8_t x, y;
  unsigned rs = threadIdx.x * 2654435761u + blockIdx.x * 40503u + 12345u;
  for (int i = 0; i < 8; ++i) {
    rs = rs * 1664525u + 1013904223u;
    x[i] = (__bf16)(rnd * ((int)(rs >> 8) % 2001 - 1000) * 0.001f + (1.f - rnd));
    rs = rs * 1664525u + 1013904223u;
    y[i] = (__bf16)(rnd * ((int)(rs >> 8) % 2001 - 1000) * 0.001f + (1.f - rnd) * 0.5f);
  }
  probe_f32x16_t c0 = {0}, c1 = {0}, c2 = {0}, c3 = {0};
  const unsigned long long t0 = __builtin_readcyclecounter(), r0 = __builtin_amdgcn_s_memrealtime();
  for (int i = 0; i < iters; ++i) {
#pragma unroll
    for (int u = 0; u < kProbeMfmaPerIter / 4; ++u) {
      c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x, y, c0, 0, 0, 0);
      c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x, y, c1, 0, 0, 0);
      c2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x, y, c2, 0, 0, 0);
      c3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x, y, c3, 0, 0, 0);
    }
  }
  const unsigned long long t1 = __builtin_readcyclecounter(), r1 = __builtin_amdgcn_s_memrealtime();
  const float sink = c0[0] + c1[1] + c2[2] + c3[3];
  if (threadIdx.x == 0) {
    out[3 * blockIdx.x] = t1 - t0;
    out[3 * blockIdx.x + 1] = r1 - r0;
    out[3 * blockIdx.x + 2] = __float_as_uint(sink);   // keeps the loop alive
  }
}

static std::atomic<int> g_prefill_clocks{0}, g_prefill_variant{0};
bool diag_prefill_clocks() { return g_prefill_clocks.load(std::memory_order_relaxed) != 0; }
int prefill_variant() { return g_prefill_variant.load(std::memory_order_relaxed); }

}  // namespace tca

using namespace tca;

extern "C" void tca_diag_prefill_clocks(int enable) { g_prefill_clocks.store(enable ? 1 : 0); }

extern "C" int tca_diag_prefill_variant(int variant) {
  if (variant < 0 || variant > 3) return fail(TCA_ERR_INVALID, "tca_diag_prefill_variant: %d", variant);
  g_prefill_variant.store(variant);
  return TCA_OK;
}

extern "C" int64_t tca_diag_prefill_xcd_plan(const tca_params* prm, const int64_t* offs, int64_t q_pos0,
                                             int64_t n_queries, int part, int gather_free, int32_t* start_out) {
  if (check_params(prm) != TCA_OK || prm->dtype != TCA_BF16 || !offs || !start_out || q_pos0 < 0 || n_queries < 1) return -1;
  if (part != TCA_PART_ALL && part != TCA_PART_WINDOW && part != TCA_PART_GLOBAL) return -1;
  return prefill_mfma_xcd_plan(prm, offs, q_pos0, n_queries, part, gather_free != 0, start_out);
}

extern "C" size_t tca_probe_workspace_bytes(void) { return (size_t)kProbeBlocks * 3 * sizeof(unsigned long long); }

extern "C" int tca_probe_mfma(int random_operands, int iters, double* tflops, double* shader_ghz, void* ws,
                              size_t ws_bytes, void* stream) {
  if (!tflops || !shader_ghz || !ws) return fail(TCA_ERR_INVALID, "tca_probe_mfma: NULL pointer argument");
  if (iters < 1 || iters > (1 << 22)) return fail(TCA_ERR_INVALID, "tca_probe_mfma: iters=%d", iters);
  if (ws_bytes < tca_probe_workspace_bytes() || ((uintptr_t)ws & 255))
    return fail(TCA_ERR_WORKSPACE, "tca_probe_mfma: workspace needs %zu bytes, 256-byte aligned",
                tca_probe_workspace_bytes());
  hipStream_t st = (hipStream_t)stream;
  hipEvent_t e0, e1;
  TCA_HIP_CHECK(hipEventCreate(&e0));
  TCA_HIP_CHECK(hipEventCreate(&e1));
  unsigned long long* out = (unsigned long long*)ws;
  const float rnd = random_operands ? 1.f : 0.f;
  hipLaunchKernelGGL(probe_mfma_kernel, dim3(kProbeBlocks), dim3(256), 0, st, iters, rnd, out);   // warm-up
  TCA_HIP_CHECK(hipEventRecord(e0, st));
  hipLaunchKernelGGL(probe_mfma_kernel, dim3(kProbeBlocks), dim3(256), 0, st, iters, rnd, out);
  TCA_HIP_CHECK(hipEventRecord(e1, st));
  TCA_HIP_CHECK(hipEventSynchronize(e1));
  float ms = 0.f;
  TCA_HIP_CHECK(hipEventElapsedTime(&ms, e0, e1));
  unsigned long long h[2 * 3];
  TCA_HIP_CHECK(hipMemcpyAsync(h, out, sizeof(h), hipMemcpyDeviceToHost, st));
  TCA_HIP_CHECK(hipStreamSynchronize(st));
  TCA_HIP_CHECK(hipEventDestroy(e0));
  TCA_HIP_CHECK(hipEventDestroy(e1));
  const double flops = (double)kProbeBlocks * 4 * iters * kProbeMfmaPerIter * (2.0 * 32 * 32 * 16);
  *tflops = flops / (ms * 1e-3) / 1e12;
  *shader_ghz = h[1] ? (double)h[0] / ((double)h[1] * 10.0) : 0.0;
  return TCA_OK;
}
