// Layer integration in front of the path (extensions; the paper takes Q and K as given, after
// position encoding): rotary position embedding of Q / K rows, in place.
//
// The pair (x_a, x_b) of a row at position t is turned by the angle t * base^(-2i/d),
// i = 0 .. d/2-1 (the RoFormer rotation); pair i is (i, i + d/2) or (2i, 2i+1).  Angles, sines and
// cosines are fp64 (a position of 10^5 times a frequency near 1 leaves fp32 no fraction digits
// to speak of), one per (row, pair), shared by the heads; the products are fp64 and rounded once
// to the storage type, so the result is the correctly rounded rotation up to the last fp64 digit.
#include <hip/hip_runtime.h>

#include "tca_common.h"
#include "tca_device.h"

namespace tca {

// grid (ceil(n_rows / 4)); block 256: 4 rows per workgroup, thread (row, pair i) loops over the heads
template <typename T>
__global__ __launch_bounds__(256) void rope_kernel(T* __restrict__ X, int n_heads, int64_t n_rows, int d, int64_t pos0,
                                                   double log2_base, int interleaved) {
  const int half = d >> 1;
  const int per_row = 256 / 4;                                   // threads per row: 64 >= d/2
  const int64_t r = (int64_t)blockIdx.x * 4 + threadIdx.x / per_row;
  const int i = threadIdx.x % per_row;
  if (r >= n_rows || i >= half) return;
  const double inv_freq = exp2(-2.0 * (double)i / (double)d * log2_base);
  const double ang = (double)(pos0 + r) * inv_freq;
  double sn, cs;
  sincos(ang, &sn, &cs);
  const int ia = interleaved ? 2 * i : i, ib = interleaved ? 2 * i + 1 : i + half;
  for (int h = 0; h < n_heads; ++h) {
    T* row = X + ((size_t)h * n_rows + r) * d;
    const double a = (double)load_f32(row + ia), b = (double)load_f32(row + ib);
    store_f32(row + ia, (float)(a * cs - b * sn));
    store_f32(row + ib, (float)(b * cs + a * sn));
  }
}

}  // namespace tca

using namespace tca;

extern "C" int tca_rope(const tca_params* prm, void* X, int n_heads, int64_t n_rows, int64_t pos0, double base,
                        int pairing, void* stream) {
  int rc = check_params(prm);
  if (rc) return rc;
  if (!X || n_heads < 1 || n_rows < 0 || pos0 < 0 || !(base > 1.0))
    return fail(TCA_ERR_INVALID, "tca_rope: X=%p n_heads=%d n_rows=%lld pos0=%lld base=%g", X, n_heads,
                (long long)n_rows, (long long)pos0, base);
  if (pairing != TCA_ROPE_HALF && pairing != TCA_ROPE_INTERLEAVED)
    return fail(TCA_ERR_UNSUPPORTED, "tca_rope: pairing=%d", pairing);
  if (n_rows == 0) return TCA_OK;
  hipStream_t st = (hipStream_t)stream;
  const dim3 grid((unsigned)((n_rows + 3) / 4));
  const double l2b = __builtin_log2(base);
  if (prm->dtype == TCA_BF16)
    hipLaunchKernelGGL((rope_kernel<bf16_t>), grid, dim3(256), 0, st, (bf16_t*)X, n_heads, n_rows, prm->head_dim, pos0,
                       l2b, pairing == TCA_ROPE_INTERLEAVED);
  else
    hipLaunchKernelGGL((rope_kernel<float>), grid, dim3(256), 0, st, (float*)X, n_heads, n_rows, prm->head_dim, pos0,
                       l2b, pairing == TCA_ROPE_INTERLEAVED);
  TCA_HIP_CHECK(hipGetLastError());
  return TCA_OK;
}
