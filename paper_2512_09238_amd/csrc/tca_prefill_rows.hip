// Row-wise prefill attention (Eq. 2; Alg. 2 line 7): one wavefront per query.
//
// This is the fp32 path (TCA_F32) and the plain cross-check for the MFMA
// kernel: every query walks its own key list - the head's visible global rows
// (idx <= i-w) followed by its window (i-w, i] - with an online softmax.  A
// wave is split into four 16-lane groups; a group owns every fourth key, each
// lane a D/16 slice of the row, so the q.k reduction is a 4-step butterfly and
// the P.V accumulation needs no communication.  Groups are merged at the end.
// Logits and the running maximum are fp64 (the products of fp32 or bf16 inputs are
// exact in it), so that the exponent x - max carries no cancellation error even
// when the logits are in the hundreds; exponentials, sums and P.V are fp32.
#include <hip/hip_runtime.h>

#include "tca_common.h"
#include "tca_device.h"

namespace tca {

constexpr int kRowThreads = 256;

// count of entries <= bound in ascending idx[0..n)
__device__ __forceinline__ int count_le(const int32_t* idx, int n, int64_t bound) {
  int lo = 0, hi = n;
  while (lo < hi) {
    const int mid = (lo + hi) >> 1;
    if ((int64_t)idx[mid] <= bound) lo = mid + 1; else hi = mid;
  }
  return lo;
}

struct HeadOffs { int64_t offs[TCA_MAX_HEADS + 1]; };

template <typename T, int D>
__global__ __launch_bounds__(kRowThreads) void prefill_rows_kernel(
    const T* __restrict__ Q, int64_t q_pos0, int64_t n_queries, const T* __restrict__ K,
    const T* __restrict__ V, int64_t kv_stride, const int32_t* __restrict__ idx,
    const T* __restrict__ Kg, const T* __restrict__ Vg, HeadOffs ho,
    const int32_t* __restrict__ n_rows, int G, int GS, int w, double scale, T* __restrict__ O,
    float* __restrict__ lse, int part) {
  constexpr int EL = D / 16;                       // elements of a row per lane
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const int grp = lane >> 4, sub = lane & 15;
  const int h = blockIdx.y, kvh = h / G;
  const int64_t r = (int64_t)blockIdx.x * (kRowThreads / kWave) + wv;
  if (r >= n_queries) return;
  const int64_t i = q_pos0 + r;                    // position of this query

  double q[EL];
#pragma unroll
  for (int e = 0; e < EL; ++e) q[e] = (double)load_f32(Q + ((size_t)h * n_queries + r) * D + sub * EL + e);

  const int hs = h / GS;                           // the selection this query head reads
  const int64_t base = ho.offs[hs];
  // part: both key subsets, or one of them alone (normalised by itself; merged later through lse)
  const int n_glob = part == TCA_PART_WINDOW ? 0 : count_le(idx + base, n_rows[hs], i - w);
  const int64_t win0 = i - w + 1 > 0 ? i - w + 1 : 0;
  const int64_t n_keys = n_glob + (part == TCA_PART_GLOBAL ? 0 : i - win0 + 1);

  double m = -INFINITY;
  float l = 0.f, acc[EL];
#pragma unroll
  for (int e = 0; e < EL; ++e) acc[e] = 0.f;

  for (int64_t k0 = 0; k0 < n_keys; k0 += 4) {
    const int64_t k = k0 + grp;
    const bool ok = k < n_keys;
    const T *kr = K, *vr = V;
    if (ok) {
      if (k < n_glob) {
        if (Kg) {
          kr = Kg + (size_t)(base + k) * D;
          vr = Vg + (size_t)(base + k) * D;
        } else {                                       // gather-free call: the kept rows are read where they lie
          const size_t row = (size_t)kvh * kv_stride + idx[base + k];
          kr = K + row * D;
          vr = V + row * D;
        }
      } else {
        const size_t row = (size_t)kvh * kv_stride + (win0 + (k - n_glob));
        kr = K + row * D;
        vr = V + row * D;
      }
    }
    double s = 0.0;
    if (ok) {
#pragma unroll
      for (int e = 0; e < EL; ++e) s = fma(q[e], (double)load_f32(kr + sub * EL + e), s);
    }
    s = row16_sum(s) * scale;
    if (ok) {
      const double mn = fmax(m, s);
      const float corr = expf((float)(m - mn)), pr = expf((float)(s - mn));   // m = -inf: corr = 0
      l = l * corr + pr;
#pragma unroll
      for (int e = 0; e < EL; ++e) acc[e] = acc[e] * corr + pr * load_f32(vr + sub * EL + e);
      m = mn;
    }
  }
  // merge the four groups (lanes with equal `sub`)
  for (int o = 16; o < 64; o <<= 1) {
    const double mo = __shfl_xor(m, o, kWave);
    const float lo = __shfl_xor(l, o, kWave);
    const double mn = fmax(m, mo);
    const float ca = (m == -INFINITY) ? 0.f : expf((float)(m - mn));
    const float cb = (mo == -INFINITY) ? 0.f : expf((float)(mo - mn));
    l = l * ca + lo * cb;
#pragma unroll
    for (int e = 0; e < EL; ++e) acc[e] = acc[e] * ca + __shfl_xor(acc[e], o, kWave) * cb;
    m = mn;
  }
  if (grp == 0) {
    const float inv = l > 0.f ? 1.f / l : 0.f;         // an empty part: zeros, lse = -inf
#pragma unroll
    for (int e = 0; e < EL; ++e) store_f32(O + ((size_t)h * n_queries + r) * D + sub * EL + e, acc[e] * inv);
    if (lse && sub == 0) lse[(size_t)h * n_queries + r] = l > 0.f ? (float)(m + log((double)l)) : -INFINITY;
  }
}

template <typename T>
int launch_prefill_rows(const tca_params* prm, const T* Q, int64_t q_pos0, int64_t n_queries, const T* K,
                        const T* V, int64_t kv_stride, const int32_t* idx, const T* Kg, const T* Vg,
                        const int64_t* offs, const int32_t* n_rows, T* O, float* lse, hipStream_t st, int part) {
  HeadOffs ho;
  for (int h = 0; h <= sel_heads(prm); ++h) ho.offs[h] = offs[h];
  const int GS = sel_group(prm);
  const int G = prm->n_q_heads / prm->n_kv_heads;
  dim3 grid((unsigned)((n_queries + 3) / 4), prm->n_q_heads);
  const double scale = logit_scale(prm);
  if (prm->head_dim == 128)
    hipLaunchKernelGGL((prefill_rows_kernel<T, 128>), grid, dim3(kRowThreads), 0, st, Q, q_pos0, n_queries,
                       K, V, kv_stride, idx, Kg, Vg, ho, n_rows, G, GS, prm->window, scale, O, lse, part);
  else
    hipLaunchKernelGGL((prefill_rows_kernel<T, 64>), grid, dim3(kRowThreads), 0, st, Q, q_pos0, n_queries,
                       K, V, kv_stride, idx, Kg, Vg, ho, n_rows, G, GS, prm->window, scale, O, lse, part);
  return TCA_OK;
}

template int launch_prefill_rows<float>(const tca_params*, const float*, int64_t, int64_t, const float*,
                                        const float*, int64_t, const int32_t*, const float*, const float*,
                                        const int64_t*, const int32_t*, float*, float*, hipStream_t, int);
template int launch_prefill_rows<bf16_t>(const tca_params*, const bf16_t*, int64_t, int64_t, const bf16_t*,
                                         const bf16_t*, int64_t, const int32_t*, const bf16_t*,
                                         const bf16_t*, const int64_t*, const int32_t*, bf16_t*, float*,
                                         hipStream_t, int);

}  // namespace tca
