// Offline head-specific sparsity determination (Alg. 1; Eq. 3, Eq. 4).
//
// Runs once per model, so everything is fp64 and written for exactness, not
// speed: the decisions a_i >= tau then agree with an fp64 reference except at
// exact ties.  The dense causal attention matrix A is never materialised:
//   rowstats  : per query row j, max and sum of exp of the causal logits        (softmax denominators)
//   colmeans  : per key column k, sum_{j>=k} exp(x_jk - max_j) / sum_j, divided
//               by the structural column count L-k                              (Eq. 4 inner term)
// Both kernels give one wavefront to a row (column).  Its four 16-lane groups take 16 keys
// (queries) each per iteration; a lane holds a D/16 slice of the vectors and forms its slice of
// all 16 dot products, and a transposed butterfly (each exchange halves the products a lane still
// carries) leaves every lane with the total of a different key: 64 logits, and 64 useful
// exponentials, per wave and iteration.
// The selection of every candidate reuses the online-selection stages (scores
// and in-block ranks once, budgets per candidate); cand_score sums the column
// means of the tokens a candidate keeps (Eq. 4).
#include <hip/hip_runtime.h>

#include <vector>

#include "tca_common.h"
#include "tca_device.h"
#include "tca_select.h"

namespace tca {

constexpr int kCalThreads = 256;

template <typename T, int EL>
__device__ __forceinline__ void load_slice_f64(const T* p, double (&out)[EL]) {
  float tmp[EL];
  load_slice<T, EL>(p, tmp);
#pragma unroll
  for (int e = 0; e < EL; ++e) out[e] = (double)tmp[e];
}

// merge the (m, l) pairs of all 64 lanes of a wave
__device__ __forceinline__ void merge_lanes(double& m, double& l) {
  for (int o = 1; o < 64; o <<= 1) {
    const double mo = __shfl_xor(m, o, kWave), lo = __shfl_xor(l, o, kWave);
    const double mn = fmax(m, mo);
    const double a = (m == -INFINITY) ? 0.0 : exp(m - mn);
    const double b = (mo == -INFINITY) ? 0.0 : exp(mo - mn);
    l = l * a + lo * b;
    m = mn;
  }
}

// Dot products of this lane's slice `fixed` with the same slice of 16 consecutive rows starting
// at rows + r0 (rows at or beyond r_end count as zero), summed over the 16 lanes of the group.
// Returns the total of row r0 + (the row index this lane ends up with), and that index.
template <typename T, int D>
__device__ __forceinline__ double dots16(const T* __restrict__ rows, int64_t r0, int64_t r_end, int sub,
                                         const double (&fixed)[D / 16], int& which) {
  constexpr int EL = D / 16;
  using GR = GroupReduce<16, 16>;
  double acc[16];
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    acc[r] = 0.0;
    if (r0 + r < r_end) {
      double v[EL];
      load_slice_f64<T, EL>(rows + (size_t)(r0 + r) * D + sub * EL, v);
#pragma unroll
      for (int e = 0; e < EL; ++e) acc[r] = fma(fixed[e], v[e], acc[r]);
    }
  }
  which = GR::head_of(sub);
  return GR::run(acc, sub);
}

// grid (ceil(L/4), Hq); block 256: one wave per query row
template <typename T, int D>
__global__ __launch_bounds__(kCalThreads) void cal_rowstats_kernel(
    const T* __restrict__ Q, const T* __restrict__ K, int64_t L, int G, double scale,
    double* __restrict__ row_max, double* __restrict__ row_sum) {
  constexpr int EL = D / 16;
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6, grp = lane >> 4, sub = lane & 15;
  const int h = blockIdx.y, kvh = h / G;
  const int64_t j = L - 1 - ((int64_t)blockIdx.x * 4 + wv);       // longest rows first
  if (j < 0) return;
  double q[EL];
  load_slice_f64<T, EL>(Q + ((size_t)h * L + j) * D + sub * EL, q);
  const T* Kh = K + (size_t)kvh * L * D;
  double m = -INFINITY, l = 0.0;
  for (int64_t k0 = 0; k0 <= j; k0 += 64) {
    int r;
    const double s = dots16<T, D>(Kh, k0 + grp * 16, j + 1, sub, q, r) * scale;
    if (k0 + grp * 16 + r <= j) {
      const double mn = fmax(m, s);
      l = l * exp(m - mn) + exp(s - mn);
      m = mn;
    }
  }
  merge_lanes(m, l);
  if (lane == 0) {
    row_max[(size_t)h * L + j] = m;
    row_sum[(size_t)h * L + j] = l;
  }
}

// grid (ceil(L/4), Hq); block 256: one wave per key column
template <typename T, int D>
__global__ __launch_bounds__(kCalThreads) void cal_colmeans_kernel(
    const T* __restrict__ Q, const T* __restrict__ K, int64_t L, int G, double scale,
    const double* __restrict__ row_max, const double* __restrict__ row_sum, double* __restrict__ abar) {
  constexpr int EL = D / 16;
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6, grp = lane >> 4, sub = lane & 15;
  const int h = blockIdx.y, kvh = h / G;
  const int64_t k = (int64_t)blockIdx.x * 4 + wv;                 // longest columns first
  if (k >= L) return;
  double kv[EL];
  load_slice_f64<T, EL>(K + ((size_t)kvh * L + k) * D + sub * EL, kv);
  const T* Qh = Q + (size_t)h * L * D;
  double acc = 0.0;
  for (int64_t j0 = k; j0 < L; j0 += 64) {
    int r;
    const double s = dots16<T, D>(Qh, j0 + grp * 16, L, sub, kv, r) * scale;
    const int64_t j = j0 + grp * 16 + r;
    if (j < L) acc += exp(s - row_max[(size_t)h * L + j]) / row_sum[(size_t)h * L + j];
  }
  acc = group_sum(acc, kWave);
  if (lane == 0) abar[(size_t)h * L + k] = acc / (double)(L - k);
}

// grid (M, Hs); block 256.  a[h][i] = sum of abar over tokens with rank < t_block (Eq. 4).
// Selection head h serves query heads h*GS .. h*GS+GS-1; with GS > 1 the importance of a
// key is the mean of their column means.
__global__ __launch_bounds__(kCalThreads) void cal_cand_score_kernel(
    const uint8_t* __restrict__ tokrank, const int32_t* __restrict__ blk_t, const double* __restrict__ abar,
    int64_t L, int b, int64_t nb, int Hs, int GS, int M, double* __restrict__ a_out, int64_t* __restrict__ n_out) {
  __shared__ double red[kCalThreads];
  __shared__ long long redn[kCalThreads];
  const int i = blockIdx.x, h = blockIdx.y, tid = threadIdx.x;
  const int32_t* bt = blk_t + ((size_t)i * Hs + h) * nb;
  const uint8_t* tr = tokrank + (size_t)h * (nb * b);
  double acc = 0.0;
  long long cnt = 0;
  for (int64_t k = tid; k < nb * b; k += kCalThreads) {
    if (tr[k] < bt[k / b]) {
      double v = 0.0;
      for (int g = 0; g < GS; ++g) v += abar[(size_t)(h * GS + g) * L + k];
      acc += GS > 1 ? v / (double)GS : v;
      ++cnt;
    }
  }
  red[tid] = acc;
  redn[tid] = cnt;
  __syncthreads();
  for (int o = kCalThreads / 2; o > 0; o >>= 1) {
    if (tid < o) { red[tid] += red[tid + o]; redn[tid] += redn[tid + o]; }
    __syncthreads();
  }
  if (tid == 0) {
    a_out[(size_t)h * M + i] = red[0];
    n_out[(size_t)h * M + i] = redn[0];
  }
}

__global__ void cal_zero_kernel(int32_t* p, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0;
}

struct CalWs {
  void* select_ws;      // tokrank + stats (+ one blk_t/blk_dst pair, unused here)
  double* row_max;      // [Hq][L]
  double* row_sum;      // [Hq][L]
  double* abar;         // [Hq][L]
  int32_t* blk_t;       // [M][Hs][nb]   (Hs selection heads <= Hq; sized for Hq)
  int32_t* blk_dst;     // [M][Hs][nb]
  int32_t* n_rows;      // [M][Hs]
  double* a_dev;        // [Hs][M]
  int64_t* n_dev;       // [Hs][M]
  void* q_last;         // [Hq][D] contiguous copy of the last query rows
  size_t bytes;
};

static CalWs carve_cal_ws(void* ws, const tca_params* prm, int64_t L, int M) {
  CalWs c;
  char* base = (char*)ws;
  size_t off = 0;
  const int Hq = prm->n_q_heads;
  const int64_t nb = L / prm->block;
  const size_t sel = carve_select_ws(nullptr, prm, L).bytes;
  c.select_ws = base + off;          off = align_up(off + sel, 256);
  c.row_max = (double*)(base + off); off = align_up(off + (size_t)Hq * L * 8, 256);
  c.row_sum = (double*)(base + off); off = align_up(off + (size_t)Hq * L * 8, 256);
  c.abar = (double*)(base + off);    off = align_up(off + (size_t)Hq * L * 8, 256);
  c.blk_t = (int32_t*)(base + off);  off = align_up(off + (size_t)M * Hq * nb * 4, 256);
  c.blk_dst = (int32_t*)(base + off); off = align_up(off + (size_t)M * Hq * nb * 4, 256);
  c.n_rows = (int32_t*)(base + off); off = align_up(off + (size_t)M * Hq * 4, 256);
  c.a_dev = (double*)(base + off);   off = align_up(off + (size_t)Hq * M * 8, 256);
  c.n_dev = (int64_t*)(base + off);  off = align_up(off + (size_t)Hq * M * 8, 256);
  c.q_last = base + off;             off = align_up(off + (size_t)Hq * prm->head_dim * 4, 256);
  c.bytes = off;
  return c;
}

template <typename T>
__global__ void cal_gather_qlast_kernel(const T* __restrict__ Q, int64_t L, int D, T* __restrict__ out) {
  const int h = blockIdx.x;
  for (int e = threadIdx.x; e < D; e += blockDim.x) out[(size_t)h * D + e] = Q[((size_t)h * L + (L - 1)) * D + e];
}

template <typename T, int D>
static void run_passes(const tca_params* prm, const T* Q, const T* K, int64_t L, const CalWs& c, hipStream_t st) {
  const int Hq = prm->n_q_heads, G = Hq / prm->n_kv_heads;
  const dim3 grid((unsigned)((L + 3) / 4), Hq);
  const double sc = logit_scale(prm);
  hipLaunchKernelGGL((cal_rowstats_kernel<T, D>), grid, dim3(kCalThreads), 0, st, Q, K, L, G, sc, c.row_max, c.row_sum);
  hipLaunchKernelGGL((cal_colmeans_kernel<T, D>), grid, dim3(kCalThreads), 0, st, Q, K, L, G, sc, c.row_max, c.row_sum,
                     c.abar);
  hipLaunchKernelGGL((cal_gather_qlast_kernel<T>), dim3(Hq), dim3(128), 0, st, Q, L, D, (T*)c.q_last);
}

}  // namespace tca

using namespace tca;

extern "C" size_t tca_calibrate_workspace_bytes(const tca_params* prm, int64_t L_cal, int M) {
  if (check_params(prm) != TCA_OK || L_cal < 1 || M < 1) return 0;
  return carve_cal_ws(nullptr, prm, L_cal, M).bytes;
}

extern "C" int tca_calibrate_budgets(const tca_params* prm, const void* Qcal, const void* Kcal, int64_t L_cal,
                                     int M, double sigma, double tau, double* p_star, int32_t* cand_idx,
                                     double* a_out, int64_t* n_out, int32_t* fallback, void* ws, size_t ws_bytes,
                                     void* stream) {
  int rc = check_params(prm);
  if (rc) return rc;
  if (!Qcal || !Kcal || !p_star || !cand_idx || !ws)
    return fail(TCA_ERR_INVALID, "tca_calibrate_budgets: NULL pointer argument");
  if (L_cal < 1 || M < 1 || M > 256 || !(sigma > 0.0))
    return fail(TCA_ERR_INVALID, "tca_calibrate_budgets: L_cal=%lld M=%d sigma=%g", (long long)L_cal, M, sigma);
  const int Hs = sel_heads(prm), b = prm->block, nk = block_log2(b) + 1;
  const int64_t nb = L_cal / b;
  if (nb > TCA_MAX_BLOCKS)
    return fail(TCA_ERR_UNSUPPORTED, "tca_calibrate_budgets: %lld blocks exceed the limit of %d", (long long)nb,
                TCA_MAX_BLOCKS);
  const size_t need = tca_calibrate_workspace_bytes(prm, L_cal, M);
  if (ws_bytes < need || ((uintptr_t)ws & 255))
    return fail(TCA_ERR_WORKSPACE, "tca_calibrate_budgets: workspace needs %zu bytes, 256-byte aligned", need);
  hipStream_t st = (hipStream_t)stream;
  CalWs c = carve_cal_ws(ws, prm, L_cal, M);

  std::vector<double> cands((size_t)M * nk);
  rc = tca_make_candidates(b, M, sigma, cands.data());
  if (rc) return rc;

  // column means of the dense causal attention matrix (Alg. 1 line 1, Eq. 4)
  if (prm->dtype == TCA_BF16) {
    using T = bf16_t;
    if (prm->head_dim == 128) run_passes<T, 128>(prm, (const T*)Qcal, (const T*)Kcal, L_cal, c, st);
    else run_passes<T, 64>(prm, (const T*)Qcal, (const T*)Kcal, L_cal, c, st);
  } else {
    using T = float;
    if (prm->head_dim == 128) run_passes<T, 128>(prm, (const T*)Qcal, (const T*)Kcal, L_cal, c, st);
    else run_passes<T, 64>(prm, (const T*)Qcal, (const T*)Kcal, L_cal, c, st);
  }

  // selection of every candidate (Alg. 1 line 4): scores and ranks once, budgets per candidate
  SelectWs sw = carve_select_ws(c.select_ws, prm, L_cal);
  select_score_stage(prm, c.q_last, Kcal, L_cal, L_cal, sw, st);
  std::vector<double> a_host((size_t)Hs * M, 0.0);
  std::vector<int64_t> n_host((size_t)Hs * M, 0);
  if (nb > 0) {
    const int64_t nz = (int64_t)M * Hs;
    hipLaunchKernelGGL(cal_zero_kernel, dim3((unsigned)((nz + 255) / 256)), dim3(256), 0, st, c.n_rows, nz);
    std::vector<double> p_all((size_t)Hs * nk);
    int64_t cap[TCA_MAX_HEADS];
    for (int h = 0; h < Hs; ++h) cap[h] = INT32_MAX;
    for (int i = 0; i < M; ++i) {
      for (int h = 0; h < Hs; ++h)
        for (int e = 0; e < nk; ++e) p_all[(size_t)h * nk + e] = cands[(size_t)i * nk + e];
      select_assign_stage(prm, L_cal, p_all.data(), cap, sw.sel_stats, c.n_rows + (size_t)i * Hs,
                          c.blk_t + (size_t)i * Hs * nb, c.blk_dst + (size_t)i * Hs * nb, st);
    }
    hipLaunchKernelGGL(cal_cand_score_kernel, dim3(M, Hs), dim3(kCalThreads), 0, st, sw.tokrank, c.blk_t, c.abar,
                       L_cal, b, nb, Hs, sel_group(prm), M, c.a_dev, c.n_dev);
    TCA_HIP_CHECK(hipGetLastError());
    TCA_HIP_CHECK(hipMemcpyAsync(a_host.data(), c.a_dev, a_host.size() * 8, hipMemcpyDeviceToHost, st));
    TCA_HIP_CHECK(hipMemcpyAsync(n_host.data(), c.n_dev, n_host.size() * 8, hipMemcpyDeviceToHost, st));
  }
  TCA_HIP_CHECK(hipStreamSynchronize(st));
  TCA_HIP_CHECK(hipGetLastError());

  // Alg. 1 lines 6-8: the valid candidate with the fewest kept tokens (ties: lower index)
  for (int h = 0; h < Hs; ++h) {
    int best = -1;
    for (int i = 0; i < M; ++i) {
      if (a_host[(size_t)h * M + i] >= tau &&
          (best < 0 || n_host[(size_t)h * M + i] < n_host[(size_t)h * M + best]))
        best = i;
    }
    const bool fb = best < 0;
    if (fb) best = M - 1;
    cand_idx[h] = best;
    if (fallback) fallback[h] = fb ? 1 : 0;
    for (int e = 0; e < nk; ++e) p_star[(size_t)h * nk + e] = cands[(size_t)best * nk + e];
    if (a_out) for (int i = 0; i < M; ++i) a_out[(size_t)h * M + i] = a_host[(size_t)h * M + i];
    if (n_out) for (int i = 0; i < M; ++i) n_out[(size_t)h * M + i] = n_host[(size_t)h * M + i];
  }
  return TCA_OK;
}

// Alg. 1 for every layer of a model (Sec. IV-A: the determination is made once per model and
// covers all heads of all layers): one tca_calibrate_budgets pass per layer on that layer's
// sample, on the same workspace, results laid out layer-major.
extern "C" int tca_calibrate_layers(const tca_params* prm, int n_layers, const void* const* Qcal,
                                    const void* const* Kcal, int64_t L_cal, int M, double sigma, double tau,
                                    double* p_star, int32_t* cand_idx, double* a_out, int64_t* n_out,
                                    int32_t* fallback, void* ws, size_t ws_bytes, void* stream) {
  int rc = check_params(prm);
  if (rc) return rc;
  if (n_layers < 1 || !Qcal || !Kcal || !p_star || !cand_idx)
    return fail(TCA_ERR_INVALID, "tca_calibrate_layers: n_layers=%d or NULL pointer argument", n_layers);
  const int Hs = sel_heads(prm), nk = block_log2(prm->block) + 1;
  for (int l = 0; l < n_layers; ++l) {
    if (!Qcal[l] || !Kcal[l]) return fail(TCA_ERR_INVALID, "tca_calibrate_layers: NULL sample of layer %d", l);
    rc = tca_calibrate_budgets(prm, Qcal[l], Kcal[l], L_cal, M, sigma, tau, p_star + (size_t)l * Hs * nk,
                               cand_idx + (size_t)l * Hs, a_out ? a_out + (size_t)l * Hs * M : nullptr,
                               n_out ? n_out + (size_t)l * Hs * M : nullptr,
                               fallback ? fallback + (size_t)l * Hs : nullptr, ws, ws_bytes, stream);
    if (rc) return rc;
  }
  return TCA_OK;
}
