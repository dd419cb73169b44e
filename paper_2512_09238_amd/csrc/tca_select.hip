// Online core-context selection and compaction (Alg. 2 lines 1-6; Eq. 5-8).
//
// Three kernels, K is read from HBM exactly once and logits never leave the chip:
//   score_kernel  : one workgroup per (KV head, block of b tokens).  Streams the
//                   block's K rows with 16-byte loads, forms the logits of all G
//                   query heads of the group in fp64 (Eq. 5 numerator), reduces
//                   them to the block statistics max / sum e^x / sum e^2x that
//                   Eq. 6 needs, and emits one 64-bit ranking key per (head,
//                   token).  The rank of a token inside its block does not depend
//                   on the budget, so Eq. 8 becomes "rank < t_j" later.  For
//                   calibration (ranks reused by every candidate) the kernel also
//                   ranks and writes 1 byte per (head, token); for selection the
//                   ranking is left to gather_kernel, which is bound by HBM and
//                   has the vector ALU to spare.
//   assign_kernel : one workgroup per query head.  Global softmax normaliser,
//                   h_j (Eq. 6), rank of every block, t_j = Psi[rank] (Eq. 7),
//                   exclusive scan of t_j -> destination row of every block.
//   gather_kernel : one workgroup per (head, block).  Ranks the block's tokens by
//                   counting over their keys (skipped when t_j = b), keeps those
//                   with rank < t_j in position order and copies their K/V rows
//                   and positions into the head's flat region (App. C).
// When the query heads of a group share one selection (an extension for GQA), the
// scores of the group's heads have to be normalised before they can be averaged:
// score_kernel then leaves the fp64 logits in the workspace, group_lse_kernel turns
// the per-head block statistics into each head's normaliser, and group_score_kernel
// merges the G logits of a token into one log-domain score and produces the block
// statistics and ranking keys of that score; assign and gather run once per KV head.
#include <hip/hip_runtime.h>

#include "tca_common.h"
#include "tca_device.h"
#include "tca_select.h"

namespace tca {

constexpr int kScoreThreads = 256;
constexpr int kAssignThreads = 1024;
constexpr int kGatherThreads = 256;
constexpr int kGatherRows = 2;        // rows per thread in flight in the copy loop (4 measured the same)
constexpr int kHeadsPerLaunch = 32;
constexpr int kBlockStats = 4;        // doubles per (head, block) in SelectWs::stats

// the group's query heads are merged into one score only when there is more than one of them
static bool grouped(const tca_params* prm) { return sel_group(prm) > 1; }

SelectWs carve_select_ws(void* ws, const tca_params* prm, int64_t n_tokens) {
  const int Hq = prm->n_q_heads, Hs = sel_heads(prm), b = prm->block;
  int64_t nb = n_tokens / b, nbt = (n_tokens + b - 1) / b;
  size_t off = 0;
  SelectWs w;
  char* base = (char*)ws;
  w.tokrank = (uint8_t*)(base + off); off = align_up(off + (size_t)Hs * nb * b, 256);
  w.keys = (uint64_t*)(base + off);   off = align_up(off + (size_t)Hs * nb * b * sizeof(uint64_t), 256);
  w.stats = (double*)(base + off);    off = align_up(off + (size_t)Hq * nbt * kBlockStats * sizeof(double), 256);
  w.sel_stats = w.stats;
  w.xlog = nullptr;
  w.lse = nullptr;
  if (grouped(prm)) {
    w.sel_stats = (double*)(base + off); off = align_up(off + (size_t)Hs * nbt * kBlockStats * sizeof(double), 256);
    w.xlog = (double*)(base + off);      off = align_up(off + (size_t)Hq * nbt * b * sizeof(double), 256);
    w.lse = (double*)(base + off);       off = align_up(off + (size_t)Hq * sizeof(double), 256);
  }
  w.blk_t = (int32_t*)(base + off);   off = align_up(off + (size_t)Hs * nb * sizeof(int32_t), 256);
  w.blk_dst = (int32_t*)(base + off); off = align_up(off + (size_t)Hs * nb * sizeof(int32_t), 256);
  w.bytes = off;
  return w;
}

// ---------------------------------------------------------------- scoring --
// Monotone map of a double to an unsigned 64-bit key (larger value -> larger key).
__device__ __forceinline__ uint64_t ordered_key(double x) {
  const uint64_t u = (uint64_t)__double_as_longlong(x);
  return (u >> 63) ? ~u : (u | 0x8000000000000000ull);
}

// Number of keys of a block that beat key ki (higher logit, or the same logit at a lower
// position): the rank of its token.  keys: b 64-bit keys in LDS, 16-byte aligned.
__device__ __forceinline__ int count_greater(const uint64_t* keys, int o_begin, int o_end, uint64_t ki) {
  int cnt = 0;
  for (int o = o_begin; o < o_end; o += 2) {
    const ulonglong2 ko = *reinterpret_cast<const ulonglong2*>(&keys[o]);
    cnt += (ko.x > ki);
    cnt += (ko.y > ki);
  }
  return cnt;
}

// What score_kernel leaves behind besides the block statistics.
constexpr int kEmitKeys = 0;      // ranking keys (selection)
constexpr int kEmitRanks = 1;     // in-block ranks (calibration: reused by every candidate)
constexpr int kEmitLogits = 2;    // the fp64 logits, tail block included (shared selection: merged by group_score_kernel)

// Key that orders the tokens of a block: the ordered image of the score with its 8
// lowest mantissa bits replaced by 255 - position, so that one unsigned compare
// decides "higher score, or the same score at a lower position".  Scores that agree
// in all but those bits (relative distance below 2^-44) count as tied.
__device__ __forceinline__ uint64_t ranking_key(double x, int i) {
  return (ordered_key(x) & ~0xFFull) | (uint64_t)(255 - i);
}

// grid (nbt, Hkv); block 256.  T storage type, D head dim, G query heads per KV head.
template <typename T, int D, int G, int EMIT>
__global__ __launch_bounds__(kScoreThreads) void score_kernel(
    const T* __restrict__ K, const T* __restrict__ q_last, int64_t kv_stride, int64_t pos0,
    int64_t n_tokens, int b, int64_t n_blocks, int64_t nbt, int Hq, double scale,
    uint8_t* __restrict__ tokrank, uint64_t* __restrict__ keys_out, double* __restrict__ stats,
    double* __restrict__ xlog) {
  constexpr bool RANK = EMIT == kEmitRanks;
  constexpr int EPL = Vec16<T>::N;            // elements per lane per load
  constexpr int LPR = D / EPL;                // lanes per row
  constexpr int RPW = kWave / LPR;            // rows per wave per load
  constexpr int RPI = RPW * (kScoreThreads / kWave);   // rows per workgroup iteration
  constexpr int UNR = 2;                      // 16-byte row loads in flight per lane (more costs occupancy: measured best)
  using GR = GroupReduce<G, LPR>;
  constexpr int GP = GR::GP;
  static_assert(GP <= LPR, "more heads than lanes per row");
  __shared__ double xs[G][256];
  __shared__ __attribute__((aligned(16))) uint64_t keys[G][256];

  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int64_t j = blockIdx.x;
  const int kvh = blockIdx.y;
  const int sub = lane % LPR, rsub = lane / LPR;

  double qv[GP][EPL];
#pragma unroll
  for (int g = 0; g < GP; ++g) {
    float tmp[EPL];
    if (g < G) Vec16<T>::load(q_last + (size_t)(kvh * G + g) * D + sub * EPL, tmp);
#pragma unroll
    for (int e = 0; e < EPL; ++e) qv[g][e] = g < G ? (double)tmp[e] : 0.0;
  }

  const T* Kb = K + ((size_t)kvh * kv_stride + pos0 + j * b) * D;
  const int64_t left = n_tokens - j * b;                  // tokens from the block start to the end
  const int rows_here = left < b ? (int)left : b;
  const int my_head = GR::head_of(sub);
  const bool writer = my_head < G && (sub & (LPR / GP - 1)) == 0;   // one lane per head holds the row's total
  for (int r0 = 0; r0 < b; r0 += RPI * UNR) {
    raw16_t raw[UNR];
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      const int r = r0 + u * RPI + wv * RPW + rsub;
      if (r < rows_here) raw[u] = load_raw16(Kb + (size_t)r * D + sub * EPL);
    }
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      const int r = r0 + u * RPI + wv * RPW + rsub;
      const bool ok = r < rows_here;
      double acc[GP];
#pragma unroll
      for (int g = 0; g < GP; ++g) acc[g] = 0.0;
      if (ok) {
        float kv[EPL];
        widen_raw16<T>(raw[u], kv);
#pragma unroll
        for (int e = 0; e < EPL; ++e) {
          const double kd = (double)kv[e];
#pragma unroll
          for (int g = 0; g < GP; ++g)
            if (g < G) acc[g] = fma(kd, qv[g][e], acc[g]);
        }
      }
      const double v = GR::run(acc, sub);
      if (writer && r < b) xs[my_head][r] = ok ? v * scale : -INFINITY;
    }
  }
  __syncthreads();

  // block statistics: one wave per head
  for (int g = wv; g < G; g += kScoreThreads / kWave) {
    double mx = -INFINITY;
    for (int i = lane; i < b; i += kWave) mx = fmax(mx, xs[g][i]);
    mx = group_max(mx, kWave);
    double e1 = 0.0, e2 = 0.0, e3 = 0.0;
    for (int i = lane; i < b; i += kWave) {
      const double dx = xs[g][i] - mx;
      const double e = exp(dx);
      e1 += e;
      e2 += e * e;
      if (e > 0.0) e3 += e * dx;                         // 0 * (-inf) counts as 0
    }
    e1 = group_sum(e1, kWave);
    e2 = group_sum(e2, kWave);
    e3 = group_sum(e3, kWave);
    if (lane == 0) {
      double* st = stats + ((size_t)(kvh * G + g) * nbt + j) * kBlockStats;
      st[0] = mx; st[1] = e1; st[2] = e2; st[3] = e3;
    }
  }
  if constexpr (EMIT == kEmitLogits) {
    for (int pi = tid; pi < G * b; pi += kScoreThreads) {
      const int g = pi / b, i = pi - g * b;
      xlog[((size_t)(kvh * G + g) * nbt + j) * b + i] = xs[g][i];          // -inf past the end of the tail
    }
    return;
  }
  if (j >= n_blocks) return;             // the tail block only feeds the normaliser

  // Rank inside the block = number of tokens that beat token i (higher logit, or
  // the same logit at a lower position): one unsigned compare of ranking keys per pair.
  for (int pi = tid; pi < G * b; pi += kScoreThreads) {
    const int g = pi / b, i = pi - g * b;
    const uint64_t key = ranking_key(xs[g][i], i);
    if constexpr (RANK) keys[g][i] = key;
    else keys_out[(size_t)(kvh * G + g) * (n_blocks * b) + j * b + i] = key;
  }
  if constexpr (RANK) {
    __syncthreads();
    for (int pi = tid; pi < G * b; pi += kScoreThreads) {
      const int g = pi / b, i = pi - g * b;
      tokrank[(size_t)(kvh * G + g) * (n_blocks * b) + j * b + i] = (uint8_t)count_greater(keys[g], 0, b, keys[g][i]);
    }
  }
}

// ----------------------------------------------------------- group score --
// Shared selection: the score of a token is the mean over the group's query heads of their
// Eq. 5 scores, sbar_i = (1/G) sum_g exp(x_gi - lse_g).  It is carried in the log domain,
// y_i = ln sum_g exp(x_gi - lse_g) = ln(G sbar_i), so that the block statistics, ranking keys,
// Eq. 6 and Eq. 7 of the per-head path apply to y unchanged (the factor G cancels in the
// normalised block mass and in both concentration indices).

// grid (Hq); block 256.  lse[h] = ln sum_i e^{x_hi} from the block statistics (tail included).
__global__ __launch_bounds__(256) void group_lse_kernel(const double* __restrict__ stats, int nbt,
                                                        double* __restrict__ lse) {
  __shared__ double red[4];
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const double* st = stats + (size_t)blockIdx.x * nbt * kBlockStats;
  double mx = -INFINITY;
  for (int j = tid; j < nbt; j += 256) mx = fmax(mx, st[(size_t)j * kBlockStats]);
  mx = group_max(mx, kWave);
  if (lane == 0) red[wv] = mx;
  __syncthreads();
  mx = fmax(fmax(red[0], red[1]), fmax(red[2], red[3]));
  __syncthreads();
  double z = 0.0;
  for (int j = tid; j < nbt; j += 256) z += st[(size_t)j * kBlockStats + 1] * exp(st[(size_t)j * kBlockStats] - mx);
  z = group_sum(z, kWave);
  if (lane == 0) red[wv] = z;
  __syncthreads();
  if (tid == 0) lse[blockIdx.x] = mx + log((red[0] + red[1]) + (red[2] + red[3]));
}

// grid (nbt, Hkv); block 256: thread i owns token i of the block.
template <int G, bool RANK>
__global__ __launch_bounds__(256) void group_score_kernel(
    const double* __restrict__ xlog, const double* __restrict__ lse, int b, int64_t n_blocks, int64_t nbt,
    uint8_t* __restrict__ tokrank, uint64_t* __restrict__ keys_out, double* __restrict__ gstats) {
  __shared__ double red[4][3];
  __shared__ __attribute__((aligned(16))) uint64_t keys[256];
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int64_t j = blockIdx.x;
  const int kvh = blockIdx.y;
  double y = -INFINITY;
  if (tid < b) {
    double a[G], top = -INFINITY;
#pragma unroll
    for (int g = 0; g < G; ++g) {
      a[g] = xlog[((size_t)(kvh * G + g) * nbt + j) * b + tid] - lse[kvh * G + g];
      top = fmax(top, a[g]);
    }
    if (top > -INFINITY) {                                 // a token past the end of the tail stays at -inf
      double sum = 0.0;
#pragma unroll
      for (int g = 0; g < G; ++g) sum += exp(a[g] - top);
      y = top + log(sum);
    }
  }
  double mx = group_max(y, kWave);
  if (lane == 0) red[wv][0] = mx;
  __syncthreads();
  mx = fmax(fmax(red[0][0], red[1][0]), fmax(red[2][0], red[3][0]));
  __syncthreads();
  const double dx = y - mx;
  const double e = y > -INFINITY ? exp(dx) : 0.0;
  const double e1 = group_sum(e, kWave), e2 = group_sum(e * e, kWave);
  const double e3 = group_sum(e > 0.0 ? e * dx : 0.0, kWave);
  if (lane == 0) { red[wv][0] = e1; red[wv][1] = e2; red[wv][2] = e3; }
  __syncthreads();
  if (tid == 0) {
    double* st = gstats + ((size_t)kvh * nbt + j) * kBlockStats;
    st[0] = mx;
    st[1] = (red[0][0] + red[1][0]) + (red[2][0] + red[3][0]);
    st[2] = (red[0][1] + red[1][1]) + (red[2][1] + red[3][1]);
    st[3] = (red[0][2] + red[1][2]) + (red[2][2] + red[3][2]);
  }
  if (j >= n_blocks) return;
  const uint64_t key = ranking_key(y, tid);
  if constexpr (RANK) {
    if (tid < b) keys[tid] = key;
    __syncthreads();
    if (tid < b) tokrank[(size_t)kvh * (n_blocks * b) + j * b + tid] = (uint8_t)count_greater(keys, 0, b, key);
  } else {
    if (tid < b) keys_out[(size_t)kvh * (n_blocks * b) + j * b + tid] = key;
  }
}

// ----------------------------------------------------------------- assign --
struct AssignArgs {
  int32_t cum[kHeadsPerLaunch][TCA_MAX_COUNTS];   // cumulative Psi counts: rank < cum[e] -> budget 2^e
  int64_t cap[kHeadsPerLaunch];                   // capacity of the head's region
};

__device__ __forceinline__ double block_reduce_max(double v, double* red) {
  v = group_max(v, kWave);
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  __syncthreads();
  if (lane == 0) red[wv] = v;
  __syncthreads();
  double r = red[0];
  for (int i = 1; i < kAssignThreads / kWave; ++i) r = fmax(r, red[i]);
  return r;
}
__device__ __forceinline__ double block_reduce_sum(double v, double* red) {
  v = group_sum(v, kWave);
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  __syncthreads();
  if (lane == 0) red[wv] = v;
  __syncthreads();
  double r = 0.0;
  for (int i = 0; i < kAssignThreads / kWave; ++i) r += red[i];
  return r;
}

// grid (heads in this launch); block 1024.
__global__ __launch_bounds__(kAssignThreads) void assign_kernel(
    AssignArgs args, int head0, int nk, int m, int nbt, int b, double alpha, int metric,
    const double* __restrict__ stats, int32_t* __restrict__ n_rows,
    int32_t* __restrict__ blk_t, int32_t* __restrict__ blk_dst) {
  __shared__ double hs[TCA_MAX_BLOCKS];
  __shared__ uint16_t ts[TCA_MAX_BLOCKS];
  __shared__ uint16_t js[TCA_MAX_BLOCKS];
  __shared__ double red[kAssignThreads / kWave];
  __shared__ int32_t scan[kAssignThreads];
  const int tid = threadIdx.x;
  const int hl = blockIdx.x, h = head0 + hl;
  const double* st = stats + (size_t)h * nbt * kBlockStats;

  // the statistics of this thread's blocks (block j = tid + k * 1024, tail block included), read once
  constexpr int KMAX = TCA_MAX_BLOCKS / kAssignThreads + 1;
  double bM[KMAX], bE1[KMAX], bE2[KMAX];              // bE2: the statistic the chosen index needs
#pragma unroll
  for (int k = 0; k < KMAX; ++k) {
    const int j = tid + k * kAssignThreads;
    const bool in = j < nbt;
    bM[k] = in ? st[j * kBlockStats] : -INFINITY;
    bE1[k] = in ? st[j * kBlockStats + 1] : 0.0;
    bE2[k] = in ? st[j * kBlockStats + (metric == TCA_METRIC_ENTROPY ? 3 : 2)] : 0.0;
  }
  // global normaliser of Eq. 5 over every scored token, tail included
  double mx = -INFINITY;
#pragma unroll
  for (int k = 0; k < KMAX; ++k) mx = fmax(mx, bM[k]);
  mx = block_reduce_max(mx, red);
  double z = 0.0;
#pragma unroll
  for (int k = 0; k < KMAX; ++k) {
    bM[k] = tid + k * kAssignThreads < nbt ? bE1[k] * exp(bM[k] - mx) : 0.0;   // block mass before normalisation
    z += bM[k];
  }
  z = block_reduce_sum(z, red);

  // Eq. 6
#pragma unroll
  for (int k = 0; k < KMAX; ++k) {
    const int j = tid + k * kAssignThreads;
    if (j < m) {
      const double mass = bM[k] / z;
      // HHI of the block (Eq. 6), or the entropy of the scores renormalised inside it:
      // t_i = e_i / E1  =>  -sum t_i ln t_i = ln E1 - (sum e_i (x_i - M)) / E1
      const double spread = metric == TCA_METRIC_ENTROPY
                                ? (log(bE1[k]) - bE2[k] / bE1[k]) / log((double)b)
                                : 1.0 - bE2[k] / (bE1[k] * bE1[k]);
      hs[j] = (1.0 - alpha) * mass + alpha * spread;
    }
  }
  __syncthreads();

  // order the blocks by ascending h (ties: lower block first) with a bitonic sort
  // of (h, block) pairs in LDS, then Eq. 7: the block at sorted position r gets Psi[r]
  int P = 1;
  while (P < m) P <<= 1;
  for (int e = tid; e < P; e += kAssignThreads) {
    js[e] = (uint16_t)e;
    if (e >= m) hs[e] = INFINITY;                      // padding sorts last
  }
  __syncthreads();
  for (int k = 2; k <= P; k <<= 1) {
    for (int jj = k >> 1; jj > 0; jj >>= 1) {
      for (int e = tid; e < P; e += kAssignThreads) {
        const int pr = e ^ jj;
        if (pr > e) {
          const double ha = hs[e], hb = hs[pr];
          const uint16_t ja = js[e], jb = js[pr];
          const bool a_after_b = (ha > hb) || (ha == hb && ja > jb);
          const bool ascending = (e & k) == 0;
          if (a_after_b == ascending) {
            hs[e] = hb; hs[pr] = ha;
            js[e] = jb; js[pr] = ja;
          }
        }
      }
      // Element e is always handled by the wave that owns its aligned group of 64,
      // so a stage with partner distance < 64 touches only the wave's own
      // elements.  A workgroup barrier is needed only when this stage or the next
      // one pairs elements of different waves; otherwise the wave's own LDS
      // accesses are already ordered.
      const int next_jj = jj > 1 ? (jj >> 1) : k;        // distance of the following stage
      if (jj >= kWave || next_jj >= kWave) __syncthreads();
      else __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    }
  }
  __syncthreads();
  for (int r = tid; r < m; r += kAssignThreads) {
    int e = 0;
    while (e < nk - 1 && r >= args.cum[hl][e]) ++e;
    ts[js[r]] = (uint16_t)(1 << e);
  }
  __syncthreads();

  // exclusive scan of t_j in block order: thread t owns a run of `per` blocks
  const int per = (m + kAssignThreads - 1) / kAssignThreads;
  const int j0 = tid * per;
  int local = 0;
  for (int j = j0; j < j0 + per && j < m; ++j) local += ts[j];
  scan[tid] = local;
  __syncthreads();
  for (int o = 1; o < kAssignThreads; o <<= 1) {
    int v = tid >= o ? scan[tid - o] : 0;
    __syncthreads();
    scan[tid] += v;
    __syncthreads();
  }
  const int32_t fill = n_rows[h];
  int run = fill + scan[tid] - local;
  for (int j = j0; j < j0 + per && j < m; ++j) {
    blk_t[(size_t)h * m + j] = ts[j];
    blk_dst[(size_t)h * m + j] = run;
    run += ts[j];
  }
  __syncthreads();
  if (tid == kAssignThreads - 1) {
    int64_t total = (int64_t)fill + scan[tid];
    if (total > args.cap[hl]) total = args.cap[hl];
    n_rows[h] = (int32_t)total;
  }
}

// ----------------------------------------------------------------- gather --
// offsets of the heads' regions travel in the kernel's argument block: no copy, no extra launch
struct OffsArgs { int64_t offs[TCA_MAX_HEADS + 1]; };

// grid (n_blocks * selection heads); block 256.  G: selection heads per KV head.
// Workgroup ids go round-robin over the 8 XCDs.  The G selection heads of a KV head keep
// overlapping subsets of the same block's rows, so their workgroups are given ids 8 apart:
// same XCD, consecutive in time, and the rows a later one needs are mostly in that L2 already.
template <typename T, int D>
__global__ __launch_bounds__(kGatherThreads) void gather_kernel(
    const T* __restrict__ K, const T* __restrict__ V, int64_t kv_stride, int64_t pos0, int b,
    int64_t n_blocks, int G, const uint64_t* __restrict__ keys,
    const int32_t* __restrict__ blk_t, const int32_t* __restrict__ blk_dst,
    OffsArgs oa, int32_t* __restrict__ idx, T* __restrict__ Kg, T* __restrict__ Vg) {
  constexpr int EPL = Vec16<T>::N;
  constexpr int LPR = D / EPL;
  constexpr int RPI = kGatherThreads / LPR;
  __shared__ int32_t sel[256];
  __shared__ int32_t wave_cnt[kGatherThreads / kWave];
  __shared__ __attribute__((aligned(16))) uint64_t bkeys[256];
  __shared__ int32_t rank[256];
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  int64_t j;
  int h, kvh;
  {
    const int64_t id = blockIdx.x, pairs = (int64_t)gridDim.x / G;       // pairs = n_blocks * KV heads
    if ((pairs & 7) == 0) {
      const int64_t u = id >> 3;                                         // position in the XCD's own sequence
      const int64_t pair = (u / G) * 8 + (id & 7);
      kvh = (int)(pair / n_blocks);
      j = pair - (int64_t)kvh * n_blocks;
      h = kvh * G + (int)(u % G);
    } else {
      h = (int)(id / n_blocks);
      j = id - (int64_t)h * n_blocks;
      kvh = h / G;
    }
  }
  const int t = blk_t[(size_t)h * n_blocks + j];
  const int64_t base = oa.offs[h], cap = oa.offs[h + 1] - base;
  const int64_t dst0 = blk_dst[(size_t)h * n_blocks + j];

  // Eq. 8: rank of every token inside the block, all 256 threads share the b*b comparisons;
  // nothing to rank when the whole block is kept
  bool keep = tid < b;
  if (t < b) {
    if (tid < b) {
      bkeys[tid] = keys[(size_t)h * (n_blocks * b) + j * b + tid];
      rank[tid] = 0;
    }
    __syncthreads();
    // b is a power of two <= 256: thread (i = tid % b, part = tid / b) counts over one even-sized span
    int parts = kGatherThreads / b;
    if (parts > b / 2) parts = b / 2;
    const int i = tid % b, part = tid / b, span = b / parts;
    if (part < parts) {
      const int cnt = count_greater(bkeys, part * span, (part + 1) * span, bkeys[i]);
      if (cnt) atomicAdd(&rank[i], cnt);
    }
    __syncthreads();
    keep = tid < b && rank[tid] < t;
  }
  // compact the kept positions, in ascending position order
  const unsigned long long mask = __ballot(keep);
  if (lane == 0) wave_cnt[wv] = __popcll(mask);
  __syncthreads();
  int before = __popcll(mask & ((1ull << lane) - 1ull));
  for (int w = 0; w < wv; ++w) before += wave_cnt[w];
  if (keep) sel[before] = tid;
  __syncthreads();

  // copy the kept rows, kRows rows per thread in flight (2 * kRows 16-byte loads before the first store)
  constexpr int kRows = kGatherRows;
  const int sub = tid % LPR;
  int n_keep = t;
  if (dst0 + n_keep > cap) n_keep = cap > dst0 ? (int)(cap - dst0) : 0;
  if (!Kg) {                                           // positions only: no compacted copy is kept
    for (int k = tid; k < n_keep; k += kGatherThreads) idx[base + dst0 + k] = (int32_t)(pos0 + j * b + sel[k]);
    return;
  }
  for (int k0 = tid / LPR; k0 < n_keep; k0 += kRows * RPI) {
    uint4 kr[kRows], vr[kRows];
    int64_t pos[kRows];
#pragma unroll
    for (int u = 0; u < kRows; ++u) {
      const int k = k0 + u * RPI;
      pos[u] = pos0 + j * b + sel[k < n_keep ? k : k0];
      const size_t src = ((size_t)kvh * kv_stride + pos[u]) * D + sub * EPL;
      kr[u] = *reinterpret_cast<const uint4*>(K + src);
      vr[u] = *reinterpret_cast<const uint4*>(V + src);
    }
#pragma unroll
    for (int u = 0; u < kRows; ++u) {
      const int k = k0 + u * RPI;
      if (k < n_keep) {
        const size_t dst = (size_t)(base + dst0 + k) * D + sub * EPL;
        *reinterpret_cast<uint4*>(Kg + dst) = kr[u];
        *reinterpret_cast<uint4*>(Vg + dst) = vr[u];
        if (sub == 0) idx[base + dst0 + k] = (int32_t)pos[u];
      }
    }
  }
}

template <typename T, int D, int EMIT>
static void launch_score(int G, dim3 grid, hipStream_t st, const T* K, const T* q, int64_t kv_stride,
                         int64_t pos0, int64_t n_tokens, int b, int64_t nb, int64_t nbt, int Hq,
                         double scale, const SelectWs& w) {
#define TCA_SCORE_CASE(GG)                                                                           \
  case GG:                                                                                           \
    hipLaunchKernelGGL((score_kernel<T, D, GG, EMIT>), grid, dim3(kScoreThreads), 0, st, K, q,       \
                       kv_stride, pos0, n_tokens, b, nb, nbt, Hq, scale, w.tokrank, w.keys, w.stats, \
                       w.xlog);                                                                      \
    break;
  switch (G) {
    TCA_SCORE_CASE(1) TCA_SCORE_CASE(2) TCA_SCORE_CASE(3) TCA_SCORE_CASE(4)
    TCA_SCORE_CASE(5) TCA_SCORE_CASE(6) TCA_SCORE_CASE(7) TCA_SCORE_CASE(8)
  }
#undef TCA_SCORE_CASE
}

template <bool RANK>
static void launch_group_score(int G, int Hq, int Hkv, int b, int64_t nb, int64_t nbt, const SelectWs& w,
                               hipStream_t st) {
  hipLaunchKernelGGL(group_lse_kernel, dim3(Hq), dim3(256), 0, st, w.stats, (int)nbt, w.lse);
  const dim3 grid((unsigned)nbt, Hkv);
#define TCA_GROUP_CASE(GG)                                                                              \
  case GG:                                                                                              \
    hipLaunchKernelGGL((group_score_kernel<GG, RANK>), grid, dim3(256), 0, st, w.xlog, w.lse, b, nb, nbt, \
                       w.tokrank, w.keys, w.sel_stats);                                                 \
    break;
  switch (G) {
    TCA_GROUP_CASE(2) TCA_GROUP_CASE(3) TCA_GROUP_CASE(4) TCA_GROUP_CASE(5)
    TCA_GROUP_CASE(6) TCA_GROUP_CASE(7) TCA_GROUP_CASE(8)
  }
#undef TCA_GROUP_CASE
}

// Scores tokens [pos0, pos0 + n_tokens) for every selection head: block statistics in
// w.sel_stats, and in-block ranks in w.tokrank (RANK) or ranking keys in w.keys.
template <typename T, int D, bool RANK>
static void score_stage(const tca_params* prm, const T* q_last, const T* K, int64_t kv_stride, int64_t pos0,
                        int64_t n_tokens, const SelectWs& w, hipStream_t st) {
  const int Hq = prm->n_q_heads, Hkv = prm->n_kv_heads, G = Hq / Hkv, b = prm->block;
  const int64_t nb = n_tokens / b, nbt = (n_tokens + b - 1) / b;
  const dim3 grid((unsigned)nbt, Hkv);
  const double sc = logit_scale(prm);
  if (grouped(prm)) {
    launch_score<T, D, kEmitLogits>(G, grid, st, K, q_last, kv_stride, pos0, n_tokens, b, nb, nbt, Hq, sc, w);
    launch_group_score<RANK>(G, Hq, Hkv, b, nb, nbt, w, st);
  } else {
    launch_score<T, D, RANK ? kEmitRanks : kEmitKeys>(G, grid, st, K, q_last, kv_stride, pos0, n_tokens, b, nb,
                                                      nbt, Hq, sc, w);
  }
}

// Stage 1 of selection for callers outside this file (calibration): block statistics
// and in-block ranks of tokens [0, n_tokens) of K scored by q_last.
void select_score_stage(const tca_params* prm, const void* q_last, const void* K, int64_t kv_stride,
                        int64_t n_tokens, const SelectWs& w, hipStream_t st) {
  if (prm->dtype == TCA_BF16) {
    using T = bf16_t;
    if (prm->head_dim == 128) score_stage<T, 128, true>(prm, (const T*)q_last, (const T*)K, kv_stride, 0, n_tokens, w, st);
    else score_stage<T, 64, true>(prm, (const T*)q_last, (const T*)K, kv_stride, 0, n_tokens, w, st);
  } else {
    using T = float;
    if (prm->head_dim == 128) score_stage<T, 128, true>(prm, (const T*)q_last, (const T*)K, kv_stride, 0, n_tokens, w, st);
    else score_stage<T, 64, true>(prm, (const T*)q_last, (const T*)K, kv_stride, 0, n_tokens, w, st);
  }
}

// Stage 2: block metric, ranking and budgets for one configuration per selection head.
// blk_t / blk_dst: [Hs][nb]; n_rows: [Hs] fill counters (in/out); cap: per-head capacity.
void select_assign_stage(const tca_params* prm, int64_t n_tokens, const double* p, const int64_t* cap,
                         const double* stats, int32_t* n_rows, int32_t* blk_t, int32_t* blk_dst,
                         hipStream_t st) {
  const int Hs = sel_heads(prm), b = prm->block, nk = block_log2(b) + 1;
  const int64_t nb = n_tokens / b, nbt = (n_tokens + b - 1) / b;
  for (int h0 = 0; h0 < Hs; h0 += kHeadsPerLaunch) {
    const int nh = Hs - h0 < kHeadsPerLaunch ? Hs - h0 : kHeadsPerLaunch;
    AssignArgs aa;
    for (int hl = 0; hl < nh; ++hl) {
      int64_t c[TCA_MAX_COUNTS];
      psi_counts(nk, nb, p + (size_t)(h0 + hl) * nk, c);
      int64_t run = 0;
      for (int e = 0; e < nk; ++e) { run += c[e]; aa.cum[hl][e] = (int32_t)run; }
      aa.cap[hl] = cap[h0 + hl];
    }
    hipLaunchKernelGGL(assign_kernel, dim3(nh), dim3(kAssignThreads), 0, st, aa, h0, nk, (int)nb,
                       (int)nbt, b, prm->alpha, prm->metric, stats, n_rows, blk_t, blk_dst);
  }
}

template <typename T, int D>
static int run_select(const tca_params* prm, const T* q_last, const T* K, const T* V,
                      int64_t kv_stride, int64_t pos0, int64_t n_tokens, const double* p,
                      const int64_t* offs, int32_t* n_rows, int32_t* idx, T* Kg, T* Vg, void* ws,
                      hipStream_t st) {
  const int Hs = sel_heads(prm), Hkv = prm->n_kv_heads, b = prm->block;
  const int64_t nb = n_tokens / b;
  SelectWs w = carve_select_ws(ws, prm, n_tokens);
  OffsArgs oa;
  for (int h = 0; h <= Hs; ++h) oa.offs[h] = offs[h];

  score_stage<T, D, false>(prm, q_last, K, kv_stride, pos0, n_tokens, w, st);
  if (nb == 0) return TCA_OK;

  int64_t cap[TCA_MAX_HEADS];
  for (int h = 0; h < Hs; ++h) cap[h] = offs[h + 1] - offs[h];
  select_assign_stage(prm, n_tokens, p, cap, w.sel_stats, n_rows, w.blk_t, w.blk_dst, st);
  hipLaunchKernelGGL((gather_kernel<T, D>), dim3((unsigned)(nb * Hs)), dim3(kGatherThreads), 0, st, K, V,
                     kv_stride, pos0, b, nb, Hs / Hkv, w.keys, w.blk_t, w.blk_dst, oa, idx, Kg, Vg);
  return TCA_OK;
}

}  // namespace tca

using namespace tca;

extern "C" size_t tca_select_workspace_bytes(const tca_params* prm, int64_t n_tokens) {
  if (check_params(prm) != TCA_OK || n_tokens < 0) return 0;
  SelectWs w = carve_select_ws(nullptr, prm, n_tokens);
  return w.bytes;
}

extern "C" int tca_select(const tca_params* prm, const void* q_last, const void* K, const void* V,
                          int64_t kv_stride, int64_t pos0, int64_t n_tokens, const double* p,
                          const int64_t* offs, int32_t* n_rows, int32_t* idx, void* Kg, void* Vg,
                          void* ws, size_t ws_bytes, void* stream) {
  int rc = check_params(prm);
  if (rc) return rc;
  if (!q_last || !K || !V || !p || !offs || !n_rows || !idx || !ws)
    return fail(TCA_ERR_INVALID, "tca_select: NULL pointer argument");
  if ((Kg == nullptr) != (Vg == nullptr))
    return fail(TCA_ERR_INVALID, "tca_select: Kg and Vg must both be given, or both be NULL (positions only)");
  const int b = prm->block, Hs = sel_heads(prm);
  if (n_tokens < 0 || pos0 < 0 || pos0 % b != 0 || pos0 + n_tokens > kv_stride)
    return fail(TCA_ERR_INVALID, "tca_select: pos0=%lld n_tokens=%lld kv_stride=%lld (pos0 must be a "
                "multiple of b and the range must fit)", (long long)pos0, (long long)n_tokens,
                (long long)kv_stride);
  if (pos0 + n_tokens > INT32_MAX) return fail(TCA_ERR_UNSUPPORTED, "positions beyond int32");
  if (n_tokens / b > TCA_MAX_BLOCKS)
    return fail(TCA_ERR_UNSUPPORTED, "tca_select: %lld blocks exceed the limit of %d per call",
                (long long)(n_tokens / b), TCA_MAX_BLOCKS);
  const int nk = block_log2(b) + 1;
  for (int h = 0; h < Hs; ++h) {
    if (!valid_config(p + (size_t)h * nk, nk))
      return fail(TCA_ERR_INVALID, "tca_select: p[%d] is not a distribution", h);
    if (offs[h + 1] < offs[h]) return fail(TCA_ERR_INVALID, "tca_select: offs not ascending at %d", h);
  }
  if (offs[0] != 0) return fail(TCA_ERR_INVALID, "tca_select: offs[0] must be 0");
  if (ws_bytes < tca_select_workspace_bytes(prm, n_tokens) || ((uintptr_t)ws & 255))
    return fail(TCA_ERR_WORKSPACE, "tca_select: workspace needs %zu bytes, 256-byte aligned",
                tca_select_workspace_bytes(prm, n_tokens));
  if (n_tokens == 0) return TCA_OK;
  hipStream_t st = (hipStream_t)stream;
  const int D = prm->head_dim;
  if (prm->dtype == TCA_BF16) {
    using T = bf16_t;
    rc = D == 128 ? run_select<T, 128>(prm, (const T*)q_last, (const T*)K, (const T*)V, kv_stride, pos0,
                                       n_tokens, p, offs, n_rows, idx, (T*)Kg, (T*)Vg, ws, st)
                  : run_select<T, 64>(prm, (const T*)q_last, (const T*)K, (const T*)V, kv_stride, pos0,
                                      n_tokens, p, offs, n_rows, idx, (T*)Kg, (T*)Vg, ws, st);
  } else {
    using T = float;
    rc = D == 128 ? run_select<T, 128>(prm, (const T*)q_last, (const T*)K, (const T*)V, kv_stride, pos0,
                                       n_tokens, p, offs, n_rows, idx, (T*)Kg, (T*)Vg, ws, st)
                  : run_select<T, 64>(prm, (const T*)q_last, (const T*)K, (const T*)V, kv_stride, pos0,
                                      n_tokens, p, offs, n_rows, idx, (T*)Kg, (T*)Vg, ws, st);
  }
  if (rc) return rc;
  TCA_HIP_CHECK(hipGetLastError());
  return TCA_OK;
}
