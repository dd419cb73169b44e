// Single-token decode over the compacted KV cache, and selection of blocks
// completed while decoding (Sec. IV-B, "Online Token Selection in Decoding Stage").
//
// One step = four launches on the caller's stream:
//   prep    : write the new K/V row into the ring; per head, count the global
//             rows that have left the window (idx <= T-w; idx is ascending so
//             this is a prefix, found by a 64-way search of one wave).
//   partial : split-K attention.  grid (slot, selection head, sequence); a slot is
//             a chunk of kChunk rows of the head's global region or of the ring.
//             The 256 threads form sixteen 16-lane groups, each streaming whole
//             rows with 16-byte loads and keeping its own online softmax; groups
//             are merged into one (max, sum, acc[D]) partial per slot and query
//             head.  HBM-bound: every K/V row is read once per selection head -
//             once per query head, or, when the group shares one selection, once
//             per KV head with every row scored against the group's G queries.
//   merge   : log-sum-exp merge of a head's partials -> O.  If the new token
//             completes a block, the same workgroup scores the block's b rows
//             with this step's query in fp64 (Eq. 5 restricted to the block),
//             ranks them and appends the top t = floor(sum k p_k) to the head's
//             global region in position order.  Shared selection: the group's
//             first workgroup ranks by the sum over the group's heads of their
//             block-normalised scores and appends once per KV head.
//   advance : length += 1.
#include <hip/hip_runtime.h>

#include <atomic>
#include <type_traits>

#include "tca_common.h"
#include "tca_device.h"

namespace tca {

constexpr int kPartThreads = 256;                 // threads of a split-K workgroup (64 with 256-row slots measured 8-14 % slower)
constexpr int kPartWaves = kPartThreads / 64;
constexpr int kChunk = 4 * kPartThreads;          // rows per split-K slot: 64 per 16-lane group
constexpr int kChunkShared = 2048;                // the same when every row is scored against a group of queries (1024: 507, 2048: 480, 4096: 540 us per step)
constexpr int kDecThreads = 256;                  // the other kernels
constexpr int kMaxSlots = 4096;       // split-K slots per head the merge kernel can weigh (4M rows per head)

struct DecodeHeads {
  int64_t offs[TCA_MAX_HEADS + 1];
  int32_t t_dec[TCA_MAX_HEADS];
};

struct DecodeWs {
  int32_t* n_vis;    // [B][Hs]
  float* part;       // [B][Hq][n_slots][D+2]
  size_t bytes;
};

static DecodeWs carve_decode_ws(void* ws, int B, int Hq, int D, int n_slots) {
  DecodeWs w;
  char* base = (char*)ws;
  size_t off = 0;
  w.n_vis = (int32_t*)(base + off); off = align_up(off + (size_t)B * Hq * sizeof(int32_t), 256);   // sized for Hs = Hq
  w.part = (float*)(base + off);    off = align_up(off + (size_t)B * Hq * n_slots * (D + 2) * sizeof(float), 256);
  w.bytes = off;
  return w;
}

static int chunk_rows(const tca_params* prm) { return sel_group(prm) > 1 ? kChunkShared : kChunk; }
static int window_slots(const tca_params* prm) { return (prm->window + chunk_rows(prm) - 1) / chunk_rows(prm); }
static int global_slots(const tca_params* prm, int64_t max_head_rows) {
  return (int)((max_head_rows + chunk_rows(prm) - 1) / chunk_rows(prm));
}

// Number of entries <= bound among the ascending idx[0..n), found by a whole wave: every
// round probes the last element of up to 64 equal chunks of the open range, so 2^18 rows take
// three dependent loads instead of eighteen.  Result in every lane.
__device__ __forceinline__ int count_le_wave(const int32_t* __restrict__ idx, int n, int64_t bound) {
  const int lane = threadIdx.x & 63;
  int lo = 0, hi = n;                       // the count lies in [lo, hi]
  while (hi - lo > 64) {
    const int len = hi - lo;
    const int step = (len + 63) / 64;
    const bool has = lane * step < len;     // lane's chunk: [lo + lane*step, lo + min((lane+1)*step, len))
    const int last = lo + min((lane + 1) * step, len) - 1;
    const bool le = has && (int64_t)idx[last] <= bound;
    const int c = __popcll(__ballot(le));   // chunks that lie entirely at or below the bound (a prefix of them)
    const int nch = (len + step - 1) / step;
    if (c == nch) { lo = hi; break; }
    const int lo2 = lo + c * step;
    hi = lo + min((c + 1) * step, len) - 1; // the last element of chunk c is above the bound
    lo = lo2;
  }
  if (hi > lo) {
    const bool le = lane < hi - lo && (int64_t)idx[lo + lane] <= bound;
    lo += __popcll(__ballot(le));
  }
  return lo;
}

// max over the 16 lanes of a row, result in every lane
__device__ __forceinline__ float row16_max(float v) {
  v = fmaxf(v, dpp_f32<kDppXor1>(v));
  v = fmaxf(v, dpp_f32<kDppXor2>(v));
  v = fmaxf(v, dpp_f32<kDppHalfMirror>(v));
  v = fmaxf(v, dpp_f32<kDppMirror>(v));
  return v;
}

// Scale of an FP8 row from the largest magnitude of its elements, and its reciprocal use: the codes are
// RNE_e4m3(x / scale) with both divisions in float32 (the rule stated with TCA_KV_FP8).
__device__ __forceinline__ float fp8_row_scale(float amax) { return amax > 0.f ? amax / 448.f : 1.f; }

// One 16-lane group stores one row of D elements (a lane's slice: D/16 consecutive elements, 4 or 8)
// into a cache row of storage type KV: a plain conversion-free copy for the native types, codes and a
// scale for FP8.  x: the lane's slice widened to float.  Called by all 16 lanes of the group.
template <typename KV, int EL>
__device__ __forceinline__ void store_cache_slice(const float (&x)[EL], KV* dst_row, float* scale_slot, int sub) {
  static_assert(sizeof(KV) == 1, "native rows are copied as stored");
  float amax = 0.f;
#pragma unroll
  for (int e = 0; e < EL; ++e) amax = fmaxf(amax, fabsf(x[e]));
  amax = row16_max(amax);
  const float scale = fp8_row_scale(amax);
  uint32_t* out = reinterpret_cast<uint32_t*>(dst_row + sub * EL);
#pragma unroll
  for (int e = 0; e < EL; e += 4) out[e / 4] = f32x4_to_fp8(x[e] / scale, x[e + 1] / scale, x[e + 2] / scale, x[e + 3] / scale);
  if (sub == 0) *scale_slot = scale;
}

// grid (B, ceil(Hs/4)); block 256: one wave per selection head; the workgroups with blockIdx.y = 0
// also write the new row into the ring (KV = T: as it is; KV = fp8_t: as codes and a scale)
template <typename T, typename KV, int D>
__global__ __launch_bounds__(256) void decode_prep_kernel(tca_cache c, DecodeHeads dh, int Hs, int Hkv, int w,
                                                          const T* __restrict__ k_new, const T* __restrict__ v_new,
                                                          int32_t* __restrict__ n_vis) {
  const int s = blockIdx.x;
  const int64_t Tpos = c.length[s];
  if (blockIdx.y == 0) {
    const int slot = (int)(Tpos % w);
    KV* rk = (KV*)c.ringK;
    KV* rv = (KV*)c.ringV;
    if constexpr (std::is_same<T, KV>::value) {
      for (int e = threadIdx.x; e < Hkv * D; e += blockDim.x) {
        const int kvh = e / D, dd = e - kvh * D;
        const size_t dst = (((size_t)s * Hkv + kvh) * w + slot) * D + dd;
        rk[dst] = k_new[(size_t)s * Hkv * D + e];
        rv[dst] = v_new[(size_t)s * Hkv * D + e];
      }
    } else {
      constexpr int EL = D / 16;
      const int grp = threadIdx.x >> 4, sub = threadIdx.x & 15;       // one 16-lane group per (KV head, K or V)
      for (int job = grp; job < 2 * Hkv; job += 16) {
        const int kvh = job >> 1;
        const T* src = ((job & 1) ? v_new : k_new) + ((size_t)s * Hkv + kvh) * D + sub * EL;
        float x[EL];
        load_slice<T, EL>(src, x);
        const size_t row = ((size_t)s * Hkv + kvh) * w + slot;
        store_cache_slice<KV, EL>(x, ((job & 1) ? rv : rk) + row * D, ((job & 1) ? c.ringV_scale : c.ringK_scale) + row, sub);
      }
    }
  }
  const int h = blockIdx.y * 4 + (threadIdx.x >> 6);
  if (h >= Hs) return;
  const int32_t* ix = c.idx + (size_t)s * c.cap_rows + dh.offs[h];
  const int nv = count_le_wave(ix, c.n_rows[s * Hs + h], Tpos - w);
  if ((threadIdx.x & 63) == 0) n_vis[s * Hs + h] = nv;
}

// Tail of the split-K kernels: every 16-lane group of the workgroup holds, for each of NQ
// queries, an online-softmax state (reference m in base-2 units, sum l, acc over the lane's
// slice of d).  Merges the 4 groups of each wave, then the 4 waves through LDS, and writes one
// (reference, sum, acc[D]) partial per query at out + g * out_head, the reference still in
// base-2 units (integer references, as the fp32 path keeps them, stay exact through every merge).
template <int D, int NQ>
__device__ __forceinline__ void merge_partials(float (&m)[NQ], float (&l)[NQ], float (&acc)[NQ][D / 16],
                                               float* __restrict__ out, size_t out_head, float* red) {
  constexpr int EL = D / 16;
  constexpr int PW = EL + 2;                          // floats of one lane's share of a partial
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
#pragma unroll
  for (int g = 0; g < NQ; ++g) {
    for (int o = 16; o < 64; o <<= 1) {
      const float mo = __shfl_xor(m[g], o, kWave), lo = __shfl_xor(l[g], o, kWave);
      const float mn = fmaxf(m[g], mo);
      const float ca = (m[g] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(m[g] - mn);
      const float cb = (mo == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(mo - mn);
      l[g] = l[g] * ca + lo * cb;
#pragma unroll
      for (int e = 0; e < EL; ++e) acc[g][e] = acc[g][e] * ca + __shfl_xor(acc[g][e], o, kWave) * cb;
      m[g] = mn;
    }
    if (lane < 16) {
      red[(wv * 16 + lane) * (NQ * PW) + g * PW] = m[g];
      red[(wv * 16 + lane) * (NQ * PW) + g * PW + 1] = l[g];
#pragma unroll
      for (int e = 0; e < EL; ++e) red[(wv * 16 + lane) * (NQ * PW) + g * PW + 2 + e] = acc[g][e];
    }
  }
  __syncthreads();
  for (int pi = tid; pi < 16 * NQ; pi += kPartThreads) {
    const int g = pi >> 4, ln = pi & 15;
    float M = -INFINITY;
    for (int x = 0; x < kPartWaves; ++x) M = fmaxf(M, red[(x * 16 + ln) * (NQ * PW) + g * PW]);
    float L = 0.f, a[EL];
#pragma unroll
    for (int e = 0; e < EL; ++e) a[e] = 0.f;
    for (int x = 0; x < kPartWaves; ++x) {
      const float mx = red[(x * 16 + ln) * (NQ * PW) + g * PW];
      const float cf = (mx == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(mx - M);
      L += red[(x * 16 + ln) * (NQ * PW) + g * PW + 1] * cf;
#pragma unroll
      for (int e = 0; e < EL; ++e) a[e] += red[(x * 16 + ln) * (NQ * PW) + g * PW + 2 + e] * cf;
    }
    float* og = out + g * out_head;
    if (ln == 0) { og[0] = M; og[1] = L; }
#pragma unroll
    for (int e = 0; e < EL; ++e) og[2 + ln * EL + e] = a[e];
  }
}

// Split-K attention of NQ queries (consecutive heads, q0 = the first one's row) over rows
// [r_begin, r_end) of one K/V buffer: every row is read once and scored against all NQ queries.
// Writes one (max, sum, acc[D]) partial per query at out + g * out_head.  red: LDS scratch of
// kPartWaves * 16 * NQ * (D/16 + 2) floats.  Called by a whole workgroup.
// T: type of the queries; KV: storage type of the rows (T itself, or fp8_t with one float scale per
// row in kscale / vscale, indexed like the rows).
template <typename T, typename KV, int D, int NQ>
__device__ __forceinline__ void partial_rows(const KV* __restrict__ kbase, const KV* __restrict__ vbase,
                                             const float* __restrict__ kscale, const float* __restrict__ vscale,
                                             int r_begin, int r_end, const T* __restrict__ q0, double scale,
                                             float* __restrict__ out, size_t out_head, float* red) {
  constexpr int EL = D / 16;
  const int tid = threadIdx.x;
  const int grp = tid >> 4, sub = tid & 15;           // groups of 16 lanes
  if (r_begin >= r_end) {
    if (tid < NQ) { out[tid * out_head] = -INFINITY; out[tid * out_head + 1] = 0.f; }
    return;
  }

  // logits are carried in base-2 units (scale * log2 e) so that the exponential is one v_exp_f32.
  // bf16 storage: q.k over a lane's slice is EL/2 two-element bf16 dot products with fp32
  // accumulation straight from the loaded words, and the factor is applied to the row's sum.
  // fp32 storage: q.k is accumulated in fp64 and the reference of the exponentials is kept at an
  // integer (exact in fp32, and exact through every later merge), so that x - reference is formed
  // without cancellation error even for logits in the hundreds.
  // FP8 storage: the codes are widened to float, q.k is the fp32 dot product with the codes times the
  // row's scale, and p.v takes the V row's scale into the weight.
  constexpr double kLog2e = 1.4426950408889634;
  constexpr bool kDot2 = sizeof(KV) == 2;
  constexpr bool kFp8 = sizeof(KV) == 1;
  typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
  using logit_t = typename std::conditional<sizeof(KV) == 4, double, float>::type;
  const logit_t qk_factor = (logit_t)(scale * kLog2e);
  float qv[kDot2 ? 1 : NQ][EL];
  RawSlice<T, EL> qraw[kDot2 ? NQ : 1];
#pragma unroll
  for (int g = 0; g < NQ; ++g) {
    if constexpr (kDot2) qraw[g].load(q0 + (size_t)g * D + sub * EL);
    else load_slice<T, EL>(q0 + (size_t)g * D + sub * EL, qv[g]);
  }

  float m[NQ], l[NQ], acc[NQ][EL];
#pragma unroll
  for (int g = 0; g < NQ; ++g) {
    m[g] = -INFINITY;
    l[g] = 0.f;
#pragma unroll
    for (int e = 0; e < EL; ++e) acc[g][e] = 0.f;
  }

  // Online softmax with a lazy reference: m[g] is raised (and l, acc rescaled) only when a
  // logit exceeds it by more than kSlack, so the common row costs one subtract, one exp and
  // the multiply-adds.  Terms are then at most 2^kSlack; the result is exact because l and
  // acc share the reference, which the merge steps below carry along.
  constexpr float kSlack = 8.f;
  // Rows are fetched one iteration ahead of their use (kUnr rows of K and of V per group,
  // kept as loaded until then), so that a lane has 2*kUnr loads in flight while it computes.
  constexpr int kUnr = 2;                              // (4 for the FP8 rows, half the bytes each, measured no faster)
  using Raw = RawSlice<KV, EL>;
  Raw kr[kUnr], vr[kUnr];
  float ksc[kUnr], vsc[kUnr];                          // row scales (FP8 rows only)
  bool ok[kUnr];
  auto fetch = [&](int r0, Raw (&kk)[kUnr], Raw (&vq)[kUnr], float (&ks)[kUnr], float (&vs)[kUnr], bool (&okk)[kUnr]) {
#pragma unroll
    for (int u = 0; u < kUnr; ++u) {
      const int r = r0 + u * (kPartThreads / 16) + grp;
      okk[u] = r < r_end;
      ks[u] = vs[u] = 1.f;
      if (okk[u]) {
        kk[u].load(kbase + (size_t)r * D + sub * EL);
        vq[u].load(vbase + (size_t)r * D + sub * EL);
        if constexpr (kFp8) { ks[u] = kscale[r]; vs[u] = vscale[r]; }
      }
    }
  };
  fetch(r_begin, kr, vr, ksc, vsc, ok);
  for (int r0 = r_begin; r0 < r_end; r0 += (kPartThreads / 16) * kUnr) {
    Raw kn[kUnr], vn[kUnr];
    float ksn[kUnr], vsn[kUnr];
    bool okn[kUnr];
    fetch(r0 + (kPartThreads / 16) * kUnr, kn, vn, ksn, vsn, okn);          // nothing is loaded past r_end
#pragma unroll
    for (int u = 0; u < kUnr; ++u) {
      float kv[EL], vv[EL];
      if (ok[u]) {
        if constexpr (!kDot2) kr[u].widen(kv);
        vr[u].widen(vv);
      }
#pragma unroll
      for (int g = 0; g < NQ; ++g) {
        logit_t sc = 0;
        if (ok[u]) {
          if constexpr (kDot2) {
#pragma unroll
            for (int i = 0; i < EL / 2; ++i)
              sc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, kr[u].w[i]),
                                                   __builtin_bit_cast(bf16x2_t, qraw[g].w[i]), sc, false);
          } else {
#pragma unroll
            for (int e = 0; e < EL; ++e) {
              if constexpr (sizeof(logit_t) == 4) sc = fmaf(qv[g][e], kv[e], sc);
              else sc = fma((double)qv[g][e], (double)kv[e], sc);
            }
          }
        }
        sc = row16_sum(sc) * qk_factor;
        if constexpr (kFp8) sc *= ksc[u];
        if (ok[u]) {
          if (sc > (logit_t)m[g] + (logit_t)kSlack) {
            const float m_new = sizeof(KV) == 4 ? ceilf((float)sc) : (float)sc;
            const float corr = __builtin_amdgcn_exp2f(m[g] - m_new);    // 0 on the first row (m = -inf)
            l[g] *= corr;
#pragma unroll
            for (int e = 0; e < EL; ++e) acc[g][e] *= corr;
            m[g] = m_new;
          }
          const float pr = __builtin_amdgcn_exp2f((float)(sc - (logit_t)m[g]));
          l[g] += pr;
          const float pw = kFp8 ? pr * vsc[u] : pr;                   // the V row's scale rides on the weight
#pragma unroll
          for (int e = 0; e < EL; ++e) acc[g][e] = fmaf(pw, vv[e], acc[g][e]);
        }
      }
    }
#pragma unroll
    for (int u = 0; u < kUnr; ++u) { kr[u] = kn[u]; vr[u] = vn[u]; ksc[u] = ksn[u]; vsc[u] = vsn[u]; ok[u] = okn[u]; }
  }
  merge_partials<D, NQ>(m, l, acc, out, out_head, red);
}

// The same for bf16 rows of 128 elements and NQ > 1 queries, with q.k on the matrix cores.
// A wave takes 16 rows per iteration (its 16-lane group kb the rows 4kb .. 4kb+3).  K rows go
// from registers into a wave-private LDS tile and come back in MFMA operand order (lane
// (n, kb) = 8 consecutive elements of row n), so that four 16x16x32 MFMAs against the queries
// (operand B, columns >= NQ zero) leave S[row 4kb+i][query n] in lane (n, kb): the NQ*4 lanes
// with n < NQ hold every score once, and only they do the softmax arithmetic.  Their terms p
// return through LDS to the lanes that hold the V rows, which accumulate p.v on the vector ALU
// as before.  The reference m[g] is common to the wave and lazy (raised only when a score
// exceeds it by more than kSlack, decided by a wave-wide vote).  Against partial_rows this
// removes, per (row, query), the dot products, the 16-lane reductions and 15 of the 16 copies
// of the exponential.  tiles: LDS, kMfmaTileBytes per wave, then 256 bytes per query.
constexpr int kMfmaTileBytes = 16 * 256 + 16 * 8 * 4;
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 dec_bf16x8_t;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float dec_f32x4_t;

template <int NQ>
__device__ __forceinline__ void partial_rows_mfma(const bf16_t* __restrict__ kbase, const bf16_t* __restrict__ vbase,
                                                  int r_begin, int r_end, const bf16_t* __restrict__ q0, double scale,
                                                  float* __restrict__ out, size_t out_head, float* red,
                                                  unsigned char* tiles) {
  constexpr int D = 128, EL = 8;
  constexpr float kLog2e = 1.4426950408889634f;
  constexpr float kSlack = 8.f;
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int kb = lane >> 4, n = lane & 15;            // group inside the wave; lane inside the group
  if (r_begin >= r_end) {
    if (tid < NQ) { out[tid * out_head] = -INFINITY; out[tid * out_head + 1] = 0.f; }
    return;
  }
  unsigned char* kt = tiles + wv * kMfmaTileBytes;    // [16 rows][16 chunks of 16 B], chunk index xor row
  float* pt = reinterpret_cast<float*>(kt + 16 * 256); // [16 rows][8 queries]: scores, then terms p
  const bool holder = n < NQ;                         // this lane owns the scores of query n

  // The queries sit in LDS (chunk index xor query, like the K tile) and are read as operand B
  // of MFMA j (elements (4j + kb) * 8 .. + 7 of query n) every iteration: 4 registers instead of 16.
  unsigned char* qt = tiles + kPartWaves * kMfmaTileBytes;       // [NQ][16 chunks of 16 B]
  for (int ci = tid; ci < NQ * 16; ci += kPartThreads) {
    const int g = ci >> 4, ch = ci & 15;
    *reinterpret_cast<uint4*>(qt + g * 256 + ((ch ^ g) & 15) * 16) = *reinterpret_cast<const uint4*>(q0 + (size_t)g * D + ch * 8);
  }
  __syncthreads();
  const float factor = (float)(scale * (double)kLog2e);

  float m[NQ], l[NQ], acc[NQ][EL];
#pragma unroll
  for (int g = 0; g < NQ; ++g) {
    m[g] = -INFINITY;
    l[g] = 0.f;
#pragma unroll
    for (int e = 0; e < EL; ++e) acc[g][e] = 0.f;
  }
  float m_mine = -INFINITY, l_mine = 0.f;             // holder lanes: reference and sum of query n over rows 4kb .. 4kb+3

  // K rows are requested one iteration ahead (they are needed first, for the tile); V rows at the
  // end of the iteration before, so that they travel while the next scores are formed.
  using Raw = RawSlice<bf16_t, EL>;
  Raw kn[4], vn[4];
  bool okk[4], okv[4];
  auto fetch_k = [&](int r0) {
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int r = r0 + 16 * wv + 4 * kb + u;
      okk[u] = r < r_end;                              // nothing is loaded past r_end
      if (okk[u]) kn[u].load(kbase + (size_t)r * D + n * EL);
    }
  };
  auto fetch_v = [&](int r0) {
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int r = r0 + 16 * wv + 4 * kb + u;
      okv[u] = r < r_end;
      if (okv[u]) vn[u].load(vbase + (size_t)r * D + n * EL);
    }
  };
  fetch_k(r_begin);
  fetch_v(r_begin);
  for (int r0 = r_begin; r0 < r_end; r0 += 16 * kPartWaves) {
    // this iteration's K rows into the tile, the next ones requested
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int row = 4 * kb + u;
      if (okk[u])
        *reinterpret_cast<uint4*>(kt + row * 256 + ((n ^ row) & 15) * 16) = make_uint4(kn[u].w[0], kn[u].w[1], kn[u].w[2], kn[u].w[3]);
    }
    fetch_k(r0 + 16 * kPartWaves);
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");

    // S[row 4kb+i][query n] = sum over d; operand A of MFMA j: chunk 4j + kb of row n
    dec_f32x4_t sv = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const uint4 a = *reinterpret_cast<const uint4*>(kt + n * 256 + (((4 * j + kb) ^ n) & 15) * 16);
      uint4 bq = make_uint4(0, 0, 0, 0);               // columns >= NQ of operand B are zero
      if (holder) bq = *reinterpret_cast<const uint4*>(qt + n * 256 + (((4 * j + kb) ^ n) & 15) * 16);
      sv = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(dec_bf16x8_t, a),
                                                   __builtin_bit_cast(dec_bf16x8_t, bq), sv, 0, 0, 0);
    }
    float s2[4];
    bool raise = false;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const bool valid = r0 + 16 * wv + 4 * kb + i < r_end;      // rows past the end hold stale tile data
      s2[i] = valid ? sv[i] * factor : -INFINITY;
      raise |= holder && s2[i] > m_mine + kSlack;
    }
    if (__any(raise)) {
      // raise the references: every lane learns the largest score of each query over the 16 rows
      if (holder) {
#pragma unroll
        for (int i = 0; i < 4; ++i) pt[(4 * kb + i) * 8 + n] = s2[i];
      }
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
      float mxs[8];
#pragma unroll
      for (int g = 0; g < 8; ++g) mxs[g] = -INFINITY;
#pragma unroll 2
      for (int x = 0; x < 16; ++x) {
        float t[8];
        *reinterpret_cast<float4*>(&t[0]) = *reinterpret_cast<const float4*>(pt + x * 8);
        if constexpr (NQ > 4) *reinterpret_cast<float4*>(&t[4]) = *reinterpret_cast<const float4*>(pt + x * 8 + 4);
#pragma unroll
        for (int g = 0; g < NQ; ++g) mxs[g] = fmaxf(mxs[g], t[g]);
      }
#pragma unroll
      for (int g = 0; g < NQ; ++g) {
        const float mx = mxs[g];
        const float m_new = fmaxf(m[g], mx);
        const float corr = m_new == -INFINITY ? 1.f : __builtin_amdgcn_exp2f(m[g] - m_new);   // 0 while m[g] = -inf
#pragma unroll
        for (int e = 0; e < EL; ++e) acc[g][e] *= corr;
        if (n == g) { l_mine *= corr; m_mine = m_new; }
        m[g] = m_new;
      }
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    }
    float p[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      p[i] = (holder && s2[i] > -INFINITY) ? __builtin_amdgcn_exp2f(s2[i] - m_mine) : 0.f;
      l_mine += p[i];
    }
    if (holder) {
#pragma unroll
      for (int i = 0; i < 4; ++i) pt[(4 * kb + i) * 8 + n] = p[i];
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");

#pragma unroll
    for (int u = 0; u < 4; ++u) {
      if (okv[u]) {
        float pr[8];                                   // terms of row 4kb+u for every query
        *reinterpret_cast<float4*>(&pr[0]) = *reinterpret_cast<const float4*>(pt + (4 * kb + u) * 8);
        if constexpr (NQ > 4) *reinterpret_cast<float4*>(&pr[4]) = *reinterpret_cast<const float4*>(pt + (4 * kb + u) * 8 + 4);
        float vv[EL];
        vn[u].widen(vv);
#pragma unroll
        for (int g = 0; g < NQ; ++g) {
#pragma unroll
          for (int e = 0; e < EL; ++e) acc[g][e] = fmaf(pr[g], vv[e], acc[g][e]);
        }
      }
    }
    fetch_v(r0 + 16 * kPartWaves);
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");   // the tile and pt are rewritten by the next iteration
  }
  // the sum of query g over this group's rows sits in lane g of the group
#pragma unroll
  for (int g = 0; g < NQ; ++g) l[g] = __shfl(l_mine, (lane & 48) + g, kWave);
  merge_partials<D, NQ>(m, l, acc, out, out_head, red);
}

// grid (n_slots, Hs, B); block kPartThreads.  Selection head hs = blockIdx.y serves the GQ query
// heads hs*GQ .. hs*GQ+GQ-1 (GQ = 1: one selection per query head).  Slots below g_slots are
// chunks of the head's global region, the others chunks of the ring.  The ring belongs to the KV
// head, so with GW > GQ (one selection per query head, GW = G heads per KV head) the workgroup
// of the group's first head scores each ring row against all GW queries and the others skip it.
template <typename T, typename KV, int D, int GQ, int GW>
__global__ __launch_bounds__(kPartThreads) void decode_partial_kernel(
    tca_cache c, DecodeHeads dh, int Hq, int Hkv, int w, int g_slots, int n_slots, double scale,
    const T* __restrict__ q, const int32_t* __restrict__ n_vis, float* __restrict__ part) {
  constexpr int EL = D / 16;
  constexpr int CH = GQ > 1 ? kChunkShared : kChunk;  // rows per slot
  constexpr int NMAX = GQ > GW ? GQ : GW;
  __shared__ float red[kPartWaves * 16 * NMAX * (EL + 2)];
  constexpr bool kMfma = sizeof(KV) == 2 && D == 128;  // rows that partial_rows_mfma takes
  __shared__ __attribute__((aligned(16))) unsigned char tiles[kMfma && NMAX > 1 ? kPartWaves * kMfmaTileBytes + NMAX * 256 : 16];
  const int slot = blockIdx.x, hs = blockIdx.y, s = blockIdx.z;
  const int Hs = Hq / GQ, h0 = hs * GQ, kvh = h0 / (Hq / Hkv);
  float* out = part + (((size_t)s * Hq + h0) * n_slots + slot) * (D + 2);   // head h0 + g: + g * n_slots * (D+2)
  const size_t out_head = (size_t)n_slots * (D + 2);
  const int64_t Tpos = c.length[s];
  const T* q0 = q + ((size_t)s * Hq + h0) * D;

  if (slot < g_slots) {
    const int nv = n_vis[s * Hs + hs];
    const int r_begin = slot * CH;
    const int r_end = min(nv, r_begin + CH);
    const size_t base = (size_t)s * c.cap_rows + dh.offs[hs];
    if constexpr (kMfma && GQ > 1)
      partial_rows_mfma<GQ>((const T*)c.Kg + base * D, (const T*)c.Vg + base * D, r_begin, r_end, q0, scale, out,
                            out_head, red, tiles);
    else
      partial_rows<T, KV, D, GQ>((const KV*)c.Kg + base * D, (const KV*)c.Vg + base * D, c.Kg_scale + base,
                                 c.Vg_scale + base, r_begin, r_end, q0, scale, out, out_head, red);
  } else {
    if (GW != GQ && h0 % GW != 0) return;              // this head's ring partial is written by the group's first head
    // Slot r of the ring holds the latest position congruent to r mod w that is <= Tpos.  Once
    // Tpos >= w every slot is filled; before that only slots 0 .. Tpos are.
    const int filled = Tpos >= w ? w : (int)Tpos + 1;
    const int r_begin = (slot - g_slots) * CH;
    const int r_end = min(filled, r_begin + CH);
    const size_t base = ((size_t)s * Hkv + kvh) * w;
    if constexpr (kMfma && GW > 1)
      partial_rows_mfma<GW>((const T*)c.ringK + base * D, (const T*)c.ringV + base * D, r_begin, r_end, q0, scale,
                            out, out_head, red, tiles);
    else
      partial_rows<T, KV, D, GW>((const KV*)c.ringK + base * D, (const KV*)c.ringV + base * D, c.ringK_scale + base,
                                 c.ringV_scale + base, r_begin, r_end, q0, scale, out, out_head, red);
  }
}

// grid (Hq, B); block 256
template <typename T, typename KV, int D>
__global__ __launch_bounds__(kDecThreads) void decode_merge_kernel(
    tca_cache c, DecodeHeads dh, int Hq, int Hkv, int GS, int w, int b, int n_slots, double scale,
    const T* __restrict__ q, const float* __restrict__ part, T* __restrict__ O) {
  constexpr int EL = D / 16;
  __shared__ double xs[256];
  __shared__ double gred[kDecThreads / kWave];
  __shared__ int32_t sel[256];
  __shared__ int32_t wave_cnt[kDecThreads / kWave];
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int h = blockIdx.x, s = blockIdx.y;
  const int G = Hq / Hkv, kvh = h / G;
  const float* pp = part + ((size_t)s * Hq + h) * n_slots * (D + 2);

  // log-sum-exp merge of the head's partials: slot weights first (one thread per
  // slot), then every thread sums four output columns over a share of the slots
  __shared__ float wgt[kMaxSlots];
  __shared__ float colsum[kDecThreads / (D / 4)][D];
  __shared__ float lsum[kDecThreads / kWave];
  {
    float M = -INFINITY;
    for (int x = tid; x < n_slots; x += kDecThreads)
      if (pp[(size_t)x * (D + 2) + 1] > 0.f) M = fmaxf(M, pp[(size_t)x * (D + 2)]);
    M = group_max(M, kWave);
    if (lane == 0) lsum[wv] = M;
    __syncthreads();
    M = fmaxf(fmaxf(lsum[0], lsum[1]), fmaxf(lsum[2], lsum[3]));
    __syncthreads();
    float lpart = 0.f;
    for (int x = tid; x < n_slots; x += kDecThreads) {
      const float lx = pp[(size_t)x * (D + 2) + 1];
      const float wx = lx > 0.f ? __builtin_amdgcn_exp2f(pp[(size_t)x * (D + 2)] - M) : 0.f;   // references are in base-2 units
      wgt[x] = wx;
      lpart += lx * wx;
    }
    lpart = group_sum(lpart, kWave);
    if (lane == 0) lsum[wv] = lpart;
    __syncthreads();
    const float L = (lsum[0] + lsum[1]) + (lsum[2] + lsum[3]);
    constexpr int CQ = D / 4;                            // column quads of a partial
    constexpr int SPLIT = kDecThreads / CQ;              // threads per column quad
    const int cq = tid % CQ, part = tid / CQ;
    float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
#pragma unroll 4
    for (int x = part; x < n_slots; x += SPLIT) {
      const float wx = wgt[x];                           // an empty slot's columns were never written
      if (wx != 0.f) {
        const float* src = pp + (size_t)x * (D + 2) + 2 + 4 * cq;      // 8-byte aligned
        const float2 lo = *reinterpret_cast<const float2*>(src), hi = *reinterpret_cast<const float2*>(src + 2);
        a0 += lo.x * wx; a1 += lo.y * wx; a2 += hi.x * wx; a3 += hi.y * wx;
      }
    }
    colsum[part][4 * cq] = a0; colsum[part][4 * cq + 1] = a1;
    colsum[part][4 * cq + 2] = a2; colsum[part][4 * cq + 3] = a3;
    __syncthreads();
    if (tid < D) {
      float t = 0.f;
#pragma unroll
      for (int q2 = 0; q2 < SPLIT; ++q2) t += colsum[q2][tid];
      store_f32(O + ((size_t)s * Hq + h) * D + tid, t / L);
    }
  }

  // block completed by this token?
  const int64_t Tpos = c.length[s];
  if ((Tpos + 1) % b != 0) return;
  if (h % GS != 0) return;                             // one workgroup per selection head ranks the block
  const int hs = h / GS, Hs = Hq / GS;
  const int64_t p0 = Tpos + 1 - b;                     // first position of the block
  const int slot0 = (int)(p0 % w);                     // contiguous in the ring: w is a multiple of b
  const size_t ring_row0 = ((size_t)s * Hkv + kvh) * w + slot0;
  const KV* kb = (const KV*)c.ringK + ring_row0 * D;
  const KV* vb = (const KV*)c.ringV + ring_row0 * D;
  const int grp = tid >> 4, sub = tid & 15;
  // score of row i: the logit of the head's query, or, for a shared selection, the sum over the
  // group's heads of exp(logit - log-sum-exp over the block) (G times the mean score)
  double score = 0.0;
  for (int g = 0; g < GS; ++g) {
    float qf[EL];
    load_slice<T, EL>(q + ((size_t)s * Hq + h + g) * D + sub * EL, qf);
    __syncthreads();                                   // xs of the previous head has been consumed
    for (int r0 = 0; r0 < b; r0 += 16) {
      const int r = r0 + grp;
      double a = 0.0;
      if (r < b) {
        float kf[EL];
        RawSlice<KV, EL> raw;
        raw.load(kb + (size_t)r * D + sub * EL);
        raw.widen(kf);
#pragma unroll
        for (int e = 0; e < EL; ++e) a = fma((double)kf[e], (double)qf[e], a);
        if constexpr (sizeof(KV) == 1) a *= (double)c.ringK_scale[ring_row0 + r];   // the row read back: code * scale
      }
      a = group_sum(a, 16);
      if (r < b && sub == 0) xs[r] = a * scale;
    }
    __syncthreads();
    if (GS == 1) {
      if (tid < b) score = xs[tid];
    } else {
      const double xi = tid < b ? xs[tid] : -INFINITY;
      double mx = group_max(xi, kWave);
      if (lane == 0) gred[wv] = mx;
      __syncthreads();
      mx = fmax(fmax(gred[0], gred[1]), fmax(gred[2], gred[3]));
      __syncthreads();
      const double e = tid < b ? exp(xi - mx) : 0.0;
      const double zs = group_sum(e, kWave);
      if (lane == 0) gred[wv] = zs;
      __syncthreads();
      score += e / ((gred[0] + gred[1]) + (gred[2] + gred[3]));
    }
  }
  __syncthreads();
  if (tid < b) xs[tid] = score;
  __syncthreads();
  const int t = dh.t_dec[hs];
  bool keep = false;
  if (tid < b) {
    const double xi = xs[tid];
    int cnt = 0;
    for (int o = 0; o < b; ++o) {
      const double xo = xs[o];
      cnt += (xo > xi) || (xo == xi && o < tid);
    }
    keep = cnt < t;
  }
  const unsigned long long mask = __ballot(keep);
  if (lane == 0) wave_cnt[wv] = __popcll(mask);
  __syncthreads();
  int before = __popcll(mask & ((1ull << lane) - 1ull));
  for (int x = 0; x < wv; ++x) before += wave_cnt[x];
  if (keep) sel[before] = tid;
  __syncthreads();
  const int64_t cap = dh.offs[hs + 1] - dh.offs[hs];
  const int32_t fill = c.n_rows[s * Hs + hs];
  const size_t base = (size_t)s * c.cap_rows + dh.offs[hs];
  KV* Kg = (KV*)c.Kg;
  KV* Vg = (KV*)c.Vg;
  for (int k = grp; k < t; k += 16) {
    const int64_t row = (int64_t)fill + k;
    if (row >= cap) break;
    const int src = sel[k];
    for (int e = 0; e < EL; ++e) {                     // rows are copied as stored
      Kg[(base + row) * D + sub * EL + e] = kb[(size_t)src * D + sub * EL + e];
      Vg[(base + row) * D + sub * EL + e] = vb[(size_t)src * D + sub * EL + e];
    }
    if (sub == 0) {
      c.idx[base + row] = (int32_t)(p0 + src);
      if constexpr (sizeof(KV) == 1) {
        c.Kg_scale[base + row] = c.ringK_scale[ring_row0 + src];
        c.Vg_scale[base + row] = c.ringV_scale[ring_row0 + src];
      }
    }
  }
  __syncthreads();
  if (tid == 0) {
    int64_t nf = (int64_t)fill + t;
    c.n_rows[s * Hs + hs] = (int32_t)(nf > cap ? cap : nf);
  }
}

__global__ void decode_advance_kernel(int64_t* length, int B) {
  const int s = blockIdx.x * blockDim.x + threadIdx.x;
  if (s < B) length[s] += 1;
}

// grid (ceil(rows/16), Hkv); block 256: one 16-lane group per row
template <typename T, typename KV, int D>
__global__ __launch_bounds__(256) void load_window_kernel(tca_cache c, int seq, int Hkv, int w, const T* __restrict__ K,
                                                          const T* __restrict__ V, int64_t kv_stride, int64_t L) {
  constexpr int EL = D / 16;
  const int kvh = blockIdx.y, sub = threadIdx.x & 15;
  const int64_t first = L - w > 0 ? L - w : 0;
  const int64_t pos = first + (int64_t)blockIdx.x * 16 + (threadIdx.x >> 4);
  if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) c.length[seq] = L;
  if (pos >= L) return;
  const int slot = (int)(pos % w);
  const T* ks = K + ((size_t)kvh * kv_stride + pos) * D;
  const T* vs = V + ((size_t)kvh * kv_stride + pos) * D;
  const size_t row = ((size_t)seq * Hkv + kvh) * w + slot;
  KV* kd = (KV*)c.ringK + row * D;
  KV* vd = (KV*)c.ringV + row * D;
  if constexpr (std::is_same<T, KV>::value) {
    for (int e = sub; e < D; e += 16) { kd[e] = ks[e]; vd[e] = vs[e]; }
  } else {
    float x[EL];
    load_slice<T, EL>(ks + sub * EL, x);
    store_cache_slice<KV, EL>(x, kd, c.ringK_scale + row, sub);
    load_slice<T, EL>(vs + sub * EL, x);
    store_cache_slice<KV, EL>(x, vd, c.ringV_scale + row, sub);
  }
}

// grid (ceil(cap_rows/16)); block 256: one 16-lane group per row of the flat global buffer
template <typename T, typename KV, int D>
__global__ __launch_bounds__(256) void load_global_kernel(tca_cache c, int seq, DecodeHeads dh, int Hs,
                                                          const int32_t* __restrict__ idx, const T* __restrict__ Kg,
                                                          const T* __restrict__ Vg, const int32_t* __restrict__ n_rows) {
  constexpr int EL = D / 16;
  const int sub = threadIdx.x & 15;
  const int64_t r = (int64_t)blockIdx.x * 16 + (threadIdx.x >> 4);
  if (blockIdx.x == 0 && threadIdx.x < Hs) c.n_rows[(size_t)seq * Hs + threadIdx.x] = n_rows[threadIdx.x];
  if (r >= c.cap_rows) return;
  int h = 0;
  while (h + 1 < Hs && dh.offs[h + 1] <= r) ++h;                 // the head whose region holds row r
  if (r - dh.offs[h] >= n_rows[h]) return;                      // capacity beyond the filled rows
  const size_t dst = (size_t)seq * c.cap_rows + r;
  if (sub == 0) c.idx[dst] = idx[r];
  KV* kd = (KV*)c.Kg + dst * D;
  KV* vd = (KV*)c.Vg + dst * D;
  if constexpr (std::is_same<T, KV>::value) {
    for (int e = sub; e < D; e += 16) { kd[e] = Kg[(size_t)r * D + e]; vd[e] = Vg[(size_t)r * D + e]; }
  } else {
    float x[EL];
    load_slice<T, EL>(Kg + (size_t)r * D + sub * EL, x);
    store_cache_slice<KV, EL>(x, kd, c.Kg_scale + dst, sub);
    load_slice<T, EL>(Vg + (size_t)r * D + sub * EL, x);
    store_cache_slice<KV, EL>(x, vd, c.Vg_scale + dst, sub);
  }
}

static int check_cache(const tca_params* prm, const tca_cache* c) {
  if (!c) return fail(TCA_ERR_INVALID, "cache is NULL");
  if (c->batch < 1 || c->cap_rows < 0) return fail(TCA_ERR_INVALID, "cache: batch=%d cap_rows=%lld", c->batch,
                                                   (long long)c->cap_rows);
  if (!c->idx || !c->Kg || !c->Vg || !c->n_rows || !c->ringK || !c->ringV || !c->length)
    return fail(TCA_ERR_INVALID, "cache: NULL pointer member");
  if (c->kv_format != TCA_KV_NATIVE && c->kv_format != TCA_KV_FP8)
    return fail(TCA_ERR_UNSUPPORTED, "cache: kv_format=%d", c->kv_format);
  if (c->kv_format == TCA_KV_FP8) {
    if (prm->dtype != TCA_BF16) return fail(TCA_ERR_UNSUPPORTED, "cache: TCA_KV_FP8 requires dtype TCA_BF16");
    if (!c->Kg_scale || !c->Vg_scale || !c->ringK_scale || !c->ringV_scale)
      return fail(TCA_ERR_INVALID, "cache: NULL scale pointer with TCA_KV_FP8");
  }
  return TCA_OK;
}

template <typename T, typename KV, int D>
static int run_decode(const tca_params* prm, const tca_cache* c, const DecodeHeads& dh, int64_t max_rows,
                      const T* q, const T* k_new, const T* v_new, T* O, void* ws, hipStream_t st) {
  const int Hq = prm->n_q_heads, Hkv = prm->n_kv_heads, B = c->batch, w = prm->window;
  const int Hs = sel_heads(prm), GS = sel_group(prm);
  const int g_slots = global_slots(prm, max_rows), n_slots = g_slots + window_slots(prm);
  DecodeWs dw = carve_decode_ws(ws, B, Hq, D, n_slots);
  hipLaunchKernelGGL((decode_prep_kernel<T, KV, D>), dim3(B, (Hs + 3) / 4), dim3(256), 0, st, *c, dh, Hs, Hkv, w, k_new,
                     v_new, dw.n_vis);
  const double sc = logit_scale(prm);
  // (queries per region row, queries per ring row): (G, G) for a shared selection, else (1, G)
  const int G = Hq / Hkv;
#define TCA_PARTIAL_CASE(GG)                                                                                    \
  case GG:                                                                                                      \
    if (GS > 1)                                                                                                 \
      hipLaunchKernelGGL((decode_partial_kernel<T, KV, D, GG, GG>), dim3(n_slots, Hs, B), dim3(kPartThreads), 0, st, \
                         *c, dh, Hq, Hkv, w, g_slots, n_slots, sc, q, dw.n_vis, dw.part);                       \
    else                                                                                                        \
      hipLaunchKernelGGL((decode_partial_kernel<T, KV, D, 1, GG>), dim3(n_slots, Hs, B), dim3(kPartThreads), 0, st, \
                         *c, dh, Hq, Hkv, w, g_slots, n_slots, sc, q, dw.n_vis, dw.part);                       \
    break;
  switch (G) {
    TCA_PARTIAL_CASE(1) TCA_PARTIAL_CASE(2) TCA_PARTIAL_CASE(3) TCA_PARTIAL_CASE(4)
    TCA_PARTIAL_CASE(5) TCA_PARTIAL_CASE(6) TCA_PARTIAL_CASE(7) TCA_PARTIAL_CASE(8)
  }
#undef TCA_PARTIAL_CASE
  hipLaunchKernelGGL((decode_merge_kernel<T, KV, D>), dim3(Hq, B), dim3(kDecThreads), 0, st, *c, dh, Hq, Hkv, GS, w,
                     prm->block, n_slots, logit_scale(prm), q, dw.part, O);
  hipLaunchKernelGGL(decode_advance_kernel, dim3((B + 63) / 64), dim3(64), 0, st, c->length, B);
  return TCA_OK;
}

}  // namespace tca

using namespace tca;

extern "C" size_t tca_decode_workspace_bytes(const tca_params* prm, int batch, int64_t max_head_rows) {
  if (check_params(prm) != TCA_OK || batch < 1 || max_head_rows < 0) return 0;
  const int n_slots = global_slots(prm, max_head_rows) + window_slots(prm);
  return carve_decode_ws(nullptr, batch, prm->n_q_heads, prm->head_dim, n_slots).bytes;
}

extern "C" int tca_cache_load_window(const tca_params* prm, const tca_cache* cache, int seq, const void* K,
                                     const void* V, int64_t kv_stride, int64_t L, void* stream) {
  int rc = check_params(prm);
  if (rc) return rc;
  rc = check_cache(prm, cache);
  if (rc) return rc;
  if (!K || !V || seq < 0 || seq >= cache->batch || L < 0 || L > kv_stride)
    return fail(TCA_ERR_INVALID, "tca_cache_load_window: seq=%d L=%lld kv_stride=%lld", seq, (long long)L,
                (long long)kv_stride);
  const int w = prm->window;
  const int64_t rows = L < w ? L : w;
  dim3 grid((unsigned)((rows + 15) / 16 > 0 ? (rows + 15) / 16 : 1), prm->n_kv_heads);
  hipStream_t st = (hipStream_t)stream;
  const bool d128 = prm->head_dim == 128;
#define TCA_LOAD_WINDOW(TT, KK, DD)                                                                            \
  hipLaunchKernelGGL((load_window_kernel<TT, KK, DD>), grid, dim3(256), 0, st, *cache, seq, prm->n_kv_heads, w, \
                     (const TT*)K, (const TT*)V, kv_stride, L)
  if (cache->kv_format == TCA_KV_FP8) { if (d128) TCA_LOAD_WINDOW(bf16_t, fp8_t, 128); else TCA_LOAD_WINDOW(bf16_t, fp8_t, 64); }
  else if (prm->dtype == TCA_BF16) { if (d128) TCA_LOAD_WINDOW(bf16_t, bf16_t, 128); else TCA_LOAD_WINDOW(bf16_t, bf16_t, 64); }
  else { if (d128) TCA_LOAD_WINDOW(float, float, 128); else TCA_LOAD_WINDOW(float, float, 64); }
#undef TCA_LOAD_WINDOW
  TCA_HIP_CHECK(hipGetLastError());
  return TCA_OK;
}

extern "C" int tca_cache_load_global(const tca_params* prm, const tca_cache* cache, int seq, const int32_t* idx,
                                     const void* Kg, const void* Vg, const int64_t* offs, const int32_t* n_rows,
                                     void* stream) {
  int rc = check_params(prm);
  if (rc) return rc;
  rc = check_cache(prm, cache);
  if (rc) return rc;
  const int Hs = sel_heads(prm);
  if (!idx || !Kg || !Vg || !offs || !n_rows || seq < 0 || seq >= cache->batch)
    return fail(TCA_ERR_INVALID, "tca_cache_load_global: NULL pointer argument or seq=%d outside the batch", seq);
  if (offs[0] != 0 || offs[Hs] != cache->cap_rows)
    return fail(TCA_ERR_INVALID, "tca_cache_load_global: offs[0] must be 0 and offs[Hs] must equal cap_rows");
  DecodeHeads dh;
  for (int h = 0; h < Hs; ++h) {
    if (offs[h + 1] < offs[h]) return fail(TCA_ERR_INVALID, "tca_cache_load_global: offs not ascending at %d", h);
    dh.offs[h] = offs[h];
    dh.t_dec[h] = 0;
  }
  dh.offs[Hs] = offs[Hs];
  if (cache->cap_rows == 0) return TCA_OK;
  hipStream_t st = (hipStream_t)stream;
  dim3 grid((unsigned)((cache->cap_rows + 15) / 16));
  const bool d128 = prm->head_dim == 128;
#define TCA_LOAD_GLOBAL(TT, KK, DD)                                                                      \
  hipLaunchKernelGGL((load_global_kernel<TT, KK, DD>), grid, dim3(256), 0, st, *cache, seq, dh, Hs, idx, \
                     (const TT*)Kg, (const TT*)Vg, n_rows)
  if (cache->kv_format == TCA_KV_FP8) { if (d128) TCA_LOAD_GLOBAL(bf16_t, fp8_t, 128); else TCA_LOAD_GLOBAL(bf16_t, fp8_t, 64); }
  else if (prm->dtype == TCA_BF16) { if (d128) TCA_LOAD_GLOBAL(bf16_t, bf16_t, 128); else TCA_LOAD_GLOBAL(bf16_t, bf16_t, 64); }
  else { if (d128) TCA_LOAD_GLOBAL(float, float, 128); else TCA_LOAD_GLOBAL(float, float, 64); }
#undef TCA_LOAD_GLOBAL
  TCA_HIP_CHECK(hipGetLastError());
  return TCA_OK;
}

// Argument checks and the four launches of a step, on a caller-visible scratch buffer.
static int decode_step(const tca_params* prm, const tca_cache* cache, const int64_t* offs, const void* q,
                       const void* k_new, const void* v_new, const double* p, void* O, void* ws, size_t ws_bytes,
                       void* stream, const char* who) {
  int rc = check_params(prm);
  if (rc) return rc;
  rc = check_cache(prm, cache);
  if (rc) return rc;
  if (!offs || !q || !k_new || !v_new || !p || !O || !ws)
    return fail(TCA_ERR_INVALID, "%s: NULL pointer argument", who);
  const int Hs = sel_heads(prm), b = prm->block, nk = block_log2(b) + 1;
  if (offs[0] != 0 || offs[Hs] != cache->cap_rows)
    return fail(TCA_ERR_INVALID, "%s: offs[0] must be 0 and offs[Hs] must equal cap_rows", who);
  DecodeHeads dh;
  int64_t max_rows = 0;
  for (int h = 0; h < Hs; ++h) {
    if (offs[h + 1] < offs[h]) return fail(TCA_ERR_INVALID, "%s: offs not ascending at %d", who, h);
    if (offs[h + 1] - offs[h] > INT32_MAX) return fail(TCA_ERR_UNSUPPORTED, "head region beyond int32 rows");
    if (offs[h + 1] - offs[h] > max_rows) max_rows = offs[h + 1] - offs[h];
    if (!valid_config(p + (size_t)h * nk, nk))
      return fail(TCA_ERR_INVALID, "%s: p[%d] is not a distribution", who, h);
    dh.offs[h] = offs[h];
    dh.t_dec[h] = tca_decode_budget(b, p + (size_t)h * nk);
  }
  dh.offs[Hs] = offs[Hs];
  if (global_slots(prm, max_rows) + window_slots(prm) > kMaxSlots)
    return fail(TCA_ERR_UNSUPPORTED, "%s: more than %d split-K slots per head", who, kMaxSlots);
  const size_t need = tca_decode_workspace_bytes(prm, cache->batch, max_rows);
  if (ws_bytes < need || ((uintptr_t)ws & 255))
    return fail(TCA_ERR_WORKSPACE, "%s: scratch needs %zu bytes, 256-byte aligned; %zu available", who, need,
                ws_bytes);
  hipStream_t st = (hipStream_t)stream;
#define TCA_RUN_DECODE(TT, KK)                                                                                         \
  (prm->head_dim == 128                                                                                                \
       ? run_decode<TT, KK, 128>(prm, cache, dh, max_rows, (const TT*)q, (const TT*)k_new, (const TT*)v_new, (TT*)O, ws, st) \
       : run_decode<TT, KK, 64>(prm, cache, dh, max_rows, (const TT*)q, (const TT*)k_new, (const TT*)v_new, (TT*)O, ws, st))
  if (cache->kv_format == TCA_KV_FP8) rc = TCA_RUN_DECODE(bf16_t, fp8_t);
  else if (prm->dtype == TCA_BF16) rc = TCA_RUN_DECODE(bf16_t, bf16_t);
  else rc = TCA_RUN_DECODE(float, float);
#undef TCA_RUN_DECODE
  if (rc) return rc;
  TCA_HIP_CHECK(hipGetLastError());
  return TCA_OK;
}

extern "C" int tca_decode(const tca_params* prm, const tca_cache* cache, const int64_t* offs, const void* q,
                          const void* k_new, const void* v_new, const double* p, void* O, void* ws,
                          size_t ws_bytes, void* stream) {
  return decode_step(prm, cache, offs, q, k_new, v_new, p, O, ws, ws_bytes, stream, "tca_decode");
}

// ---- tca_decode_static: the same step for callers that cannot provide scratch memory.
// The split-K partials live in an array that is part of the library's code object: every GPU the
// library runs on holds its own copy, at its own address, from the moment the code object is
// loaded until the process ends.  `scratch` below is only a host-side handle of that array; the
// device address is asked for once per device and kept.
static __device__ __align__(256) unsigned char scratch[TCA_DECODE_STATIC_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_addr[kMaxDevices];
}  // namespace

extern "C" int tca_decode_static(const tca_params* prm, const tca_cache* cache, const int64_t* offs, const void* q,
                                 const void* k_new, const void* v_new, const double* p, void* O, void* stream) {
  int dev = -1;
  TCA_HIP_CHECK(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return fail(TCA_ERR_UNSUPPORTED, "tca_decode_static: device %d", dev);
  void* ptr = g_scratch_addr[dev].load(std::memory_order_acquire);
  if (!ptr) {                                          // first call on this device (it is the current one)
    TCA_HIP_CHECK(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
    if (!ptr) return fail(TCA_ERR_HIP, "tca_decode_static: no device address for the scratch array");
    g_scratch_addr[dev].store(ptr, std::memory_order_release);   // racing first calls store the same address
  }
  return decode_step(prm, cache, offs, q, k_new, v_new, p, O, ptr, (size_t)TCA_DECODE_STATIC_BYTES, stream,
                     "tca_decode_static");
}
