// Layer integration in front of the path (an extension; the paper's method starts from Q, K, V):
// the projections Q = X W_Q, K = X W_K, V = X W_V of Sec. III for all heads in one launch, written
// straight into the layouts tca_select / tca_prefill (head-major) or tca_decode (token-major) read.
//
// bf16: a dense contraction, so it runs on the matrix cores.  One workgroup (8 waves, two per SIMD)
// forms a 256-feature x 256-token tile of Y^T = W X^T with v_mfma_f32_32x32x16_bf16; a wave owns 128
// features (one head for d = 128, two for d = 64) x 64 tokens = 4 x 2 accumulator blocks, so that a
// k-step of 16 takes six fragment reads for eight MFMAs.  The hidden dimension is walked in stages of
// 64; the W and X slices of a stage (32 KB each) go global -> LDS with the LDS modifier of the
// buffer loads (no staging registers), XOR-swizzled so that the 16-byte fragment reads are free of
// bank conflicts, two stages resident.  The one barrier of a stage sits in front of the stage's
// last k-step, whose fragments are in registers by then: after it no wave reads the stage any more,
// so the copies of the stage after next start there, and the first fragments of the next stage are
// read under the last MFMAs.  Features are the rows of the MFMA result, so a lane ends up with four
// consecutive features of one token: one 8-byte store each.
//
// fp32: one thread per output, fp32 multiply-adds in the order of the hidden index (small cases and
// an independent check of the bf16 kernel's indexing).
#include <hip/hip_runtime.h>

#include <type_traits>

#include "tca_common.h"
#include "tca_device.h"

namespace tca {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4_t;

constexpr int kPF = 256;                         // features per workgroup
constexpr int kPT = 256;                         // tokens per workgroup
constexpr int kPK = 64;                          // the hidden size must be a multiple of this

// Where the projected rows go.  Part 0 = Q, 1 = K, 2 = V; feature f belongs to head f / d of the
// concatenation (Hq query heads, Hkv key heads, Hkv value heads).  Element e of head h (counted
// inside its part) of token t lands at base[part] + h * head_stride[part] + t * token_stride[part] + e.
struct QkvOut {
  void* base[3];
  int64_t head_stride[3], token_stride[3];
  int first_head[4];                             // part p holds the heads [first_head[p], first_head[p+1])
};

// 16 bytes per lane, global -> LDS (lanes deposit at consecutive addresses from lds_dst on); lane_off: the
// lane's byte offset into the buffer, tile_off: a scalar byte offset on top
__device__ __forceinline__ void copy16_to_lds(__amdgpu_buffer_rsrc_t rsrc, int lane_off, int tile_off,
                                              unsigned char* lds_dst) {
  __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (__attribute__((address_space(3))) void*)lds_dst, 16, lane_off,
                                           tile_off, 0, 0);
}

__device__ __forceinline__ int part_of_head(const QkvOut& o, int hg) { return hg < o.first_head[1] ? 0 : hg < o.first_head[2] ? 1 : 2; }

// WT: tokens per wave (64: eight waves, two per SIMD; 128: four waves, one per SIMD, each fragment of W
// feeding four MFMAs).  BK: hidden elements per stage (32 or 64); NST: stages resident in LDS.
// grid: 8 * groups * 4 * n_ft workgroups (see the id map below); block 2 * (256 / WT) * 64.
template <int WT, int BK, int NST>
__global__ __launch_bounds__(2 * (kPT / WT) * 64) __attribute__((amdgpu_waves_per_eu(128 / WT, 128 / WT)))
void qkv_mfma_kernel(const uint16_t* __restrict__ W, const uint16_t* __restrict__ X, const uint16_t* __restrict__ bias,
                     int n_feat, int64_t n_tok, int hidden, int d, QkvOut out, int n_ft, int n_tt) {
  constexpr int ROWB = BK * 2;                   // bytes of a tile row
  constexpr int CPR = ROWB / 16;                 // 16-byte chunks per tile row (8 or 4)
  constexpr int TILEB = kPF * ROWB;              // one operand's slice of a stage (kPF == kPT)
  constexpr int STAGEB = 2 * TILEB;
  constexpr int KS = BK / 16;                    // k-steps per stage
  constexpr int TB = WT / 32;                    // token blocks per wave
  constexpr int NW = 2 * (kPT / WT);             // waves
  constexpr int NL = TILEB / 1024 / NW;          // wave-loads per wave, per operand and stage
  static_assert(NST * STAGEB <= 160 * 1024 && NL >= 1 && 2 * NL < 64, "shape");
  __shared__ __attribute__((aligned(16))) unsigned char lds[NST * STAGEB];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  // Workgroup ids go round-robin over the 8 XCDs.  An XCD takes every eighth token tile; the 32
  // workgroups it runs at a time are 8 feature tiles x 4 token tiles, which walk the hidden dimension
  // side by side: their L2 sees each W slice four times and each X slice eight times.
  const int x = blockIdx.x & 7, u = blockIdx.x >> 3;
  const int per_group = 4 * n_ft;
  const int grp = u / per_group, in = u - grp * per_group;
  const int ft = in >> 2, tt = (grp * 4 + (in & 3)) * 8 + x;
  if (tt >= n_tt) return;
  const int wf = wv & 1, wt = wv >> 1;           // the wave's 128 features and WT tokens inside the tile
  const int64_t f0 = (int64_t)ft * kPF, t0 = (int64_t)tt * kPT;
  const int rows_w = n_feat - f0 < kPF ? (int)(n_feat - f0) : kPF;
  const int rows_x = n_tok - t0 < kPT ? (int)(n_tok - t0) : kPT;

  // ---- copies.  Chunk c of tile row r sits at chunk position c ^ swz(r), where swz makes the 16 rows a
  // quarter-wave reads at one chunk column fall into distinct banks.  Rows past the end of W or X read
  // as zero (range check of the descriptor).
  auto swz_of = [](int r) { return CPR == 8 ? (r >> 1) & 7 : (r >> 2) & 3; };
  constexpr int kRsrcFlags = 0x00020000;         // raw buffer, 32-bit data format
  const __amdgpu_buffer_rsrc_t rs_w = __builtin_amdgcn_make_buffer_rsrc((void*)(W + f0 * hidden), 0, rows_w * hidden * 2, kRsrcFlags);
  const __amdgpu_buffer_rsrc_t rs_x = __builtin_amdgcn_make_buffer_rsrc((void*)(X + t0 * hidden), 0, rows_x * hidden * 2, kRsrcFlags);
  int lo[NL];                                    // this lane's byte offset into the operand, per wave-load (same for W and X)
#pragma unroll
  for (int j = 0; j < NL; ++j) {
    const int cid = (wv * NL + j) * 64 + lane;   // 16-byte chunk of the LDS tile this lane fills
    const int r = cid / CPR, pch = cid % CPR;
    lo[j] = r * hidden * 2 + ((pch ^ swz_of(r)) << 4);
  }
  auto issue = [&](int kt, int s) {
#pragma unroll
    for (int j = 0; j < NL; ++j) {
      unsigned char* dst = lds + s * STAGEB + (wv * NL + j) * 1024;
      copy16_to_lds(rs_w, lo[j], kt * ROWB, dst);
      copy16_to_lds(rs_x, lo[j], kt * ROWB, dst + TILEB);
    }
  };

  // ---- fragments: lane = (row lane & 31, k half lane >> 5) of a 32-row block
  const int lrow = lane & 31, hh = lane >> 5;
  int fo[KS];                                    // byte offset inside a block of 32 rows, per k-step of a stage
#pragma unroll
  for (int kk = 0; kk < KS; ++kk) fo[kk] = lrow * ROWB + (((kk * 2 + hh) ^ swz_of(lrow)) << 4);
  const unsigned char* const wbase = lds + wf * (128 * ROWB);
  const unsigned char* const xbase = lds + TILEB + wt * (WT * ROWB);
  f32x16_t acc[4][TB];
#pragma unroll
  for (int fb = 0; fb < 4; ++fb)
#pragma unroll
    for (int tb = 0; tb < TB; ++tb)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[fb][tb][i] = 0.f;
  auto mma = [&](const bf16x8_t (&a)[4], const bf16x8_t (&b)[TB]) {
#pragma unroll
    for (int fb = 0; fb < 4; ++fb)
#pragma unroll
      for (int tb = 0; tb < TB; ++tb) acc[fb][tb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[fb], b[tb], acc[fb][tb], 0, 0, 0);
  };

  // Stage kt lives in place kt % NST.  The loop is cut at the barriers: a stretch starts behind the
  // barrier of stage kt - 1 with that stage's last k-step (its fragments are in registers), under
  // which the copies of stage kt + NST - 1 start, into the place stage kt - 1 has just left, and the
  // first fragments of stage kt arrive; then come the other k-steps of stage kt and its barrier.  There
  // is one copy of the stretch in the code (the place is a run-time offset; the first stretch
  // multiplies zeros for the stage that is not there, the last ones copy the last stage again instead
  // of stages that are not there), because every further copy of it costs registers the accumulators
  // need.  The order of a stretch's instructions is written out and fenced (sched_barrier): one MFMA,
  // behind every second one a fragment read of the next k-step in the order of need, behind each of the
  // stretch's first ones a copy.  Left to itself the compiler issues the copies in one burst and the
  // fragment reads in clumps (5 % slower, as is an order merely suggested through sched_group_barrier).
  static_assert(KS == 4 && NST >= 2, "the stretch below is four k-steps");
  const int nk = hidden / BK;
  constexpr int kGroup = 2 * NL;                 // loads of one stage, per wave
  constexpr int kAhead = (NST - 2) * kGroup;     // loads that may still be in flight when the next stage must be in
  static_assert(kAhead < 64, "vmcnt is six bits wide");
  constexpr int kWaitNext = 0x0F70 | (kAhead & 15) | ((kAhead >> 4) << 14);   // vmcnt: bits [3:0] and [15:14]
  bf16x8_t a0[4], b0[TB], a1[4], b1[TB];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
#pragma unroll
    for (int fb = 0; fb < 4; ++fb) a1[fb][i] = (__bf16)0.f;
#pragma unroll
    for (int tb = 0; tb < TB; ++tb) b1[tb][i] = (__bf16)0.f;
  }
#pragma unroll
  for (int j = 0; j + 1 < NST; ++j) issue(j < nk ? j : nk - 1, j);
  __builtin_amdgcn_s_waitcnt(kWaitNext);         // stage 0 is in
  __syncthreads();
  int s = 0;                                     // place of stage kt
  // fragment i of k-step kk of the stage in place sp, in the order the MFMAs need them: W block 0, the X
  // blocks, the other W blocks
  auto read_one = [&](int sp, int kk, int i, bf16x8_t (&a)[4], bf16x8_t (&b)[TB]) {
    if (i == 0) a[0] = *reinterpret_cast<const bf16x8_t*>(wbase + sp * STAGEB + fo[kk]);
    else if (i <= TB) b[i - 1] = *reinterpret_cast<const bf16x8_t*>(xbase + sp * STAGEB + (i - 1) * (32 * ROWB) + fo[kk]);
    else a[i - TB] = *reinterpret_cast<const bf16x8_t*>(wbase + sp * STAGEB + (i - TB) * (32 * ROWB) + fo[kk]);
  };
  // copy i of this wave's share of stage kt into place sp
  auto issue_one = [&](int kt, int sp, int i) {
    const int j = i >> 1;
    unsigned char* dst = lds + sp * STAGEB + (wv * NL + j) * 1024;
    if (i & 1) copy16_to_lds(rs_x, lo[j], kt * ROWB, dst + TILEB);
    else copy16_to_lds(rs_w, lo[j], kt * ROWB, dst);
  };
  // one k-step: the MFMAs of the current fragments (ca, cb); the reads of the fragments (na, nb) of k-step
  // kk of place sp; with COPY the copies of stage ckt into place cs
  constexpr int NM = 4 * TB, NR = 4 + TB, RSTEP = NM / NR > 1 ? 2 : 1;
  auto kstep = [&](const bf16x8_t (&ca)[4], const bf16x8_t (&cb)[TB], bf16x8_t (&na)[4], bf16x8_t (&nb)[TB], int sp, int kk,
                   auto copy_tag, int ckt, int cs) {
    constexpr bool COPY = decltype(copy_tag)::value;
#pragma unroll
    for (int j = 0; j < NM; ++j) {
      const int fb = j / TB, tb = j % TB;
      acc[fb][tb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ca[fb], cb[tb], acc[fb][tb], 0, 0, 0);
      if (j % RSTEP == 0 && j / RSTEP < NR) read_one(sp, kk, j / RSTEP, na, nb);
      if (COPY && j < kGroup) issue_one(ckt, cs, j);
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  for (int kt = 0; kt < nk; ++kt) {
    const int s_prev = s == 0 ? NST - 1 : s - 1;
    const int ckt = kt + NST - 1 < nk ? kt + NST - 1 : nk - 1;
    __builtin_amdgcn_sched_barrier(0);
    kstep(a1, b1, a0, b0, s, 0, std::true_type{}, ckt, s_prev);          // the last k-step of stage kt - 1
    kstep(a0, b0, a1, b1, s, 1, std::false_type{}, 0, 0);
    kstep(a1, b1, a0, b0, s, 2, std::false_type{}, 0, 0);
    kstep(a0, b0, a1, b1, s, 3, std::false_type{}, 0, 0);
    __builtin_amdgcn_s_waitcnt(kWaitNext);       // this wave's share of stage kt + 1 has landed
    __syncthreads();                             // everyone's has, and nobody reads stage kt any more
    s = s + 1 == NST ? 0 : s + 1;
  }
  mma(a1, b1);                                   // the last k-step of the last stage
  __builtin_amdgcn_s_waitcnt(0x0F70);            // no copy into this workgroup's LDS may outlive it

  // ---- epilogue: lane holds token column lrow of block tb; register 4 q4 + j is feature 8 q4 + 4 hh + j of block fb
#pragma unroll
  for (int fb = 0; fb < 4; ++fb) {
    const int64_t fblk = f0 + wf * 128 + fb * 32;            // first feature of the block (uniform)
    if (fblk >= n_feat) continue;                            // n_feat is a multiple of d >= 64: whole blocks
    const int hg = (int)(fblk / d), e0 = (int)(fblk - (int64_t)hg * d);
    const int p = part_of_head(out, hg);
    uint16_t* const hbase = (uint16_t*)out.base[p] + (int64_t)(hg - out.first_head[p]) * out.head_stride[p] + e0;
    float bs[4][4];
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4)
#pragma unroll
      for (int j = 0; j < 4; ++j) bs[q4][j] = bias ? bf16_to_f32(bias[fblk + 8 * q4 + 4 * hh + j]) : 0.f;
#pragma unroll
    for (int tb = 0; tb < TB; ++tb) {
      const int64_t t = t0 + wt * WT + tb * 32 + lrow;
      if (t >= n_tok) continue;
      uint16_t* const row = hbase + t * out.token_stride[p];
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        bf16x4_t pk;
#pragma unroll
        for (int j = 0; j < 4; ++j) pk[j] = (__bf16)(acc[fb][tb][4 * q4 + j] + bs[q4][j]);
        *reinterpret_cast<bf16x4_t*>(row + 8 * q4 + 4 * hh) = pk;
      }
    }
  }
}

// grid (ceil(n_feat / 256), n_tok); block 256: thread = one feature of one token.
template <typename T>
__global__ __launch_bounds__(256) void qkv_rows_kernel(const T* __restrict__ W, const T* __restrict__ X,
                                                       const T* __restrict__ bias, int n_feat, int hidden, int d,
                                                       QkvOut out) {
  const int f = blockIdx.x * 256 + threadIdx.x;
  const int64_t t = blockIdx.y;
  if (f >= n_feat) return;
  const T* w = W + (size_t)f * hidden;
  const T* xr = X + (size_t)t * hidden;
  float acc = 0.f;
  for (int c = 0; c < hidden; ++c) acc = fmaf(load_f32(xr + c), load_f32(w + c), acc);
  if (bias) acc += load_f32(bias + f);
  const int hg = f / d, e = f - hg * d;
  const int p = part_of_head(out, hg);
  store_f32((T*)out.base[p] + (int64_t)(hg - out.first_head[p]) * out.head_stride[p] + t * out.token_stride[p] + e, acc);
}

}  // namespace tca

using namespace tca;

// The shape in use: 64 tokens per wave (eight waves), stages of 64 hidden elements, two of them resident.
// Measured at 131072 rows, hidden 4096, 6144 features: 128 tokens per wave (four waves, a third fewer
// fragment reads) 8 % slower; stages of 32 elements, three to five resident (a copy has longer to
// arrive, twice the barriers) 15 % slower.
static constexpr int kWT = 64, kBK = 64, kNST = 2;

extern "C" int tca_qkv_project(const tca_params* prm, const void* X, int64_t n_tokens, int hidden, const void* W,
                               const void* bias, void* Q, int64_t q_token_stride, int64_t q_head_stride, void* K,
                               void* V, int64_t kv_token_stride, int64_t kv_head_stride, void* stream) {
  int rc = check_params(prm);
  if (rc) return rc;
  if (!X || !W || !Q || !K || !V || n_tokens < 0 || hidden < 1)
    return fail(TCA_ERR_INVALID, "tca_qkv_project: NULL pointer argument, n_tokens=%lld or hidden=%d", (long long)n_tokens,
                hidden);
  const int Hq = prm->n_q_heads, Hkv = prm->n_kv_heads, d = prm->head_dim;
  const int n_feat = (Hq + 2 * Hkv) * d;
  if (q_token_stride < d && n_tokens > 1) return fail(TCA_ERR_INVALID, "tca_qkv_project: q_token_stride=%lld", (long long)q_token_stride);
  if (kv_token_stride < d && n_tokens > 1) return fail(TCA_ERR_INVALID, "tca_qkv_project: kv_token_stride=%lld", (long long)kv_token_stride);
  if (q_head_stride < d || kv_head_stride < d)
    return fail(TCA_ERR_INVALID, "tca_qkv_project: head strides %lld, %lld", (long long)q_head_stride, (long long)kv_head_stride);
  if (n_tokens == 0) return TCA_OK;
  QkvOut out;
  out.base[0] = Q; out.base[1] = K; out.base[2] = V;
  out.head_stride[0] = q_head_stride; out.head_stride[1] = out.head_stride[2] = kv_head_stride;
  out.token_stride[0] = q_token_stride; out.token_stride[1] = out.token_stride[2] = kv_token_stride;
  out.first_head[0] = 0; out.first_head[1] = Hq; out.first_head[2] = Hq + Hkv; out.first_head[3] = Hq + 2 * Hkv;
  hipStream_t st = (hipStream_t)stream;
  if (prm->dtype == TCA_F32) {
    if (n_tokens > 65535) return fail(TCA_ERR_UNSUPPORTED, "tca_qkv_project (fp32): more than 65535 rows per call");
    hipLaunchKernelGGL((qkv_rows_kernel<float>), dim3((n_feat + 255) / 256, (unsigned)n_tokens), dim3(256), 0, st,
                       (const float*)W, (const float*)X, (const float*)bias, n_feat, hidden, d, out);
  } else {
    if (hidden % kPK) return fail(TCA_ERR_UNSUPPORTED, "tca_qkv_project (bf16): hidden=%d is not a multiple of %d", hidden, kPK);
    if ((int64_t)kPF * hidden * 2 > INT32_MAX) return fail(TCA_ERR_UNSUPPORTED, "tca_qkv_project (bf16): hidden=%d", hidden);
    if ((q_token_stride | q_head_stride | kv_token_stride | kv_head_stride) & 3 || ((uintptr_t)Q | (uintptr_t)K | (uintptr_t)V) & 7 ||
        ((uintptr_t)X | (uintptr_t)W) & 15)
      return fail(TCA_ERR_INVALID, "tca_qkv_project (bf16): strides must be multiples of 4 elements, outputs 8-byte and inputs 16-byte aligned");
    const int n_ft = (n_feat + kPF - 1) / kPF;
    const int64_t n_tt = (n_tokens + kPT - 1) / kPT;
    const int64_t groups = ((n_tt + 7) / 8 + 3) / 4;
    const int64_t n_wg = 8 * groups * 4 * n_ft;
    if (n_wg > INT32_MAX) return fail(TCA_ERR_UNSUPPORTED, "tca_qkv_project: n_tokens=%lld", (long long)n_tokens);
    hipLaunchKernelGGL((qkv_mfma_kernel<kWT, kBK, kNST>), dim3((unsigned)n_wg), dim3(2 * (kPT / kWT) * 64), 0, st, (const uint16_t*)W, (const uint16_t*)X,
                       (const uint16_t*)bias, n_feat, n_tokens, hidden, d, out, n_ft, (int)n_tt);
  }
  TCA_HIP_CHECK(hipGetLastError());
  return TCA_OK;
}
