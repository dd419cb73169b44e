// bf16 MFMA flash-attention prefill over the global and local subsets (Eq. 2;
// Alg. 2 line 7) for gfx950.
//
// Work decomposition.  One workgroup = 4 wavefronts = one tile of BM = 128
// consecutive queries of one query head; wave v owns 32 of them.  The
// workgroup walks 64-key tiles: first the head's compacted global rows (tiles
// of the head's region of Kg), then the dense keys of the sliding window
// (absolute 64-key tiles of K).  Visibility is a prefix test in both parts:
//   global row g of the region : g  < nvis(i) = #{idx <= i-w}   (idx ascends)
//   dense key j                : i-w < j <= i
// so only boundary tiles evaluate a mask.
//
// MFMA mapping (v_mfma_f32_32x32x16_bf16, 64 lanes; lane = (hh = lane/32, c = lane%32)):
//   S^T = K Q^T  : A = K rows (key = c, 8 consecutive d), B = Q (query = c, same 8 d),
//                  C[key = 8*(r/4)+4*hh+r%4][query = c].  A lane therefore holds 16
//                  keys of ONE query per 32-key sub-tile: the softmax max/sum are
//                  in-register reductions plus one exchange between the two halves.
//   O^T = V^T P^T: B = P^T taken straight from the C registers of S^T (registers
//                  8g..8g+7 -> one bf16x8), A = V^T (d = c, the same 8 keys).  V^T
//                  tiles are produced once per call by a transposing pre-pass into
//                  the workspace, with the 64 keys of a tile stored in the order
//                  the C registers hold them, so the A operand is one 16-byte LDS read.
//   O^T accumulators: C[d = 32*s + 8*(r/4)+4*hh+r%4][query = c]: every register of
//                  a lane belongs to the same query, so rescaling is a per-lane scalar.
//
// LDS holds a ring of two K tiles [64][D] and a ring of two V^T tiles [D][64] with
// XOR-swizzled 16-byte chunks (conflict-free b128 reads without padding), filled by
// direct global -> LDS loads.  The loop is software-pipelined by one tile (see the
// kernel); one barrier per tile.
#include <hip/hip_runtime.h>

#include <type_traits>

#include "tca_prefill.h"

namespace tca {
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4_t;

constexpr int kBN = 64;              // keys per tile
constexpr int kFragAhead = 4;        // LDS fragment reads in flight ahead of the MFMA that uses them

struct PrefillHeads {
  int64_t offs[TCA_MAX_HEADS + 1];      // row offsets of the heads' regions
  int32_t tile_off[TCA_MAX_HEADS + 1];  // V^T tile offsets of the heads' regions
};

// position p (0..63) inside a stored V^T tile -> key (0..63) of the tile
__host__ __device__ inline int vt_key_of_pos(int p) {
  const int sub = p >> 5, q = p & 31;
  const int g = q >> 4, hh = (q >> 3) & 1, e = q & 7;
  return sub * 32 + 16 * g + 8 * (e >> 2) + 4 * hh + (e & 3);
}

// ---------------------------------------------------------------- pre-pass --
// Transposes 64-row tiles of a row-major [rows, D] bf16 matrix into
// [D][64] tiles (keys permuted by vt_key_of_pos); rows >= n_valid become zero.
// grid (tiles, groups); block 256.
template <int D>
__global__ __launch_bounds__(256) void transpose_tiles_kernel(
    const uint16_t* __restrict__ src, int64_t group_stride_rows, const int32_t* group_valid,
    int64_t valid_all, int64_t first_row, uint16_t* __restrict__ dst, int tiles_per_group,
    PrefillHeads ph, int mode, unsigned long long* clk) {
  // mode 0: global regions (group = selection head; rows from ph.offs, valid rows from group_valid)
  // mode 1: dense K/V (group = KV head; absolute rows first_row + 64*tile, valid while < valid_all)
  __shared__ uint16_t tile[kBN][D + 8];
  const int g = blockIdx.y, t = blockIdx.x, tid = threadIdx.x;
  if (clk && g == 0 && t == 0 && tid < 2) clk[tid] = 0;      // the attention kernel that follows accumulates here
  int64_t row0;
  int64_t n_valid;
  size_t out_tile;
  if (mode == 0) {
    const int64_t cap = ph.offs[g + 1] - ph.offs[g];
    const int ntile = (int)((cap + kBN - 1) / kBN);
    if (t >= ntile) return;
    row0 = ph.offs[g] + (int64_t)t * kBN;
    n_valid = (int64_t)group_valid[g] - (int64_t)t * kBN;
    out_tile = (size_t)ph.tile_off[g] + t;
  } else {
    row0 = (int64_t)g * group_stride_rows + first_row + (int64_t)t * kBN;
    n_valid = valid_all - (first_row + (int64_t)t * kBN);
    out_tile = (size_t)g * tiles_per_group + t;
  }
  constexpr int CPR = D / 8;                       // 16-byte chunks per row
  for (int c = tid; c < kBN * CPR; c += 256) {
    const int r = c / CPR, part = c - r * CPR;
    uint4 v = make_uint4(0, 0, 0, 0);
    if (r < n_valid) v = *reinterpret_cast<const uint4*>(src + (size_t)(row0 + r) * D + part * 8);
    *reinterpret_cast<uint4*>(&tile[r][part * 8]) = v;
  }
  __syncthreads();
  uint16_t* out = dst + out_tile * (size_t)(D * kBN);
  for (int c = tid; c < D * (kBN / 8); c += 256) {
    const int dd = c / (kBN / 8), part = c - dd * (kBN / 8);
    uint16_t v[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = tile[vt_key_of_pos(part * 8 + e)][dd];
    uint4 pk;
    pk.x = v[0] | ((uint32_t)v[1] << 16);
    pk.y = v[2] | ((uint32_t)v[3] << 16);
    pk.z = v[4] | ((uint32_t)v[5] << 16);
    pk.w = v[6] | ((uint32_t)v[7] << 16);
    *reinterpret_cast<uint4*>(out + (size_t)dd * kBN + part * 8) = pk;
  }
}

// ------------------------------------------------------------- main kernel --
__device__ __forceinline__ int64_t i64min(int64_t a, int64_t b) { return a < b ? a : b; }

__device__ __forceinline__ int count_le_i32(const int32_t* idx, int n, int64_t bound) {
  int lo = 0, hi = n;
  while (lo < hi) {
    const int mid = (lo + hi) >> 1;
    if ((int64_t)idx[mid] <= bound) lo = mid + 1; else hi = mid;
  }
  return lo;
}

// Cross-half exchange: returns max over the two 32-lane halves, in every lane.
__device__ __forceinline__ float half_max(float v) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float half_sum(float v) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// LDS byte offset of 16-byte chunk `ch` of K row r / V^T row dd (XOR swizzle, no padding)
template <int D> __device__ __forceinline__ int k_off(int r, int ch) {
  const int swz = (D / 8 == 16) ? (r & 15) : ((r >> 1) & 7);
  return r * (D * 2) + ((ch ^ swz) << 4);
}
__device__ __forceinline__ int v_off(int dd, int ch) { return dd * (kBN * 2) + ((ch ^ ((dd >> 1) & 7)) << 4); }

// Tile copies go global -> LDS directly (buffer loads with the LDS modifier: no
// staging registers, no ds_write).  Every lane of a wave-load deposits 16 bytes at
// consecutive LDS addresses, so the lane that fills LDS chunk position p of a row
// fetches the global chunk the XOR swizzle assigns to p: a per-lane byte offset
// inside the tile that never changes.  The tile itself is selected by the scalar
// offset of the load, and rows past the end of a buffer read as zero (range check of
// the buffer descriptor), so a copy costs no vector ALU work at all.  A K tile is CPR
// wave-loads, a V^T tile D/8; each wave issues its share one load at a time, spread
// between the MFMAs instead of queueing up behind the barrier.
template <int D, int NW>
struct TileCopy {
  static constexpr int CPR = D / 8;
  static constexpr int NK = CPR / NW;               // K wave-loads per wave
  static constexpr int NV = D / 8 / NW;             // V^T wave-loads per wave
  static constexpr int N = NK + NV;
  static_assert(NK >= 1 && NV >= 1 && N <= D / 16, "too many or too few waves for this tile");
  // byte offset inside a K tile of the chunk this lane fetches in wave-load q
  static __device__ __forceinline__ int k_lane_offset(int q, int lane) {
    const int cid = q * 64 + lane;                  // 16-byte chunk of the LDS tile this lane fills
    const int r = cid / CPR, pch = cid % CPR;
    const int swz = (CPR == 16) ? (r & 15) : ((r >> 1) & 7);
    return (r * D + (pch ^ swz) * 8) * 2;
  }
  static __device__ __forceinline__ int v_lane_offset(int q, int lane) {
    const int cid = q * 64 + lane;
    const int dd = cid >> 3, pch = cid & 7;
    return (dd * kBN + (pch ^ ((dd >> 1) & 7)) * 8) * 2;
  }
};

__device__ __forceinline__ void copy16_to_lds(__amdgpu_buffer_rsrc_t rsrc, int lane_off, int tile_off,
                                              unsigned char* lds_dst) {
  __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (__attribute__((address_space(3))) void*)lds_dst, 16, lane_off,
                                           tile_off, 0, 0);
}

// Software pipeline over the tiles of a workgroup (tile t = 0 .. n_tiles-1: first the
// n_gt tiles of the head's compacted region, then the dense tiles of the window):
//   iteration t :  S(t+1) = K(t+1) Q^T      (MFMA)     }  one basic block: the MFMAs of the
//                  P(t)   = softmax step on S(t) (VALU) }  next tile run under this tile's exps
//                  O     += V(t)^T P(t)     (MFMA)
// K(t+2) and V^T(t+1) are copied global -> LDS during iteration t.  The K ring and
// the V^T ring hold two tiles each; one barrier per iteration.
// Positions and byte offsets are 32-bit here: the host checks (q_pos0 + n_queries) * D * 2 < 2^31.
template <int D, int NW>
__global__ __launch_bounds__(NW * 64, 8 / NW) void prefill_mfma_kernel(
    const uint16_t* __restrict__ Q, int64_t q_pos0, int64_t n_queries, const uint16_t* __restrict__ K,
    int64_t kv_stride, const int32_t* __restrict__ idx, const uint16_t* __restrict__ Kg,
    const int32_t* __restrict__ n_rows, const uint16_t* __restrict__ Vgt, const uint16_t* __restrict__ Vt,
    int64_t dense_tile0, int dense_tiles, PrefillHeads ph, int Hq, int G, int GS, int w, float scale,
    uint16_t* __restrict__ O, float* __restrict__ lse, unsigned long long* __restrict__ clk) {
  constexpr int KK = D / 16;             // MFMA k-steps over the head dimension
  constexpr int DS = D / 32;             // 32-row slices of O^T
  constexpr int BM = NW * 32;            // queries per workgroup, 32 per wave
  const unsigned long long clk_c0 = __builtin_readcyclecounter(), clk_r0 = __builtin_amdgcn_s_memrealtime();
  constexpr int KBYTES = kBN * D * 2;    // K tile
  constexpr int VBYTES = D * kBN * 2;    // V^T tile
  // Rows are not padded; the 16-byte chunk index is XOR-swizzled with the row so that
  // the b128 reads of 16 consecutive rows at one chunk column fall into distinct banks.
  __shared__ __attribute__((aligned(16))) unsigned char lds[2 * KBYTES + 2 * VBYTES];
  unsigned char* const kring = lds;
  unsigned char* const vring = lds + 2 * KBYTES;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);     // wave index, scalar
  const int hh = lane >> 5, c = lane & 31;
  const int n_qt = (int)((n_queries + BM - 1) / BM);
  const int bid = blockIdx.x;
  // Workgroup ids go round-robin over the 8 XCDs, each with an L2 of its own.  With Hq a multiple
  // of 8, XCD x is given the heads x*Hq/8 .. (x+1)*Hq/8 - 1 and works through them one at a time:
  // the query tiles in flight on an XCD then belong to one head and stream the same K / V^T tiles
  // through its L2 (and the heads of a KV group, which share the dense tiles - with a shared
  // selection all tiles - follow each other on the same XCD).
  int h, qtile;
  if ((Hq & 7) == 0) {
    const int u = bid >> 3;                        // position in the XCD's own sequence
    h = (bid & 7) * (Hq >> 3) + u / n_qt;          // one head at a time per XCD
    qtile = n_qt - 1 - u % n_qt;                   // longest tiles first
  } else {
    h = bid % Hq;
    qtile = n_qt - 1 - bid / Hq;
  }
  const int kvh = h / G;
  const int64_t r0 = (int64_t)qtile * BM;          // first query row of the workgroup
  const int64_t last_row = n_queries - 1;
  const float sl2e = scale * 1.4426950408889634f;

  // ---- per-lane query state (lane column c = one query)
  const int hs = h / GS;                           // the selection this query head reads (GS query heads share it)
  const int64_t base = ph.offs[hs];
  const int nr = n_rows[hs];
  int64_t qrow_i = r0 + wv * 32 + c;
  if (qrow_i > last_row) qrow_i = last_row;         // clamped rows compute a duplicate; never stored
  const int qpos = (int)(q_pos0 + qrow_i);
  const int nvis = count_le_i32(idx + base, nr, (int64_t)qpos - w);
  bf16x8_t qf[KK];
  {
    const uint16_t* qrow = Q + ((size_t)h * n_queries + qrow_i) * D;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) qf[kk] = *reinterpret_cast<const bf16x8_t*>(qrow + kk * 16 + hh * 8);
  }
  // wave-level visibility bounds (queries ascend with the lane index c; clamped rows repeat the last)
  const int wave_first = (int)(q_pos0 + i64min(r0 + wv * 32, last_row));
  const int wave_last = (int)(q_pos0 + i64min(r0 + wv * 32 + 31, last_row));
  const int wg_last = (int)(q_pos0 + i64min(r0 + BM - 1, last_row));
  const int wg_first = (int)(q_pos0 + r0);
  const int last_pos = (int)(q_pos0 + last_row);
  // the searches below take wave-uniform arguments; readfirstlane keeps the results scalar
  const int nv_wave_lo = __builtin_amdgcn_readfirstlane(count_le_i32(idx + base, nr, (int64_t)wave_first - w));  // visible to every query of the wave
  const int nv_wg_hi = __builtin_amdgcn_readfirstlane(count_le_i32(idx + base, nr, (int64_t)wg_last - w));
  const int n_gt = (nv_wg_hi + kBN - 1) / kBN;
  const int win_lo = wg_first - w + 1 > 0 ? wg_first - w + 1 : 0;
  const int wt0 = win_lo / kBN, wt1 = wg_last / kBN;                      // absolute dense tiles [wt0, wt1]
  const int n_tiles = n_gt + (wt1 - wt0 + 1);
  const int last = n_tiles - 1;
  const int dshift = wt0 - n_gt;                   // tile t >= n_gt is the dense tile t + dshift

  // ---- sources of the tile copies: one descriptor per buffer, the tile chosen by a scalar byte offset
  using Copy = TileCopy<D, NW>;
  constexpr int kRsrcFlags = 0x00020000;           // raw buffer, 32-bit data format
  const __amdgpu_buffer_rsrc_t krs_g = __builtin_amdgcn_make_buffer_rsrc(
      (void*)(Kg + (size_t)base * D), 0, nr * (D * 2), kRsrcFlags);
  const __amdgpu_buffer_rsrc_t krs_d = __builtin_amdgcn_make_buffer_rsrc(
      (void*)(K + (size_t)kvh * kv_stride * D), 0, (last_pos + 1) * (D * 2), kRsrcFlags);
  const __amdgpu_buffer_rsrc_t vrs_g = __builtin_amdgcn_make_buffer_rsrc(
      (void*)(Vgt + (size_t)ph.tile_off[hs] * (D * kBN)), 0, n_gt * VBYTES, kRsrcFlags);
  const __amdgpu_buffer_rsrc_t vrs_d = __builtin_amdgcn_make_buffer_rsrc(
      (void*)(Vt + (size_t)kvh * dense_tiles * (D * kBN)), 0, dense_tiles * VBYTES, kRsrcFlags);
  const int vdshift = dshift - (int)dense_tile0;   // tile t >= n_gt is tile t + vdshift of the dense V^T buffer
  int klo[Copy::NK], vlo[Copy::NV];                // this lane's byte offsets inside a tile, per wave-load
#pragma unroll
  for (int j = 0; j < Copy::NK; ++j) klo[j] = Copy::k_lane_offset(wv * Copy::NK + j, lane);
#pragma unroll
  for (int j = 0; j < Copy::NV; ++j) vlo[j] = Copy::v_lane_offset(wv * Copy::NV + j, lane);
  // One K tile and one V^T tile to copy: descriptors and scalar offsets chosen once, then
  // load(j) issues wave-load j of the K tile (j < NK) or of the V^T tile (j >= NK)
  struct CopyJob {
    __amdgpu_buffer_rsrc_t krs, vrs;
    int koff, voff;
    unsigned char* kdst;
    unsigned char* vdst;
  };
  auto copy_job = [&](int tk, int tv, unsigned char* kstage, unsigned char* vstage) {
    CopyJob j;
    const bool kg = tk < n_gt, vg = tv < n_gt;
    j.krs = kg ? krs_g : krs_d;
    j.vrs = vg ? vrs_g : vrs_d;
    j.koff = (tk + (kg ? 0 : dshift)) * KBYTES;
    j.voff = (tv + (vg ? 0 : vdshift)) * VBYTES;
    j.kdst = kstage + wv * (Copy::NK * 1024);
    j.vdst = vstage + wv * (Copy::NV * 1024);
    return j;
  };
  auto copy_load = [&](const CopyJob& job, int j) {
    if (j < Copy::NK) copy16_to_lds(job.krs, klo[j], job.koff, job.kdst + j * 1024);
    else copy16_to_lds(job.vrs, vlo[j - Copy::NK], job.voff, job.vdst + (j - Copy::NK) * 1024);
  };

  f32x16_t o[DS];
  float m = -INFINITY, l = 0.f;
#pragma unroll
  for (int sl = 0; sl < DS; ++sl)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[sl][r] = 0.f;

  // per-lane LDS byte offsets of the MFMA fragments inside a tile (the rest is compile-time constant):
  // K fragment (sub, kk) sits at kfa[kk] + sub * 32 rows, V^T fragment (sl, sg) at vfa[sg] + sl * 32 rows;
  // the swizzles depend on the row only through c
  int kfa[KK], vfa[4];
#pragma unroll
  for (int kk = 0; kk < KK; ++kk) kfa[kk] = k_off<D>(c, 2 * kk + hh);
#pragma unroll
  for (int sg = 0; sg < 4; ++sg) vfa[sg] = v_off(c, 2 * sg + hh);

  // S^T = K Q^T for the 64 keys of the tile at kb (two 32-key sub-tiles = two accumulation
  // chains that alternate; fragments read kFragAhead MFMAs ahead); between_pairs(kk) runs after
  // the kk-th pair of MFMAs (the place where the tile copies are issued)
  auto s_tile = [&](const unsigned char* kb, f32x16_t (&s)[2], auto between_pairs) {
    auto kfrag = [&](int i) {
      return *reinterpret_cast<const bf16x8_t*>(kb + kfa[i >> 1] + (i & 1) * (32 * D * 2));
    };
#pragma unroll
    for (int sub = 0; sub < 2; ++sub)
#pragma unroll
      for (int r = 0; r < 16; ++r) s[sub][r] = 0.f;
    bf16x8_t fr[kFragAhead];
#pragma unroll
    for (int i = 0; i < kFragAhead; ++i) fr[i] = kfrag(i);
#pragma unroll
    for (int i = 0; i < 2 * KK; ++i) {
      const int sub = i & 1, kk = i >> 1;
      s[sub] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[i % kFragAhead], qf[kk], s[sub], 0, 0, 0);
      if (i + kFragAhead < 2 * KK) fr[i % kFragAhead] = kfrag(i + kFragAhead);
      if (sub == 1) between_pairs(kk);
    }
  };

  // maximum over the 32 scores a lane holds of its query, then over the two lanes of the query
  auto lane_max = [&](const f32x16_t (&s)[2]) {
    float m8[8];
#pragma unroll
    for (int r = 0; r < 8; ++r) m8[r] = fmaxf(fmaxf(s[0][r], s[0][r + 8]), fmaxf(s[1][r], s[1][r + 8]));
    return half_max(fmaxf(fmaxf(fmaxf(m8[0], m8[1]), fmaxf(m8[2], m8[3])), fmaxf(fmaxf(m8[4], m8[5]), fmaxf(m8[6], m8[7]))));
  };

  // One pipeline step: tile `it` (scores in sc, their unmasked maximum in mx_pre) goes through softmax
  // and P V; the scores of tile it+1 go to sn, and their maximum is taken under the P V MFMAs.
  auto step = [&](int it, f32x16_t (&sc)[2], f32x16_t (&sn)[2], float& mx_pre) {
    // the loads issued during the previous step (K(it+1), V^T(it)) have landed for this wave; after the
    // barrier for every wave, and every wave is done reading K(it) and V^T(it-1)
    __builtin_amdgcn_s_waitcnt(0x0F70);           // vmcnt(0)
    __syncthreads();
    const int tk = it + 2 < last ? it + 2 : last, tv = it + 1 < last ? it + 1 : last;   // past the end: a harmless reload
    const CopyJob job = copy_job(tk, tv, kring + (it & 1) * KBYTES, vring + ((it + 1) & 1) * VBYTES);
    const unsigned char* kb = kring + ((it + 1) & 1) * KBYTES;
    const unsigned char* vb = vring + (it & 1) * VBYTES;
    const bool is_glob = it < n_gt;
    const int key0 = (it + (is_glob ? 0 : dshift)) * kBN;

    // ---- mask of tile `it` (boundary tiles only; a tile this wave sees nothing of is fully masked)
    const bool masked = is_glob ? (key0 + kBN > nv_wave_lo)
                                : !(key0 + kBN - 1 <= wave_first && key0 > wave_last - w);
    float mx = mx_pre;
    if (masked) {
      // visible <=> lo <= key - key0 < hi, with one unsigned compare per element
      int lo, hi;
      if (is_glob) {
        lo = 0;
        hi = nvis - key0 < kBN ? nvis - key0 : kBN;
      } else {
        const int l32 = qpos - w + 1 - key0, h32 = qpos + 1 - key0;
        lo = l32 < 0 ? 0 : (l32 > kBN ? kBN : l32);
        hi = h32 < 0 ? 0 : (h32 > kBN ? kBN : h32);
      }
      const unsigned span = hi > lo ? (unsigned)(hi - lo) : 0u;
      const int rel0 = 4 * hh - lo;
#pragma unroll
      for (int sub = 0; sub < 2; ++sub)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const unsigned kr = (unsigned)(rel0 + sub * 32 + 8 * (r >> 2) + (r & 3));
          sc[sub][r] = kr < span ? sc[sub][r] : -INFINITY;
        }
      mx = lane_max(sc);
    }

    // ---- running maximum of the query (lane column); rescale only when some lane's maximum moved
    const float m_new = fmaxf(m, mx);
    if (__any(m_new > m)) {
      const float alpha = (m_new > m) ? __builtin_amdgcn_exp2f((m - m_new) * sl2e) : 1.f;
      l *= alpha;
#pragma unroll
      for (int sl = 0; sl < DS; ++sl)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[sl][r] *= alpha;
      m = m_new;
    }
    const float mb = (m_new == -INFINITY) ? 0.f : m_new * sl2e;

    // ---- scores of the next tile (MFMA) under the exponentials of this one (VALU)
    s_tile(kb, sn, [&](int kk) {       // copies spread as evenly as the counts allow: load j after pair j * KK / N
      if ((kk * Copy::N) % KK == 0 && kk * Copy::N / KK < Copy::N) copy_load(job, kk * Copy::N / KK);
    });
    bf16x8_t pf[2][2];
    float ls[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int sub = 0; sub < 2; ++sub)
#pragma unroll
      for (int g = 0; g < 2; ++g) {
        bf16x8_t pk;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float p = __builtin_amdgcn_exp2f(fmaf(sc[sub][8 * g + e], sl2e, -mb));
          ls[e & 3] += p;
          pk[e] = (__bf16)p;
        }
        pf[sub][g] = pk;
      }
    l += (ls[0] + ls[1]) + (ls[2] + ls[3]);

    // ---- O^T += V^T P^T: the DS accumulation chains alternate; V^T fragments are read ahead
    auto vfrag = [&](int j) {
      return *reinterpret_cast<const bf16x8_t*>(vb + vfa[j / DS] + (j % DS) * (32 * kBN * 2));
    };
    bf16x8_t vfr[kFragAhead];
#pragma unroll
    for (int j = 0; j < kFragAhead; ++j) vfr[j] = vfrag(j);
#pragma unroll
    for (int j = 0; j < 4 * DS; ++j) {
      const int sl = j % DS, sg = j / DS;           // sg = sub*2 + g: 16 keys
      o[sl] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vfr[j % kFragAhead], pf[sg >> 1][sg & 1], o[sl], 0, 0, 0);
      if (j + kFragAhead < 4 * DS) vfr[j % kFragAhead] = vfrag(j + kFragAhead);
    }
    mx_pre = lane_max(sn);              // vector ALU work for the shadow of the MFMAs above
  };

  // ---- prologue: K(0), V^T(0) in; S(0) computed while K(1) comes in
  f32x16_t sa[2], sb[2];
  {
    const CopyJob first = copy_job(0, 0, kring, vring);
#pragma unroll
    for (int j = 0; j < Copy::N; ++j) copy_load(first, j);
    __builtin_amdgcn_s_waitcnt(0x0F70);
    __syncthreads();
    const int t1 = last < 1 ? last : 1;
    const CopyJob second = copy_job(t1, t1, kring + KBYTES, vring + VBYTES);
    s_tile(kring, sa, [&](int kk) {     // K(1) only; V^T(1) is step 0's load
      if (kk < Copy::NK) copy_load(second, kk);
    });
  }
  float mx_pre = lane_max(sa);
  for (int it = 0; it < n_tiles; it += 2) {
    step(it, sa, sb, mx_pre);
    if (it + 1 < n_tiles) step(it + 1, sb, sa, mx_pre);
  }
  __builtin_amdgcn_s_waitcnt(0x0F70);             // no copy into this workgroup's LDS may outlive it
  if (tid == 0) {                                 // elapsed shader-clock cycles and 100 MHz ticks of this workgroup
    atomicAdd(clk, (unsigned long long)__builtin_readcyclecounter() - clk_c0);
    atomicAdd(clk + 1, (unsigned long long)__builtin_amdgcn_s_memrealtime() - clk_r0);
  }

  // ---- normalise and store
  {
    const int64_t r = r0 + wv * 32 + c;
    const float lt = half_sum(l);
    if (r <= last_row) {
      const float inv = 1.f / lt;
      uint16_t* orow = O + ((size_t)h * n_queries + r) * D;
#pragma unroll
      for (int sl = 0; sl < DS; ++sl)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          bf16x4_t pk;
#pragma unroll
          for (int j = 0; j < 4; ++j) pk[j] = (__bf16)(o[sl][4 * q4 + j] * inv);
          *reinterpret_cast<bf16x4_t*>(orow + sl * 32 + 8 * q4 + 4 * hh) = pk;
        }
      if (lse && hh == 0) lse[(size_t)h * n_queries + r] = m * scale + __logf(lt);
    }
  }
}

// ------------------------------------------------------------------ host side --
struct MfmaWs {
  unsigned long long* clk;   // {sum of workgroup shader-clock cycles, sum of workgroup 100 MHz ticks} of the last call
  uint16_t* Vgt;       // [g_tiles][D][64]
  uint16_t* Vt;        // [Hkv][dense_tiles][D][64]
  size_t bytes;
};

static int64_t max_region_tiles(int Hq, int64_t cap_rows) { return (cap_rows + kBN - 1) / kBN + Hq; }
static int64_t max_dense_tiles(int64_t n_queries, int w) { return (n_queries + w) / kBN + 2; }

static MfmaWs carve_mfma_ws(void* ws, const tca_params* prm, int64_t g_tiles, int64_t d_tiles) {
  MfmaWs m;
  char* b = (char*)ws;
  size_t off = 0;
  const size_t tile_bytes = (size_t)prm->head_dim * kBN * 2;
  m.clk = (unsigned long long*)(b + off); off = align_up(off + 2 * sizeof(unsigned long long), 256);
  m.Vgt = (uint16_t*)(b + off); off = align_up(off + (size_t)g_tiles * tile_bytes, 256);
  m.Vt = (uint16_t*)(b + off);  off = align_up(off + (size_t)prm->n_kv_heads * d_tiles * tile_bytes, 256);
  m.bytes = off;
  return m;
}

size_t prefill_mfma_workspace_bytes(const tca_params* prm, int64_t n_queries, int64_t cap_rows) {
  return carve_mfma_ws(nullptr, prm, max_region_tiles(sel_heads(prm), cap_rows),
                       max_dense_tiles(n_queries, prm->window)).bytes;
}

template <int D>
static void run_mfma(const tca_params* prm, const uint16_t* Q, int64_t q_pos0, int64_t n_queries,
                     const uint16_t* K, const uint16_t* V, int64_t kv_stride, const int32_t* idx,
                     const uint16_t* Kg, const uint16_t* Vg, const int64_t* offs, const int32_t* n_rows,
                     uint16_t* O, float* lse, void* ws, hipStream_t st) {
  const int Hq = prm->n_q_heads, Hkv = prm->n_kv_heads, Hs = sel_heads(prm), w = prm->window;
  PrefillHeads ph;
  int32_t run = 0;
  int max_tiles = 0;
  for (int h = 0; h < Hs; ++h) {
    ph.offs[h] = offs[h];
    ph.tile_off[h] = run;
    const int nt = (int)((offs[h + 1] - offs[h] + kBN - 1) / kBN);
    run += nt;
    if (nt > max_tiles) max_tiles = nt;
  }
  ph.offs[Hs] = offs[Hs];
  ph.tile_off[Hs] = run;
  const int64_t win_lo = q_pos0 - w + 1 > 0 ? q_pos0 - w + 1 : 0;
  const int64_t dt0 = win_lo / kBN, dt1 = (q_pos0 + n_queries - 1) / kBN;
  const int d_tiles = (int)(dt1 - dt0 + 1);
  MfmaWs mw = carve_mfma_ws(ws, prm, max_region_tiles(Hs, offs[Hs]), max_dense_tiles(n_queries, w));

  if (max_tiles > 0)
    hipLaunchKernelGGL((transpose_tiles_kernel<D>), dim3(max_tiles, Hs), dim3(256), 0, st, Vg, (int64_t)0,
                       n_rows, (int64_t)0, (int64_t)0, mw.Vgt, 0, ph, 0, (unsigned long long*)nullptr);
  hipLaunchKernelGGL((transpose_tiles_kernel<D>), dim3(d_tiles, Hkv), dim3(256), 0, st, V, kv_stride,
                     (const int32_t*)nullptr, q_pos0 + n_queries, dt0 * kBN, mw.Vt, d_tiles, ph, 1, mw.clk);

  // Wavefronts per workgroup.  Eight (256 queries, one workgroup per CU) halve the tile copies per
  // query; the board is power-limited under this kernel and the lighter L2 -> LDS traffic lets it
  // clock about 10 % higher.  Four (128 queries, two workgroups per CU) keep the chip full when
  // there are few query tiles.
  auto launch = [&](auto nw_tag) {
    constexpr int NW = decltype(nw_tag)::value;
    const int n_qt = (int)((n_queries + NW * 32 - 1) / (NW * 32));
    hipLaunchKernelGGL((prefill_mfma_kernel<D, NW>), dim3((unsigned)n_qt * Hq), dim3(NW * 64), 0, st, Q,
                       q_pos0, n_queries, K, kv_stride, idx, Kg, n_rows, mw.Vgt, mw.Vt, dt0, d_tiles, ph, Hq,
                       Hq / Hkv, sel_group(prm), w, (float)logit_scale(prm), O, lse, mw.clk);
  };
  if (((n_queries + 255) / 256) * Hq >= 1024) launch(std::integral_constant<int, 8>{});
  else launch(std::integral_constant<int, 4>{});
}

int launch_prefill_mfma(const tca_params* prm, const bf16_t* Q, int64_t q_pos0, int64_t n_queries,
                        const bf16_t* K, const bf16_t* V, int64_t kv_stride, const int32_t* idx,
                        const bf16_t* Kg, const bf16_t* Vg, const int64_t* offs, const int32_t* n_rows,
                        bf16_t* O, float* lse, void* ws, hipStream_t st) {
  // the kernel addresses tiles with 32-bit byte offsets inside each buffer
  const int64_t row_bytes = (int64_t)prm->head_dim * 2;
  int64_t max_rows = q_pos0 + n_queries + prm->window + 2 * kBN;
  for (int h = 0; h < sel_heads(prm); ++h)
    if (offs[h + 1] - offs[h] + kBN > max_rows) max_rows = offs[h + 1] - offs[h] + kBN;
  if (max_rows * row_bytes > (int64_t)INT32_MAX)
    return fail(TCA_ERR_UNSUPPORTED, "tca_prefill (bf16): %lld rows of %lld bytes exceed 2 GiB per head buffer",
                (long long)max_rows, (long long)row_bytes);
  auto u = [](const bf16_t* p) { return reinterpret_cast<const uint16_t*>(p); };
  if (prm->head_dim == 128)
    run_mfma<128>(prm, u(Q), q_pos0, n_queries, u(K), u(V), kv_stride, idx, u(Kg), u(Vg), offs, n_rows,
                  reinterpret_cast<uint16_t*>(O), lse, ws, st);
  else
    run_mfma<64>(prm, u(Q), q_pos0, n_queries, u(K), u(V), kv_stride, idx, u(Kg), u(Vg), offs, n_rows,
                 reinterpret_cast<uint16_t*>(O), lse, ws, st);
  return TCA_OK;
}

}  // namespace tca
