// bf16 MFMA flash-attention prefill over the global and local subsets (Eq. 2;
// Alg. 2 line 7) for gfx950.
//
// Work decomposition.  One workgroup = NW wavefronts = one tile of BM = 32 NW
// consecutive queries of one query head; wave v owns 32 of them (NW = 8, 256
// queries, for long calls; NW = 4 when a call has few query tiles).  The
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
// LDS holds a ring of K tiles [64][D] and a ring of V^T tiles [D][64] (two tiles each; three
// in the two-blocks-per-wave shape) with XOR-swizzled 16-byte chunks (conflict-free b128
// reads without padding), filled by direct global -> LDS loads.  The loop is
// software-pipelined by one tile (see the kernel); one barrier per tile.
//
// Softmax bookkeeping.  One block per wave (the shapes the library launches by itself): the
// reference m of a query's exponentials is the running maximum of its visible scores; the
// state is rescaled, before a tile's exponentials, only when some query's maximum moved.
// Two blocks per wave (a diagnostic shape): the reference is lazy - any earlier maximum of
// visible scores, raised only when a tile's terms would come near the top of the fp32 range
// (row sum of the tile >= kRaise); terms, sum and accumulators share the reference, so the
// quotient is the same, and the common tile needs no maximum at all.
#include <hip/hip_runtime.h>

#include <type_traits>
#include <vector>

#include "tca_prefill.h"

namespace tca {
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4_t;
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));

constexpr int kBN = 64;              // keys per tile
constexpr int kFragAhead = 4;        // LDS fragment reads in flight ahead of the MFMA that uses them
constexpr float kRaise = 0x1p60f;    // a tile whose terms sum to this much raises the softmax reference

struct PrefillHeads {
  int64_t offs[TCA_MAX_HEADS + 1];      // row offsets of the heads' regions
  int32_t tile_off[TCA_MAX_HEADS + 1];  // V^T tile offsets of the heads' regions
  int32_t xcd_start[9];                 // the range of the (head, query tile) sequence each XCD works through
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
    PrefillHeads ph, int mode, unsigned long long* clk, const int32_t* __restrict__ gather_idx, int sel_per_kv) {
  // mode 0: global regions (group = selection head; rows from ph.offs, valid rows from group_valid).
  //         gather_idx != NULL: src is the dense [KV head][group_stride_rows][D] matrix and row r of the
  //         region is its row gather_idx[ph.offs[g] + r] of KV head g / sel_per_kv (no compacted copy exists)
  // mode 1: dense K/V (group = KV head; absolute rows first_row + 64*tile, valid while < valid_all)
  __shared__ uint16_t tile[kBN][D + 8];
  const int g = blockIdx.y, t = blockIdx.x, tid = threadIdx.x;
  if (clk && g == 0 && t == 0 && tid < 4) clk[tid] = 0;      // the attention kernel that follows accumulates here
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
    if (r < n_valid) {
      size_t row = (size_t)(row0 + r);
      if (mode == 0 && gather_idx) row = (size_t)(g / sel_per_kv) * group_stride_rows + gather_idx[row0 + r];
      v = *reinterpret_cast<const uint4*>(src + row * D + part * 8);
    }
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

// The same count for a bound all 64 lanes share, found by the wave together: every round probes 64
// evenly spaced elements of the remaining range at once, so 2^18 elements take three dependent loads
// instead of eighteen.  n, bound: wave-uniform; the result is uniform as well.
__device__ __forceinline__ int count_le_wave(const int32_t* idx, int n, int64_t bound, int lane) {
  int lo = 0, len = n;                               // the count lies in [lo, lo + len]
  while (len > 0) {
    const int step = (len + 63) >> 6;
    const int p = lo + (lane + 1) * step - 1;        // ascending probes: the lanes that pass form a prefix
    const bool le = p < lo + len && (int64_t)idx[p] <= bound;
    const int k = __builtin_popcountll(__ballot(le));
    lo += k * step;
    const int left = n - lo;                         // elements from lo to the end of the array
    len = k == 64 ? 0 : (step - 1 < left ? step - 1 : left);
    if (k == 64) lo = lo < n ? lo : n;
  }
  return lo;
}

// O^T += V^T P^T step.  With two query blocks per wave the O^T accumulators (128 registers for
// d = 128) are pinned to the accumulation registers, which only the matrix pipe touches, so that
// the scores and the exponentials' terms keep the vector registers.  The instruction is written
// out because the register file of an operand cannot be chosen through the builtin; what the
// compiler then cannot see is that o is being written for 8 passes after issue: every vector
// ALU read of o goes through settle_acc() first.
template <bool ACC>
__device__ __forceinline__ void pv_mfma(f32x16_t& o, const bf16x8_t& a, const bf16x8_t& b) {
  if constexpr (ACC) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(o) : "v"(a), "v"(b));
  else o = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, o, 0, 0, 0);
}
// S^T = K Q^T steps for two query blocks per wave: scores in vector registers, Q fragments in
// accumulation registers.  FIRST starts a chain from zero.
template <bool FIRST>
__device__ __forceinline__ void s_mfma(f32x16_t& s, const bf16x8_t& k, const bf16x8_t& q) {
  if constexpr (FIRST) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(s) : "v"(k), "a"(q));
  else asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(s) : "v"(k), "a"(q));
}
// The last step of the four chains of a tile (two blocks x two 32-key sub-tiles), followed by the
// wait states the vector ALU needs before it may touch their results (19 at most; the compiler
// inserts them for the builtin, not for a written-out instruction).
__device__ __forceinline__ void s_mfma_last(f32x16_t& s00, f32x16_t& s10, f32x16_t& s01, f32x16_t& s11,
                                            const bf16x8_t& k0, const bf16x8_t& k1, const bf16x8_t& q0,
                                            const bf16x8_t& q1) {
  asm volatile(
      "v_mfma_f32_32x32x16_bf16 %0, %4, %6, %0\n\t"
      "v_mfma_f32_32x32x16_bf16 %1, %4, %7, %1\n\t"
      "v_mfma_f32_32x32x16_bf16 %2, %5, %6, %2\n\t"
      "v_mfma_f32_32x32x16_bf16 %3, %5, %7, %3\n\t"
      "s_nop 15\n\ts_nop 7"
      : "+v"(s00), "+v"(s10), "+v"(s01), "+v"(s11)
      : "v"(k0), "v"(k1), "a"(q0), "a"(q1));
}
// Marks the accumulators as living in the accumulation registers at this point (no instruction):
// placed after every vector-ALU update of o, so that the value the loop carries has one home and
// is not shuttled between the two register files on every iteration.
template <int N>
__device__ __forceinline__ void home_acc(f32x16_t (&o)[N]) {
#pragma unroll
  for (int i = 0; i < N; ++i) asm volatile("" : "+a"(o[i]));
}
// Waits out the matrix pipe's pending writes to accumulators before the vector ALU reads them.
template <int N>
__device__ __forceinline__ void settle_acc(f32x16_t (&o)[N]) {
  static_assert(N == 2 || N == 4, "one statement per supported slice count");
  if constexpr (N == 4)
    asm volatile("s_nop 15\n\ts_nop 7" : "+a"(o[0]), "+a"(o[1]), "+a"(o[2]), "+a"(o[3]));
  else
    asm volatile("s_nop 15\n\ts_nop 7" : "+a"(o[0]), "+a"(o[1]));
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
// n_gt tiles of the head's compacted region, then the dense tiles of the window).  A wave
// owns QB blocks of 32 queries.  With QB = 1, iteration t is
//   slot A :  S(t+1) = K(t+1) Q^T          (MFMA)  }  one basic block: the MFMAs of the next
//             P(t)   = exp step on S(t)    (VALU)  }  tile run under this tile's exponentials
//   slot B :  O     += V(t)^T P(t)         (MFMA)
// With QB = 2 every K / V^T fragment read from LDS feeds two MFMAs (one per block; the LDS
// port moves 128 bytes per clock and CU, which with one fragment per MFMA is as much of a
// limit as the matrix pipe itself), the wave has a SIMD to itself (512 registers), and the
// second block's softmax runs half an iteration late so that both slots pair 32 MFMAs with
// one block's exponentials, neither depending on the other:
//   slot A :  S_a(t+1), S_b(t+1)           (MFMA)  |  P_a(t)   from S_a(t)     (VALU)
//   slot B :  O_a += V(t)^T P_a(t), O_b += V(t)^T P_b(t)  |  P_b(t+1) from S_b(t+1)
// K(t+RING) and V^T(t+RING-1) are copied global -> LDS during iteration t, into the places
// of K(t) and V^T(t-1); the rings hold RING = 2 or 3 tiles each; one barrier per iteration.
// Positions and byte offsets are 32-bit here: the host checks (q_pos0 + n_queries) * D * 2 < 2^31.
// GATHER: no compacted K exists; the K rows of a region tile are fetched from the dense K through
// idx (the position of every row is read one iteration ahead and becomes the lane's offset of the
// tile copy); the V^T tiles were built through idx by the pre-pass.
template <int D, int NW, int QB, bool GATHER>
__global__ __launch_bounds__(NW * 64) __attribute__((amdgpu_waves_per_eu(2 / QB, 2 / QB)))
void prefill_mfma_kernel(
    const uint16_t* __restrict__ Q, int64_t q_pos0, int64_t n_queries, const uint16_t* __restrict__ K,
    int64_t kv_stride, const int32_t* __restrict__ idx, const uint16_t* __restrict__ Kg,
    const int32_t* __restrict__ n_rows, const uint16_t* __restrict__ Vgt, const uint16_t* __restrict__ Vt,
    int64_t dense_tile0, int dense_tiles, PrefillHeads ph, int Hq, int G, int GS, int w, float scale,
    uint16_t* __restrict__ O, float* __restrict__ lse, unsigned long long* __restrict__ clk, int part) {
  // part: TCA_PART_ALL, or one of the two key subsets alone (TCA_PART_WINDOW: the dense window;
  // TCA_PART_GLOBAL: the region), each normalised by itself, to be merged through lse
  constexpr int KK = D / 16;             // MFMA k-steps over the head dimension
  constexpr int DS = D / 32;             // 32-row slices of O^T
  constexpr int WQ = QB * 32;            // queries per wave
  constexpr int BM = NW * WQ;            // queries per workgroup
  const unsigned long long clk_c0 = __builtin_readcyclecounter(), clk_r0 = __builtin_amdgcn_s_memrealtime();
  constexpr int KBYTES = kBN * D * 2;    // K tile
  constexpr int VBYTES = D * kBN * 2;    // V^T tile
  // Rows are not padded; the 16-byte chunk index is XOR-swizzled with the row so that
  // the b128 reads of 16 consecutive rows at one chunk column fall into distinct banks.
  // Tiles in flight: rings of two K and two V^T tiles, a copy has one iteration to arrive (with two
  // waves per SIMD a third tile measured no faster); the one-wave-per-SIMD shape, where nothing else
  // covers a late copy, keeps three.
  constexpr int RING = QB == 2 ? 3 : 2;
  __shared__ __attribute__((aligned(16))) unsigned char lds[RING * (KBYTES + VBYTES)];
  unsigned char* const kring = lds;
  unsigned char* const vring = lds + RING * KBYTES;

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
  // Heads differ in the rows they keep, so whole heads per XCD leave the XCDs unevenly loaded: the
  // sequence (head-major, a head's query tiles longest first) is cut instead into eight ranges of equal
  // estimated work (xcd_start, from the host).  An XCD takes the piece of the head its range ends in
  // first (that head's longest tiles) and the rest in order, so that it ends on a head's shortest tiles.
  int h, qtile;
  if ((Hq & 7) == 0) {
    const int x = bid & 7, u = bid >> 3;           // XCD, position in the XCD's own sequence
    const int s = ph.xcd_start[x], e = ph.xcd_start[x + 1];
    if (u >= e - s) return;                        // the grid is sized for the longest range
    const int he = e / n_qt * n_qt;                // where the head begins in which the range ends
    const int len_e = he > s ? e - he : 0;
    const int g = u < len_e ? he + u : s + (u - len_e);
    h = g / n_qt;
    qtile = n_qt - 1 - g % n_qt;
  } else {
    h = bid % Hq;
    qtile = n_qt - 1 - bid / Hq;
  }
  const int kvh = h / G;
  const int64_t r0 = (int64_t)qtile * BM;          // first query row of the workgroup
  const int64_t last_row = n_queries - 1;
  const float sl2e = scale * 1.4426950408889634f;

  // ---- per-lane query state (lane column c = one query of each block)
  const int hs = h / GS;                           // the selection this query head reads (GS query heads share it)
  const int64_t base = ph.offs[hs];
  const int nr = part == TCA_PART_WINDOW ? 0 : n_rows[hs];     // without the region nothing below sees a global row
  int qpos[QB], nvis[QB];
  bf16x8_t qf[QB][KK];
#pragma unroll
  for (int blk = 0; blk < QB; ++blk) {
    int64_t qrow_i = r0 + wv * WQ + blk * 32 + c;
    if (qrow_i > last_row) qrow_i = last_row;       // clamped rows compute a duplicate; never stored
    qpos[blk] = (int)(q_pos0 + qrow_i);
    const uint16_t* qrow = Q + ((size_t)h * n_queries + qrow_i) * D;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) qf[blk][kk] = *reinterpret_cast<const bf16x8_t*>(qrow + kk * 16 + hh * 8);
  }
  // wave-level visibility bounds (queries ascend with block and lane column; clamped rows repeat the last)
  const int wave_first = (int)(q_pos0 + i64min(r0 + wv * WQ, last_row));
  const int wave_last = (int)(q_pos0 + i64min(r0 + wv * WQ + WQ - 1, last_row));
  const int wg_last = (int)(q_pos0 + i64min(r0 + BM - 1, last_row));
  const int wg_first = (int)(q_pos0 + r0);
  const int last_pos = (int)(q_pos0 + last_row);
  // Global rows visible to every query of the wave, to some query of the workgroup: two searches with
  // wave-uniform bounds, done by the wave together (a workgroup has the CU to itself, so what its
  // prologue waits for is lost; a binary search per lane was 17 dependent loads).  A lane's own count
  // follows from the first: its query lies at most WQ - 1 positions behind the wave's first one, and
  // positions are distinct and ascending, so only the next WQ rows can make the difference.
  const int nv_wave_lo = __builtin_amdgcn_readfirstlane(count_le_wave(idx + base, nr, (int64_t)wave_first - w, lane));
  const int nv_wg_hi = __builtin_amdgcn_readfirstlane(count_le_wave(idx + base, nr, (int64_t)wg_last - w, lane));
  {
    const int nxt = nv_wave_lo + lane < nr ? idx[base + nv_wave_lo + lane] : 0x7FFFFFFF;   // lane j: row nv_wave_lo + j
#pragma unroll
    for (int blk = 0; blk < QB; ++blk) nvis[blk] = nv_wave_lo;
#pragma unroll
    for (int j = 0; j < WQ - 1; ++j) {
      const int pj = __builtin_amdgcn_readlane(nxt, j);
#pragma unroll
      for (int blk = 0; blk < QB; ++blk) nvis[blk] += (int64_t)pj <= (int64_t)qpos[blk] - w;
    }
  }
  const int n_gt = (nv_wg_hi + kBN - 1) / kBN;
  const int win_lo = wg_first - w + 1 > 0 ? wg_first - w + 1 : 0;
  const int wt0 = win_lo / kBN, wt1 = wg_last / kBN;                      // absolute dense tiles [wt0, wt1]
  const int n_tiles = n_gt + (part == TCA_PART_GLOBAL ? 0 : wt1 - wt0 + 1);
  const int last = n_tiles - 1;
  if (n_tiles == 0) {                              // TCA_PART_GLOBAL with no visible global row: an empty part
#pragma unroll
    for (int blk = 0; blk < QB; ++blk) {
      const int64_t r = r0 + wv * WQ + blk * 32 + c;
      if (r <= last_row) {
        uint16_t* orow = O + ((size_t)h * n_queries + r) * D;
#pragma unroll
        for (int sl = 0; sl < DS; ++sl)
#pragma unroll
          for (int q4 = 0; q4 < 4; ++q4) *reinterpret_cast<uint2*>(orow + sl * 32 + 8 * q4 + 4 * hh) = make_uint2(0u, 0u);
        if (lse && hh == 0) lse[(size_t)h * n_queries + r] = -INFINITY;
      }
    }
    return;
  }
  const int dshift = wt0 - n_gt;                   // tile t >= n_gt is the dense tile t + dshift

  // ---- sources of the tile copies: one descriptor per buffer, the tile chosen by a scalar byte offset
  using Copy = TileCopy<D, NW>;
  constexpr int kRsrcFlags = 0x00020000;           // raw buffer, 32-bit data format
  const __amdgpu_buffer_rsrc_t krs_g = __builtin_amdgcn_make_buffer_rsrc(
      (void*)(GATHER ? K : Kg + (size_t)base * D), 0, GATHER ? 0 : nr * (D * 2), kRsrcFlags);   // GATHER: never read
  const __amdgpu_buffer_rsrc_t krs_d = __builtin_amdgcn_make_buffer_rsrc(
      (void*)(K + (size_t)kvh * kv_stride * D), 0, (last_pos + 1) * (D * 2), kRsrcFlags);
  const __amdgpu_buffer_rsrc_t vrs_g = __builtin_amdgcn_make_buffer_rsrc(
      (void*)(Vgt + (size_t)ph.tile_off[hs] * (D * kBN)), 0, n_gt * VBYTES, kRsrcFlags);
  const __amdgpu_buffer_rsrc_t vrs_d = __builtin_amdgcn_make_buffer_rsrc(
      (void*)(Vt + (size_t)kvh * dense_tiles * (D * kBN)), 0, dense_tiles * VBYTES, kRsrcFlags);
  const int vdshift = dshift - (int)dense_tile0;   // tile t >= n_gt is tile t + vdshift of the dense V^T buffer
  int klo[Copy::NK], vlo[Copy::NV];                // this lane's byte offsets inside a tile, per wave-load
  int krow[Copy::NK];                              // the tile row this lane copies a chunk of, per K wave-load
#pragma unroll
  for (int j = 0; j < Copy::NK; ++j) {
    klo[j] = Copy::k_lane_offset(wv * Copy::NK + j, lane);
    krow[j] = ((wv * Copy::NK + j) * 64 + lane) / Copy::CPR;
  }
#pragma unroll
  for (int j = 0; j < Copy::NV; ++j) vlo[j] = Copy::v_lane_offset(wv * Copy::NV + j, lane);
  // One K tile and one V^T tile to copy: descriptors and scalar offsets chosen once, then
  // load(j) issues wave-load j of the K tile (j < NK) or of the V^T tile (j >= NK)
  struct CopyJob {
    __amdgpu_buffer_rsrc_t krs, vrs;
    int koff, voff;
    unsigned char* kdst;
    unsigned char* vdst;
    bool k_through_idx;              // GATHER: a region tile, its rows fetched from the dense K
    int kgo[Copy::NK];               // GATHER: this lane's byte offset into the dense K, per wave-load
  };
  // GATHER: positions of the rows this lane copies from region tile t (rows past the region's end get
  // an offset beyond the buffer, which the descriptor's range check turns into zeros)
  struct TileRows { int pos[Copy::NK]; };
  auto load_tile_rows = [&](int t) {
    TileRows tr;
#pragma unroll
    for (int j = 0; j < Copy::NK; ++j) {
      const int r = t * kBN + krow[j];
      tr.pos[j] = (t < n_gt && r < nr) ? idx[base + r] : -1;
    }
    return tr;
  };
  auto copy_job = [&](int tk, int tv, unsigned char* kstage, unsigned char* vstage, const TileRows& rows_k) {
    CopyJob j;
    const bool kg = tk < n_gt, vg = tv < n_gt;
    j.krs = (kg && !GATHER) ? krs_g : krs_d;
    j.vrs = vg ? vrs_g : vrs_d;
    j.koff = (tk + (kg ? 0 : dshift)) * KBYTES;
    j.voff = (tv + (vg ? 0 : vdshift)) * VBYTES;
    j.kdst = kstage + wv * (Copy::NK * 1024);
    j.vdst = vstage + wv * (Copy::NV * 1024);
    j.k_through_idx = GATHER && kg;
    if constexpr (GATHER) {
#pragma unroll
      for (int q = 0; q < Copy::NK; ++q)       // the chunk inside the row stays the swizzled one of klo
        j.kgo[q] = rows_k.pos[q] >= 0 ? rows_k.pos[q] * (D * 2) + (klo[q] - krow[q] * (D * 2)) : 0x7FFFFFF0;
    }
    return j;
  };
  auto copy_load = [&](const CopyJob& job, int j) {
    if (j < Copy::NK) {
      if (GATHER && job.k_through_idx) copy16_to_lds(job.krs, job.kgo[j], 0, job.kdst + j * 1024);
      else copy16_to_lds(job.krs, klo[j], job.koff, job.kdst + j * 1024);
    } else {
      copy16_to_lds(job.vrs, vlo[j - Copy::NK], job.voff, job.vdst + (j - Copy::NK) * 1024);
    }
  };

  f32x16_t o[QB][DS];
  float m[QB], l[QB];
#pragma unroll
  for (int blk = 0; blk < QB; ++blk) {
    m[blk] = -INFINITY;
    l[blk] = 0.f;
#pragma unroll
    for (int sl = 0; sl < DS; ++sl)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[blk][sl][r] = 0.f;
    if constexpr (QB == 2) home_acc(o[blk]);
  }

  // per-lane LDS byte offsets of the MFMA fragments inside a tile (the rest is compile-time constant):
  // K fragment (sub, kk) sits at kfa[kk] + sub * 32 rows, V^T fragment (sl, sg) at vfa[sg] + sl * 32 rows;
  // the swizzles depend on the row only through c
  int kfa[KK], vfa[4];
#pragma unroll
  for (int kk = 0; kk < KK; ++kk) kfa[kk] = k_off<D>(c, 2 * kk + hh);
#pragma unroll
  for (int sg = 0; sg < 4; ++sg) vfa[sg] = v_off(c, 2 * sg + hh);

  // S^T = K Q^T for the 64 keys of the tile at kb and every query block of the wave (two 32-key
  // sub-tiles per block = 2 QB accumulation chains that alternate; fragments read kFragAhead
  // ahead and used once per block); between_pairs(kk) runs after the kk-th pair of fragments
  // (the place where the tile copies are issued)
  auto s_tile = [&](const unsigned char* kb, f32x16_t (&s)[QB][2], auto after_fragment) {
    auto kfrag = [&](int i) {
      return *reinterpret_cast<const bf16x8_t*>(kb + kfa[i >> 1] + (i & 1) * (32 * D * 2));
    };
    bf16x8_t fr[kFragAhead];
#pragma unroll
    for (int i = 0; i < kFragAhead; ++i) fr[i] = kfrag(i);
    if constexpr (QB == 1) {
#pragma unroll
      for (int sub = 0; sub < 2; ++sub)
#pragma unroll
        for (int r = 0; r < 16; ++r) s[0][sub][r] = 0.f;
#pragma unroll
      for (int i = 0; i < 2 * KK; ++i) {
        const int sub = i & 1, kk = i >> 1;
        s[0][sub] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[i % kFragAhead], qf[0][kk], s[0][sub], 0, 0, 0);
        if (i + kFragAhead < 2 * KK) fr[i % kFragAhead] = kfrag(i + kFragAhead);
        after_fragment(i);
      }
    } else {
      // the Q fragments (64 registers for d = 128) sit in the accumulation registers as well; the
      // last MFMA of every chain and the wait for their results share one statement
#pragma unroll
      for (int i = 0; i < 2 * KK - 2; ++i) {
        const int sub = i & 1, kk = i >> 1;
#pragma unroll
        for (int blk = 0; blk < QB; ++blk) {
          if (kk == 0) s_mfma<true>(s[blk][sub], fr[i % kFragAhead], qf[blk][kk]);
          else s_mfma<false>(s[blk][sub], fr[i % kFragAhead], qf[blk][kk]);
        }
        if (i + kFragAhead < 2 * KK) fr[i % kFragAhead] = kfrag(i + kFragAhead);
        after_fragment(i);
      }
      s_mfma_last(s[0][0], s[1][0], s[0][1], s[1][1], fr[(2 * KK - 2) % kFragAhead], fr[(2 * KK - 1) % kFragAhead],
                  qf[0][KK - 1], qf[1][KK - 1]);
      after_fragment(2 * KK - 2);
      after_fragment(2 * KK - 1);
    }
  };

  // maximum over the 32 scores a lane holds of its query, then over the two lanes of the query
  auto lane_max = [&](const f32x16_t (&s)[2]) {
    float m8[8];
#pragma unroll
    for (int r = 0; r < 8; ++r) m8[r] = fmaxf(fmaxf(s[0][r], s[0][r + 8]), fmaxf(s[1][r], s[1][r + 8]));
    return half_max(fmaxf(fmaxf(fmaxf(m8[0], m8[1]), fmaxf(m8[2], m8[3])), fmaxf(fmaxf(m8[4], m8[5]), fmaxf(m8[6], m8[7]))));
  };

  // exponentials of the scores s against the reference mb (already in base-2 units): bf16 terms in
  // operand order, and their sum over the lane's 32 keys.  With the running maximum as reference
  // (QB = 1) the largest term of a query is exactly 1, which bf16 holds exactly, and the sum takes
  // the fp32 terms; summing the bf16-rounded ones instead (one v_dot2_f32_bf16 per pair), so that
  // numerator and denominator carry the same rounding, was measured: 1.2 % slower, and 8.3e-3
  // instead of 9.7e-3 worst error on logits in the hundreds, both far inside the 2e-2 the outputs
  // are held to.  With the lazy reference (QB = 2) the largest term is an arbitrary number whose
  // rounding (2^-9 relative) goes straight into the output of a query that attends to one key:
  // there the sum must take the rounded terms, so that the quotient cancels that rounding.
  auto exp_tile = [&](const f32x16_t (&s)[2], float mb, bf16x8_t (&pf)[2][2]) {
    float ls[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int sub = 0; sub < 2; ++sub)
#pragma unroll
      for (int g = 0; g < 2; ++g) {
        bf16x8_t pk;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float p = __builtin_amdgcn_exp2f(fmaf(s[sub][8 * g + e], sl2e, -mb));
          pk[e] = (__bf16)p;
          ls[e & 3] += QB == 2 ? (float)pk[e] : p;
        }
        pf[sub][g] = pk;
      }
    return (ls[0] + ls[1]) + (ls[2] + ls[3]);
  };

  // The same work cut into NCH pieces for the two-block schedule, where the written-out MFMAs pin
  // the instruction order and the pieces are placed between them by hand: piece i forms the
  // exponentials of elements i*EPC .. i*EPC+EPC-1 and rounds, stores and sums those of piece i-1
  // (one piece later, so that no instruction waits on the exponential it has just issued);
  // piece NCH only finishes piece NCH-1.  ls must start at zero; the tile's sum is ls[0..3] added up.
  constexpr int NCH = 2 * KK;            // = fragments of a K tile = fragments of a V^T tile
  constexpr int EPC = 32 / NCH;          // elements of a lane's 32 per piece: 2 (d = 128) or 4 (d = 64)
  auto exp_piece = [&](int i, const f32x16_t (&s)[2], float mb, bf16x8_t (&pf)[2][2], float (&ls)[4], float (&pend)[EPC]) {
    const bf16x2_t ones = {(__bf16)1.f, (__bf16)1.f};
    if (i >= 1) {
#pragma unroll
      for (int k = 0; k < EPC; k += 2) {                 // the sum takes the rounded terms (see exp_tile)
        const int n = (i - 1) * EPC + k;                 // even element of a pair
        const bf16x2_t pr = {(__bf16)pend[k], (__bf16)pend[k + 1]};
        pf[n >> 4][(n >> 3) & 1][n & 7] = pr[0];
        pf[n >> 4][(n >> 3) & 1][(n & 7) + 1] = pr[1];
        ls[(n >> 1) & 3] = __builtin_amdgcn_fdot2_f32_bf16(pr, ones, ls[(n >> 1) & 3], false);
      }
    }
    if (i < NCH) {
#pragma unroll
      for (int k = 0; k < EPC; ++k) {
        const int n = i * EPC + k;
        pend[k] = __builtin_amdgcn_exp2f(fmaf(s[n >> 4][n & 15], sl2e, -mb));
      }
    }
  };

  // Does every query of the wave see every key of tile t?  (wave-uniform)
  auto mask_tile_is_clear = [&](int t) {
    const bool is_glob = t < n_gt;
    const int key0 = (t + (is_glob ? 0 : dshift)) * kBN;
    return t <= last && (is_glob ? (key0 + kBN <= nv_wave_lo) : (key0 + kBN - 1 <= wave_first && key0 > wave_last - w));
  };
  // Mask of tile t on the scores s of block blk (boundary tiles only; a tile this wave sees nothing
  // of, or past the last one, is fully masked).  Returns whether this lane's query sees any key of it.
  auto mask_tile = [&](int t, int blk, f32x16_t (&s)[2]) {
    const bool is_glob = t < n_gt;
    const int key0 = (t + (is_glob ? 0 : dshift)) * kBN;
    const bool beyond = t > last;
    const bool masked = beyond || (is_glob ? (key0 + kBN > nv_wave_lo)
                                           : !(key0 + kBN - 1 <= wave_first && key0 > wave_last - w));
    bool sees = true;
    if (masked) {
      // visible <=> lo <= key - key0 < hi, with one unsigned compare per element
      int lo, hi;
      if (is_glob) {
        lo = 0;
        hi = nvis[blk] - key0 < kBN ? nvis[blk] - key0 : kBN;
      } else {
        const int l32 = qpos[blk] - w + 1 - key0, h32 = qpos[blk] + 1 - key0;
        lo = l32 < 0 ? 0 : (l32 > kBN ? kBN : l32);
        hi = h32 < 0 ? 0 : (h32 > kBN ? kBN : h32);
      }
      const unsigned span = (hi > lo && !beyond) ? (unsigned)(hi - lo) : 0u;
      sees = span != 0u;
      const int rel0 = 4 * hh - lo;
#pragma unroll
      for (int sub = 0; sub < 2; ++sub)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const unsigned kr = (unsigned)(rel0 + sub * 32 + 8 * (r >> 2) + (r & 3));
          s[sub][r] = kr < span ? s[sub][r] : -INFINITY;
        }
    }
    return sees;
  };

  // The uncommon tile: the query's first visible keys, or terms too large for the reference.
  // The reference becomes the maximum over the visible scores so far (the same in both lanes of
  // a query), the state is rescaled and the tile's terms are formed again.
  auto softmax_fixup = [&](int blk, const f32x16_t (&s)[2], bool cold, bool sees, float& lt, bf16x8_t (&pf)[2][2]) {
    if (__any(lt >= kRaise || (cold && sees))) {
      const float m_new = fmaxf(m[blk], lane_max(s));
      const float alpha = (m_new > m[blk]) ? __builtin_amdgcn_exp2f((m[blk] - m_new) * sl2e) : 1.f;   // 0 when m was -inf
      l[blk] *= alpha;
      if constexpr (QB == 2) settle_acc(o[blk]);
#pragma unroll
      for (int sl = 0; sl < DS; ++sl)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[blk][sl][r] *= alpha;
      if constexpr (QB == 2) home_acc(o[blk]);
      m[blk] = m_new;
      lt = exp_tile(s, (m_new == -INFINITY) ? 0.f : m_new * sl2e, pf);
    }
  };

  bf16x8_t pf[QB][2][2];                 // P of block 0: formed and used inside a step; of block 1: formed one step ahead

  int rpos = 0;                          // it % RING of the step about to run
  float mx_pre = -INFINITY;              // QB = 1: unmasked maximum of the scores the next step starts from
  TileRows rows_ahead = {};              // GATHER: row positions of tile it + RING, read during step it - 1
  static_assert((RING - 2) * Copy::N < 16, "the wait below encodes its count in four bits");

  // One pipeline step: tile `it` (scores in sc; with QB = 2 those of block 1 are already in pf[1])
  // goes through softmax and P V; the scores of tile it+1 go to sn.
  // clear_tag: std::true_type when the caller knows that this wave sees every key of tile `it` (the
  // stretches of the loop below where no tile needs a mask), which saves the test per step
  auto step = [&](int it, f32x16_t (&sc)[QB][2], f32x16_t (&sn)[QB][2], auto clear_tag) {
    constexpr bool kKnownClear = decltype(clear_tag)::value;
    // K(it+1) and V^T(it) have landed for this wave (only the copies of the previous step may still
    // be on their way when the rings hold three tiles); after the barrier for every wave, and every
    // wave is done reading K(it) and V^T(it-1).  With one block per wave this wait and barrier sit
    // inside the previous step, before its last P V MFMAs (see there).
    if constexpr (QB != 1) {
      __builtin_amdgcn_s_waitcnt(0x0F70 | ((RING - 2) * Copy::N));     // vmcnt((RING - 2) * N)
      __syncthreads();
    }
    const int tk = it + RING < last ? it + RING : last, tv = it + RING - 1 < last ? it + RING - 1 : last;   // past the end: a harmless reload
    // ring places (it - 1, it, it + 1) % RING; with two places they follow from the parity of `it`, which the
    // twice-unrolled loop makes a constant of each copy of the step (LDS offsets fold into the instructions)
    const int r_cur = RING == 2 ? (it & 1) : rpos;
    const int r_next = RING == 2 ? ((it + 1) & 1) : (rpos + 1 == RING ? 0 : rpos + 1);
    const int r_prev = RING == 2 ? r_next : (rpos == 0 ? RING - 1 : rpos - 1);
    const CopyJob job = copy_job(tk, tv, kring + r_cur * KBYTES, vring + r_prev * VBYTES, rows_ahead);
    // GATHER: the positions for the copies of the next step are requested before this step's copies,
    // so that the wait at the top of the next step, which lets only the newest copies pass, covers them
    if constexpr (GATHER) rows_ahead = load_tile_rows(it + 1 + RING < last ? it + 1 + RING : last);
    const unsigned char* kb = kring + r_next * KBYTES;
    const unsigned char* vb = vring + r_cur * VBYTES;
    if constexpr (RING != 2) rpos = r_next;

    // ---- slot A: scores of the next tile (MFMA) under the exponentials of this one (VALU), taken
    // against the reference as it stands
    auto issue_copies = [&](int i) {     // copies spread as evenly as the counts allow: load j after fragment pair j * KK / N
      const int kk = i >> 1;
      if ((i & 1) && (kk * Copy::N) % KK == 0 && kk * Copy::N / KK < Copy::N) copy_load(job, kk * Copy::N / KK);
    };
    auto vfrag = [&](int j) {
      return *reinterpret_cast<const bf16x8_t*>(vb + vfa[j / DS] + (j % DS) * (32 * kBN * 2));
    };
    bf16x8_t vfr[kFragAhead];
    if constexpr (QB == 1) {
      // One block per wave, two waves per SIMD: the reference is the running maximum of the visible
      // scores.  The maximum of this tile was taken under the previous step's P V MFMAs (again after
      // masking on a boundary tile); the state is rescaled, before the exponentials, only when some
      // query's maximum moved.  Everything from here to the end of the step is one basic block, so
      // that the first P V MFMAs can start while the later exponentials are still being formed.
      const bool masked = !kKnownClear && !mask_tile_is_clear(it);
      float mx = mx_pre;
      if (masked) {
        mask_tile(it, 0, sc[0]);
        mx = lane_max(sc[0]);
      }
      const float m_new = fmaxf(m[0], mx);
      if (__any(m_new > m[0])) {
        const float alpha = (m_new > m[0]) ? __builtin_amdgcn_exp2f((m[0] - m_new) * sl2e) : 1.f;   // 0 when m was -inf
        l[0] *= alpha;
#pragma unroll
        for (int sl = 0; sl < DS; ++sl)
#pragma unroll
          for (int r = 0; r < 16; ++r) o[0][sl][r] *= alpha;
        m[0] = m_new;
      }
      s_tile(kb, sn, issue_copies);
      l[0] += exp_tile(sc[0], (m_new == -INFINITY) ? 0.f : m_new * sl2e, pf[0]);
    } else {
      const bool sees = mask_tile(it, 0, sc[0]);
      const bool cold = m[0] == -INFINITY;          // no reference yet: no key seen so far
      const float mb = cold ? 0.f : m[0] * sl2e;
      float ls[4] = {0.f, 0.f, 0.f, 0.f}, pend[EPC];
      __builtin_amdgcn_sched_barrier(0);
      s_tile(kb, sn, [&](int i) {
        issue_copies(i);
        exp_piece(i, sc[0], mb, pf[0], ls, pend);
        __builtin_amdgcn_sched_barrier(0);
      });
      exp_piece(NCH, sc[0], mb, pf[0], ls, pend);
      float lt = (ls[0] + ls[1]) + (ls[2] + ls[3]);
      softmax_fixup(0, sc[0], cold, sees, lt, pf[0]);
      l[0] += lt;
    }

    // ---- slot B: O^T += V^T P^T for every block (the accumulation chains alternate; V^T fragments
    // are read ahead and used once per block), under the exponentials of block 1's next tile
    bool sees1 = true, cold1 = false;
    float mb1 = 0.f, ls1[4] = {0.f, 0.f, 0.f, 0.f}, pend1[EPC];
    bf16x8_t pn[2][2];
    if constexpr (QB == 2) {
      sees1 = mask_tile(it + 1, 1, sn[1]);
      cold1 = m[1] == -INFINITY;
      mb1 = cold1 ? 0.f : m[1] * sl2e;
      __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int j = 0; j < kFragAhead; ++j) vfr[j] = vfrag(j);
#pragma unroll
    for (int j = 0; j < 4 * DS; ++j) {
      const int sl = j % DS, sg = j / DS;           // sg = sub*2 + g: 16 keys
      if constexpr (QB == 1) {
        // The barrier of the next step, taken as soon as the last V^T fragment of this tile has been
        // requested (the reads run kFragAhead ahead): the MFMAs still to come work from registers and
        // cover the first fragment reads of the next tile, which cannot start before the barrier.
        if (j == 4 * DS - kFragAhead) {
          __builtin_amdgcn_s_waitcnt(0x0F70);          // this wave's copies of K(it+2), V^T(it+1) have landed
          __syncthreads();
        }
      }
#pragma unroll
      for (int blk = 0; blk < QB; ++blk) pv_mfma<QB == 2>(o[blk][sl], vfr[j % kFragAhead], pf[blk][sg >> 1][sg & 1]);
      if (j + kFragAhead < 4 * DS) vfr[j % kFragAhead] = vfrag(j + kFragAhead);
      if constexpr (QB == 2) {
        exp_piece(j, sn[1], mb1, pn, ls1, pend1);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    if constexpr (QB == 1) mx_pre = lane_max(sn[0]);    // vector ALU work for the shadow of the MFMAs above
    if constexpr (QB == 1) {
      // The order of the step's instructions, spelled out for the scheduler (the step is one scheduling
      // region): behind every MFMA one fragment read and an even share of the plain vector ALU work, the
      // exponentials left to fall where they may, which is two per MFMA of the S half.  Left to itself the
      // scheduler starts the step with eight bare MFMAs and crowds the exponentials into the middle;
      // measured 2 - 2.5 % faster than that (2 .. 6 instructions behind an MFMA of S and 3 .. 6 behind
      // one of P V tried: within 1 % of each other).  Pinning the exponentials or the scalar
      // instructions as well measured 8 % slower.
      constexpr int kMfma = 0x008, kValu = 0x002, kDsRead = 0x100, kVmemRead = 0x020;
      constexpr int VA = 384 / D, VB = 640 / D;        // plain vector ALU instructions behind an MFMA of S, of P V
      __builtin_amdgcn_sched_group_barrier(kDsRead, kFragAhead, 0);
#pragma unroll
      for (int i = 0; i < 2 * KK; ++i) {
        __builtin_amdgcn_sched_group_barrier(kMfma, 1, 0);
        __builtin_amdgcn_sched_group_barrier(kDsRead, 1, 0);
        if ((i & 1) && ((i >> 1) * Copy::N) % KK == 0 && (i >> 1) * Copy::N / KK < Copy::N)
          __builtin_amdgcn_sched_group_barrier(kVmemRead, 1, 0);
        __builtin_amdgcn_sched_group_barrier(kValu, VA, 0);
      }
#pragma unroll
      for (int j = 0; j < 4 * DS; ++j) {
        __builtin_amdgcn_sched_group_barrier(kMfma, 1, 0);
        if (j + kFragAhead < 4 * DS) __builtin_amdgcn_sched_group_barrier(kDsRead, 1, 0);
        __builtin_amdgcn_sched_group_barrier(kValu, VB, 0);
      }
    }
    if constexpr (QB == 2) {
      exp_piece(NCH, sn[1], mb1, pn, ls1, pend1);
      float lt = (ls1[0] + ls1[1]) + (ls1[2] + ls1[3]);
      softmax_fixup(1, sn[1], cold1, sees1, lt, pn);
      l[1] += lt;
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int g = 0; g < 2; ++g) pf[1][a][g] = pn[a][g];
    }
  };

  // ---- prologue: everything the steps do not copy themselves - K(0) .. K(RING-1), V^T(0) ..
  // V^T(RING-2) - is requested here, oldest first; S(0) is formed as soon as K(0) is in
  f32x16_t sa[QB][2], sb[QB][2];
  {
    auto tile_or_last = [&](int t) { return t < last ? t : last; };
    const CopyJob first = copy_job(0, 0, kring, vring, load_tile_rows(0));
#pragma unroll
    for (int j = 0; j < Copy::N; ++j) copy_load(first, j);
    const CopyJob second = copy_job(tile_or_last(1), 0, kring + KBYTES, vring, load_tile_rows(tile_or_last(1)));
#pragma unroll
    for (int j = 0; j < Copy::NK; ++j) copy_load(second, j);
    if constexpr (RING == 3) {
      const CopyJob third = copy_job(tile_or_last(2), tile_or_last(1), kring + 2 * KBYTES, vring + VBYTES,
                                     load_tile_rows(tile_or_last(2)));
#pragma unroll
      for (int j = 0; j < Copy::N; ++j) copy_load(third, j);
    }
    if constexpr (GATHER) rows_ahead = load_tile_rows(tile_or_last(RING));    // for the copies of step 0
    // K(0), V^T(0) are in (GATHER: the positions just requested count among the newest as well)
    __builtin_amdgcn_s_waitcnt(0x0F70 | (Copy::NK + (RING - 2) * Copy::N + (GATHER ? Copy::NK : 0)));
    __syncthreads();
    s_tile(kring, sa, [&](int) {});
    if constexpr (QB == 1) mx_pre = lane_max(sa[0]);
    if constexpr (QB == 2) {            // block 1 runs half a step ahead with its exponentials
      const bool sees = mask_tile(0, 1, sa[1]);
      float lt = exp_tile(sa[1], 0.f, pf[1]);
      softmax_fixup(1, sa[1], true, sees, lt, pf[1]);
      l[1] += lt;
    }
  }
  const unsigned long long clk_loop = __builtin_readcyclecounter();
  if constexpr (QB == 1) {
    __builtin_amdgcn_s_waitcnt(0x0F70);              // K(1) is in: the barrier of step 0 (every later one sits in the step before)
    __syncthreads();
  }
  // (the stretches below pay off with eight waves; with four the scheduler no longer follows the order
  // pinned in the step for the test-free copies of it, and the plain loop is faster)
  if constexpr (QB == 1 && NW == 8) {
    // The tiles this wave sees all of form two stretches: the region tiles below the rows visible to its
    // first query, and the window tiles between its last query's window start and its first query.  Their
    // ends are moved to even steps (a clear tile may always take the masked path), so that every stretch
    // is a run of the twice-unrolled loop.
    const int a0 = nv_wave_lo / kBN;                                         // region tiles [0, a0) are clear
    const int t_lo = wave_last - w < 0 ? 0 : (wave_last - w) / kBN + 1;       // dense tiles [t_lo, t_hi] are clear
    const int t_hi = wave_first - (kBN - 1) < 0 ? -1 : (wave_first - (kBN - 1)) / kBN;
    int b0 = t_lo - dshift, c0 = t_hi + 1 - dshift;                           // as steps: [b0, c0)
    if (b0 < n_gt) b0 = n_gt;
    if (c0 > n_tiles) c0 = n_tiles;
    const int a = a0 & ~1;
    int b = (b0 + 1) & ~1, c = c0 & ~1;
    if (b < a) b = a;
    if (c < b) c = b;
    if (b > n_tiles) b = c = n_tiles & ~1;
    for (int it = 0; it < a; it += 2) {
      step(it, sa, sb, std::true_type{});
      step(it + 1, sb, sa, std::true_type{});
    }
    for (int it = a; it < b; it += 2) {
      step(it, sa, sb, std::false_type{});
      if (it + 1 < n_tiles) step(it + 1, sb, sa, std::false_type{});
    }
    for (int it = b; it < c; it += 2) {
      step(it, sa, sb, std::true_type{});
      step(it + 1, sb, sa, std::true_type{});
    }
    for (int it = c; it < n_tiles; it += 2) {
      step(it, sa, sb, std::false_type{});
      if (it + 1 < n_tiles) step(it + 1, sb, sa, std::false_type{});
    }
  } else {
    for (int it = 0; it < n_tiles; it += 2) {
      step(it, sa, sb, std::false_type{});
      if (it + 1 < n_tiles) step(it + 1, sb, sa, std::false_type{});
    }
  }
  __builtin_amdgcn_s_waitcnt(0x0F70);             // no copy into this workgroup's LDS may outlive it
  if (clk && tid == 0) {                          // diagnostics only: elapsed shader-clock cycles and 100 MHz ticks of this workgroup
    atomicAdd(clk, (unsigned long long)__builtin_readcyclecounter() - clk_c0);
    atomicAdd(clk + 1, (unsigned long long)__builtin_amdgcn_s_memrealtime() - clk_r0);
    atomicAdd(clk + 2, clk_loop - clk_c0);        // of which before the first step
    atomicAdd(clk + 3, (unsigned long long)n_tiles);
  }

  // ---- normalise and store
#pragma unroll
  for (int blk = 0; blk < QB; ++blk) {
    const int64_t r = r0 + wv * WQ + blk * 32 + c;
    const float lt = half_sum(l[blk]);
    if constexpr (QB == 2) settle_acc(o[blk]);
    if (r <= last_row) {
      const float inv = lt > 0.f ? 1.f / lt : 0.f;    // a query that sees nothing of this part: zeros, lse = -inf
      uint16_t* orow = O + ((size_t)h * n_queries + r) * D;
#pragma unroll
      for (int sl = 0; sl < DS; ++sl)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          bf16x4_t pk;
#pragma unroll
          for (int j = 0; j < 4; ++j) pk[j] = (__bf16)(o[blk][sl][4 * q4 + j] * inv);
          *reinterpret_cast<bf16x4_t*>(orow + sl * 32 + 8 * q4 + 4 * hh) = pk;
        }
      if (lse && hh == 0) lse[(size_t)h * n_queries + r] = lt > 0.f ? m[blk] * scale + __logf(lt) : -INFINITY;
    }
  }
}

// ------------------------------------------------------------------ host side --
struct MfmaWs {
  unsigned long long* clk;   // sums over the workgroups of the last call: {shader-clock cycles, 100 MHz ticks, cycles before the first step, tiles}
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
  m.clk = (unsigned long long*)(b + off); off = align_up(off + 4 * sizeof(unsigned long long), 256);
  m.Vgt = (uint16_t*)(b + off); off = align_up(off + (size_t)g_tiles * tile_bytes, 256);
  m.Vt = (uint16_t*)(b + off);  off = align_up(off + (size_t)prm->n_kv_heads * d_tiles * tile_bytes, 256);
  m.bytes = off;
  return m;
}

size_t prefill_mfma_workspace_bytes(const tca_params* prm, int64_t n_queries, int64_t cap_rows) {
  return carve_mfma_ws(nullptr, prm, max_region_tiles(sel_heads(prm), cap_rows),
                       max_dense_tiles(n_queries, prm->window)).bytes;
}

// Chooses the ranges of the (head, query tile) sequence, in the order the kernel walks it, that the eight
// XCDs work through, and returns the length of the longest.  Two candidates: whole heads per XCD, and
// eight ranges of equal estimated work (heads keep different numbers of rows).  The estimate is in tile
// steps: the dense tiles of the window, exactly; the visible part of a head's region as if its rows
// were spread evenly over the positions seen so far (the host does not know idx); a constant for what a
// workgroup does before and after its loop.  Each candidate is played through (`slots` workgroups at a
// time per XCD, the next item to the first free slot) and the one that ends sooner is taken: with few
// long items per slot a range of equal work but one item more than the slots divide costs a whole
// round.  A poor estimate costs balance, never correctness.
static int64_t plan_xcds(PrefillHeads& ph, const tca_params* prm, const int64_t* offs, int64_t q_pos0,
                         int64_t n_queries, int BM, int part, int slots) {
  const int Hq = prm->n_q_heads, GS = sel_group(prm), w = prm->window;
  const int64_t n_qt = (n_queries + BM - 1) / BM, L_end = q_pos0 + n_queries, n_items = Hq * n_qt;
  constexpr int64_t kFixedSteps = 4;
  auto cost = [&](int64_t g) {                     // item g: head g / n_qt, its query tiles longest first
    const int64_t h = g / n_qt, qt = n_qt - 1 - g % n_qt, cap = offs[h / GS + 1] - offs[h / GS];
    const int64_t first = q_pos0 + qt * BM, lastq = first + BM - 1 < L_end - 1 ? first + BM - 1 : L_end - 1;
    int64_t c = kFixedSteps;
    if (part != TCA_PART_GLOBAL) c += lastq / kBN - (first - w + 1 > 0 ? first - w + 1 : 0) / kBN + 1;
    if (part != TCA_PART_WINDOW && lastq >= w) c += (cap * (lastq - w + 1) / L_end + kBN - 1) / kBN;
    return c;
  };
  std::vector<int32_t> c((size_t)n_items);
  int64_t total = 0;
  for (int64_t g = 0; g < n_items; ++g) total += c[g] = (int32_t)cost(g);
  int32_t by_head[9], by_work[9];
  for (int x = 0; x <= 8; ++x) by_head[x] = (int32_t)(x * (Hq / 8) * n_qt);
  int64_t acc = 0;
  int x = 0;
  by_work[0] = 0;
  for (int64_t g = 0; g < n_items; ++g) {
    acc += c[g];
    while (x < 7 && acc * 8 >= total * (x + 1)) by_work[++x] = (int32_t)(g + 1);
  }
  while (x < 8) by_work[++x] = (int32_t)n_items;
  // when the slowest XCD ends, the kernel's own order inside a range: the piece of the head the range ends in first
  auto makespan = [&](const int32_t* st) {
    int64_t worst = 0, free_at[64];
    for (int xc = 0; xc < 8; ++xc) {
      const int64_t s = st[xc], e = st[xc + 1], he = e / n_qt * n_qt, len_e = he > s ? e - he : 0;
      for (int i = 0; i < slots; ++i) free_at[i] = 0;
      for (int64_t u = 0; u < e - s; ++u) {
        int first = 0;
        for (int i = 1; i < slots; ++i)
          if (free_at[i] < free_at[first]) first = i;
        free_at[first] += c[u < len_e ? he + u : s + (u - len_e)];
      }
      for (int i = 0; i < slots; ++i)
        if (free_at[i] > worst) worst = free_at[i];
    }
    return worst;
  };
  // with many rounds per slot the last, shortest items even the ends out and equal work wins
  const bool few_rounds = n_items < (int64_t)8 * slots * 16;
  const int32_t* best = !few_rounds || makespan(by_work) < makespan(by_head) ? by_work : by_head;
  int64_t longest = 0;
  for (x = 0; x <= 8; ++x) ph.xcd_start[x] = best[x];
  for (x = 0; x < 8; ++x)
    if (best[x + 1] - best[x] > longest) longest = best[x + 1] - best[x];
  return longest;
}

// The workgroup shape of a call: waves, and blocks of 32 queries per wave.  The size of the call chooses
// between eight and four waves of 32 queries; the diagnostics switch can force a shape.
struct WgShape { int nw, qb; };
static WgShape choose_shape(const tca_params* prm, int64_t n_queries, bool gather) {
  const int variant = prefill_variant();
  const bool many = ((n_queries + 255) / 256) * prm->n_q_heads >= 1024;
  if (gather) return {variant == 3 || (variant != 1 && many) ? 8 : 4, 1};
  if (variant == 3 || (variant == 0 && many)) return {8, 1};
  if (variant == 2) return {4, 2};
  return {4, 1};
}

template <int D>
static void run_mfma(const tca_params* prm, const uint16_t* Q, int64_t q_pos0, int64_t n_queries,
                     const uint16_t* K, const uint16_t* V, int64_t kv_stride, const int32_t* idx,
                     const uint16_t* Kg, const uint16_t* Vg, const int64_t* offs, const int32_t* n_rows,
                     uint16_t* O, float* lse, void* ws, hipStream_t st, int part) {
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
  // cycle counters only when asked for (and not for a part: two parts may run side by side on one workspace,
  // where the window part touches only the dense V^T tiles and the global part only the regions')
  unsigned long long* clk = diag_prefill_clocks() && part == TCA_PART_ALL ? mw.clk : nullptr;

  // gather-free call (no compacted copy of the kept rows): V^T tiles of the regions are built from the
  // dense V through idx, and the attention kernel fetches the K rows of its region tiles the same way
  const bool gather = Kg == nullptr;
  if (max_tiles > 0 && part != TCA_PART_WINDOW) {
    if (gather)
      hipLaunchKernelGGL((transpose_tiles_kernel<D>), dim3(max_tiles, Hs), dim3(256), 0, st, V, kv_stride, n_rows,
                         (int64_t)0, (int64_t)0, mw.Vgt, 0, ph, 0, (unsigned long long*)nullptr, idx, Hs / Hkv);
    else
      hipLaunchKernelGGL((transpose_tiles_kernel<D>), dim3(max_tiles, Hs), dim3(256), 0, st, Vg, (int64_t)0, n_rows,
                         (int64_t)0, (int64_t)0, mw.Vgt, 0, ph, 0, (unsigned long long*)nullptr,
                         (const int32_t*)nullptr, 1);
  }
  if (part != TCA_PART_GLOBAL)
    hipLaunchKernelGGL((transpose_tiles_kernel<D>), dim3(d_tiles, Hkv), dim3(256), 0, st, V, kv_stride,
                       (const int32_t*)nullptr, q_pos0 + n_queries, dt0 * kBN, mw.Vt, d_tiles, ph, 1, clk,
                       (const int32_t*)nullptr, 1);

  // Shape of a workgroup.  Long calls: eight waves of 32 queries (256 queries, one workgroup per CU,
  // two waves per SIMD).  Calls with few query tiles: four waves of 32 queries
  // (128 queries, two workgroups per CU), which keeps more of the chip busy.  Four waves of 64
  // queries (one wave per SIMD, every LDS fragment feeds two MFMAs, half the LDS reads) stay
  // selectable through the diagnostics switch: measured 5-8 % slower on 128K tokens, because a
  // lone wave cannot issue its vector, LDS and scalar instructions fast enough beside the MFMAs.
  auto launch = [&](auto nw_tag, auto qb_tag, auto gather_tag) {
    constexpr int NW = decltype(nw_tag)::value, QB = decltype(qb_tag)::value;
    constexpr bool GATHER = decltype(gather_tag)::value;
    const int n_qt = (int)((n_queries + NW * QB * 32 - 1) / (NW * QB * 32));
    // workgroups an XCD runs at a time: 32 CUs, one eight-wave workgroup or two four-wave ones each
    const unsigned n_wg = (Hq & 7) == 0 ? 8u * (unsigned)plan_xcds(ph, prm, offs, q_pos0, n_queries, NW * QB * 32, part,
                                                                   NW == 8 || QB == 2 ? 32 : 64)
                                        : (unsigned)n_qt * Hq;
    hipLaunchKernelGGL((prefill_mfma_kernel<D, NW, QB, GATHER>), dim3(n_wg), dim3(NW * 64), 0, st, Q,
                       q_pos0, n_queries, K, kv_stride, idx, Kg, n_rows, mw.Vgt, mw.Vt, dt0, d_tiles, ph, Hq,
                       Hq / Hkv, sel_group(prm), w, (float)logit_scale(prm), O, lse, clk, part);
  };
  using I1 = std::integral_constant<int, 1>;
  using I2 = std::integral_constant<int, 2>;
  using I4 = std::integral_constant<int, 4>;
  using I8 = std::integral_constant<int, 8>;
  const WgShape sh = choose_shape(prm, n_queries, gather);
  if (gather) {
    if (sh.nw == 8) launch(I8{}, I1{}, std::true_type{});
    else launch(I4{}, I1{}, std::true_type{});
  } else if (sh.nw == 8) launch(I8{}, I1{}, std::false_type{});
  else if (sh.qb == 2) launch(I4{}, I2{}, std::false_type{});
  else launch(I4{}, I1{}, std::false_type{});
}

int64_t prefill_mfma_xcd_plan(const tca_params* prm, const int64_t* offs, int64_t q_pos0, int64_t n_queries, int part,
                              bool gather, int32_t* start_out) {
  if ((prm->n_q_heads & 7) != 0) return -1;
  const WgShape sh = choose_shape(prm, n_queries, gather);
  PrefillHeads ph;
  const int64_t longest = plan_xcds(ph, prm, offs, q_pos0, n_queries, sh.nw * sh.qb * 32, part,
                                    sh.nw == 8 || sh.qb == 2 ? 32 : 64);
  for (int x = 0; x <= 8; ++x) start_out[x] = ph.xcd_start[x];
  return 8 * longest;
}

int launch_prefill_mfma(const tca_params* prm, const bf16_t* Q, int64_t q_pos0, int64_t n_queries,
                        const bf16_t* K, const bf16_t* V, int64_t kv_stride, const int32_t* idx,
                        const bf16_t* Kg, const bf16_t* Vg, const int64_t* offs, const int32_t* n_rows,
                        bf16_t* O, float* lse, void* ws, hipStream_t st, int part) {
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
                  reinterpret_cast<uint16_t*>(O), lse, ws, st, part);
  else
    run_mfma<64>(prm, u(Q), q_pos0, n_queries, u(K), u(V), kv_stride, idx, u(Kg), u(Vg), offs, n_rows,
                 reinterpret_cast<uint16_t*>(O), lse, ws, st, part);
  return TCA_OK;
}

}  // namespace tca
