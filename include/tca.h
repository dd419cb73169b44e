/*
 * tca.h - C ABI of the MI355X (gfx950) hot path of TCA-Attention
 * (Training-free Context-adaptive Attention, arxiv 2512.09238).
 *
 * The library implements, for one attention layer on one GPU:
 *   - offline head-specific sparsity determination   (Alg. 1, Eq. 3, Eq. 4)
 *   - online core-context selection                   (Alg. 2 lines 1-6, Eq. 5-8)
 *     followed by compaction of the retained K/V rows (App. C, "parallel tokens gathering")
 *   - causal prefill attention over [K^G; K^L]        (Alg. 2 line 7, Eq. 2)
 *   - single-token decode over the compacted cache,
 *     with selection of each block completed while decoding (Sec. IV-B, last paragraph)
 *
 * Conventions
 *   - "device" pointers are GPU memory owned by the caller; "host" pointers are
 *     ordinary CPU memory owned by the caller.  The library never allocates or
 *     frees device memory.  Scratch comes in through (ws, ws_bytes); query the
 *     size with the matching tca_*_workspace_bytes().  ws must be 256-byte aligned.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     All work is enqueued on it; only tca_calibrate_budgets waits for it.
 *   - Tensors are dense, row-major, innermost dimension head_dim:
 *       Q, O : [n_q_heads , rows, head_dim]
 *       K, V : [n_kv_heads, kv_stride rows, head_dim]  (kv_stride >= rows used)
 *     Element type per tca_params.dtype: TCA_BF16 (bfloat16) or TCA_F32 (float).
 *   - Query head h reads KV head h / (n_q_heads / n_kv_heads).  Every query head
 *     owns its own selection (the method is applied to each head independently, Sec. IV):
 *     there are Hs = n_q_heads "selection heads".  With tca_params.share =
 *     TCA_SHARE_GROUP (an extension for grouped-query attention, not in the paper)
 *     the query heads of a group share one selection, Hs = n_kv_heads, and selection
 *     head n serves query heads n*G .. n*G+G-1; tca_selection_heads() returns Hs.
 *     Every per-head argument below that concerns the selection (p, offs, n_rows,
 *     rows_out, the regions of idx / Kg / Vg) has one entry per selection head.
 *   - Compacted global subset: idx / Kg / Vg hold, for selection head n, rows
 *     offs[n] .. offs[n] + n_rows[n] - 1 of a flat buffer (offs = capacity prefix
 *     sums, host array of Hs+1 entries; the heads' rows share one flat buffer
 *     addressed through precomputed offsets, the layout of App. C).  idx is the
 *     absolute token position of each row, ascending within a head.
 *   - Positions are 0-based.  The local subset of the query at position i is the
 *     window (i-w, i]; a global row at position j is visible to it iff j <= i-w,
 *     so no key is counted twice (Sec. IV, "no overlap").
 *   - Return value: 0 on success, a negative TCA_ERR_* otherwise; nothing is
 *     launched when an argument check fails.  tca_last_error() returns a
 *     thread-local description of the last failure.
 *
 * Limits: head_dim in {64, 128}; block b a power of two, 2 <= b <= 256;
 * window w >= b and a multiple of b; n_q_heads <= 128, group size
 * n_q_heads/n_kv_heads <= 8; at most 4096 blocks per tca_select call.
 */
#ifndef TCA_H
#define TCA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define TCA_BF16 0
#define TCA_F32  1

#define TCA_OK               0
#define TCA_ERR_INVALID     -1   /* null pointer, inconsistent sizes, p not a distribution ... */
#define TCA_ERR_UNSUPPORTED -2   /* head_dim / block / dtype / size outside the limits above  */
#define TCA_ERR_WORKSPACE   -3   /* ws_bytes too small or ws misaligned                       */
#define TCA_ERR_HIP         -4   /* a HIP runtime call failed (see tca_last_error)            */

#define TCA_METRIC_HHI      0
#define TCA_METRIC_ENTROPY  1

#define TCA_SHARE_HEAD      0
#define TCA_SHARE_GROUP     1

#define TCA_MAX_HEADS   128
#define TCA_MAX_GROUP   8
#define TCA_MAX_COUNTS  9        /* log2(256) + 1 */
#define TCA_MAX_BLOCKS  4096

typedef struct tca_params {
  int32_t n_q_heads;   /* Hq                                                  */
  int32_t n_kv_heads;  /* Hkv, divides Hq                                      */
  int32_t head_dim;    /* d_h                                                 */
  int32_t block;       /* b, block size of Sec. IV-A (paper: 128)             */
  int32_t window;      /* w, local window of Sec. IV (paper: 4096)            */
  int32_t dtype;       /* TCA_BF16 or TCA_F32: type of Q, K, V, O, Kg, Vg     */
  double  alpha;       /* balance of Eq. 6 (paper: 0.5)                       */
  double  scale;       /* logit scale; 0 selects 1/sqrt(head_dim) of Eq. 1    */
  int32_t metric;      /* concentration index of Eq. 6: TCA_METRIC_HHI (the method's) or
                          TCA_METRIC_ENTROPY (the appendix ablation: entropy of the scores
                          renormalised inside the block, divided by ln b)          */
  int32_t share;       /* TCA_SHARE_HEAD: one selection per query head (the method's);
                          TCA_SHARE_GROUP: one per KV head, tokens scored by the mean over
                          the group's query heads of their Eq. 5 scores, so that the
                          compacted cache holds each kept row once per KV head          */
} tca_params;

/* ------------------------------------------------------------------ host --
 * Small fp64 host routines: configurations (Eq. 3), the rank->budget map
 * (Eq. 7) and the sizes that follow from them.  No GPU is touched. */

/* Hs, the number of selections kept per layer: n_q_heads, or n_kv_heads with
 * TCA_SHARE_GROUP.  Negative on invalid params. */
int tca_selection_heads(const tca_params* prm);

/* Number of entries of a configuration p: |K| = log2(b)+1 for K={1,2,4,..,b}
 * (Sec. IV-A).  Returns TCA_ERR_UNSUPPORTED if b is not a supported block size. */
int tca_num_counts(int b);

/* Eq. 3: M candidates, mu^i = log2(1 + (i-1)(b-1)/(M-1)), fixed sigma.
 * p_out: host [M][nk], row i = p^{i+1}.  M >= 1, sigma > 0. */
int tca_make_candidates(int b, int M, double sigma, double* p_out);

/* Configuration of the Eq. 3 family (fixed sigma, mu found by bisection)
 * whose mean budget sum_k k p_k equals frac*b.  frac >= 1: one-hot at k=b;
 * above the family's largest mean: the mu=log2(b) member; below its smallest
 * mean: one-hot at k=1.  p_out: host [nk]. */
int tca_config_from_budget(int b, double sigma, double frac, double* p_out);

/* Eq. 7: c_k = floor(m p_k) entries of value k in Psi; the m - sum c_k
 * blocks left over take the minimum budget (added to c_1).  p: host [nk]
 * (non-negative, sums to 1 within 1e-9).  counts_out: host [nk]. */
int tca_psi_counts(int b, int64_t m, const double* p, int64_t* counts_out);

/* Rows one tca_select call over n_blocks full blocks appends per head:
 * sum_k k c_k, independent of the data.  p: host [Hs][nk].  rows_out: host
 * [Hs] (nullable).  Returns the total over heads, or a negative error. */
int64_t tca_select_rows(const tca_params* prm, int64_t n_blocks, const double* p, int64_t* rows_out);

/* t = floor(sum_k k p_k): rows kept from a block completed during decoding
 * (Sec. IV-B, last paragraph).  p: host [nk].  Negative on error. */
int tca_decode_budget(int b, const double* p);

size_t tca_select_workspace_bytes(const tca_params* prm, int64_t n_tokens);
/* cap_rows: total rows of the flat global buffer (offs[Hs]). */
size_t tca_prefill_workspace_bytes(const tca_params* prm, int64_t n_queries, int64_t cap_rows);
/* max_head_rows: the largest capacity of one head's region, max_h (offs[h+1]-offs[h]). */
size_t tca_decode_workspace_bytes(const tca_params* prm, int batch, int64_t max_head_rows);
size_t tca_calibrate_workspace_bytes(const tca_params* prm, int64_t L_cal, int M);

/* ---------------------------------------------------------------- device --*/

/* Online core-context selection + compaction (Alg. 2 lines 1-6; Eq. 5-8).
 *
 * Scores tokens [pos0, pos0+n_tokens) of K with the query q_last:
 *   x_j = scale * q_last . k_j,  s = softmax(x) over these n_tokens keys   (Eq. 5)
 * splits them into m = n_tokens / b full blocks (a tail of n_tokens mod b
 * tokens only takes part in the softmax normaliser and is never selected),
 * evaluates h_j (Eq. 6), ranks the blocks by h (ties: lower block first),
 * gives the block of rank r (0 = smallest h) the r-th entry of the ascending
 * list Psi (Eq. 7), keeps each block's t_j highest-scoring tokens (ties: lower
 * position first; Eq. 8) and appends their K and V rows and positions, in
 * ascending position order, to each head's region of idx / Kg / Vg, starting
 * at row offs[h] + n_rows[h]; n_rows[h] grows by tca_select_rows()[h].
 * Rows that would pass offs[h+1] are dropped (never written).
 * TCA_SHARE_GROUP: the score of token j is sbar_j = (1/G) sum_g s_{g,j} over the G query
 * heads of the group, each s_g the softmax of Eq. 5 for that head; Eq. 6-8 run on sbar.
 *
 *   q_last : device [Hq, d]
 *   K, V   : device [Hkv, kv_stride, d]; pos0 is a multiple of b; pos0+n_tokens <= kv_stride
 *   p      : host [Hs][nk]
 *   offs   : host [Hs+1]
 *   n_rows : device int32 [Hs], in/out (zero it before the first call)
 *   idx    : device int32 [offs[Hs]]; Kg, Vg: device [offs[Hs], d]
 * Kg and Vg may both be NULL: only the positions (idx) and n_rows are written, for a caller that
 * keeps no compacted copy and calls tca_prefill the same way.
 * All scoring arithmetic is fp64.  Inside a block, tokens whose scores agree to within
 * 2^-44 relative are ordered by position, like exact ties (the ranking key drops the last
 * 8 mantissa bits), so the selected sets agree with an fp64 reference except at such
 * near-ties.  Does not synchronise. */
int tca_select(const tca_params* prm, const void* q_last, const void* K, const void* V,
               int64_t kv_stride, int64_t pos0, int64_t n_tokens,
               const double* p, const int64_t* offs, int32_t* n_rows,
               int32_t* idx, void* Kg, void* Vg,
               void* ws, size_t ws_bytes, void* stream);

/* Causal prefill attention over the global and local subsets (Eq. 2; Alg. 2 line 7).
 *
 * Query row r of Q sits at position i = q_pos0 + r and attends to
 *   { global rows g of its head with idx[g] <= i-w }  U  { dense keys max(0,i-w+1) .. i }
 * with one softmax over the union; O gets the weighted sum of the matching V rows.
 *
 *   Q, O   : device [Hq, n_queries, d]
 *   K, V   : device [Hkv, kv_stride, d], dense rows; q_pos0 + n_queries <= kv_stride
 *   idx, Kg, Vg, offs, n_rows : as written by tca_select (n_rows: device int32 [Hs])
 *   lse    : device float [Hq, n_queries] or NULL: natural-log sum of exp of the scaled logits
 * Kg and Vg may both be NULL (gather-free call): the global rows are read from K and V through
 * idx, for a prefill whose kept rows are not needed afterwards as a compacted cache.
 * TCA_BF16: bf16 MFMA products, fp32 softmax and accumulation.  TCA_F32: fp64 logits, fp32
 * exponentials and accumulation.
 * TCA_BF16 limit: (q_pos0 + n_queries + w + 128) * d * 2 bytes and every head's region must stay
 * below 2 GiB (8M positions at d = 128); beyond that the call returns TCA_ERR_UNSUPPORTED.
 * Does not synchronise. */
int tca_prefill(const tca_params* prm, const void* Q, int64_t q_pos0, int64_t n_queries,
                const void* K, const void* V, int64_t kv_stride,
                const int32_t* idx, const void* Kg, const void* Vg,
                const int64_t* offs, const int32_t* n_rows,
                void* O, float* lse, void* ws, size_t ws_bytes, void* stream);

/* Eq. 2 over one of the two key subsets alone, and the merge of two such results: the pieces of
 * tca_select_prefill_overlapped below, usable on their own.
 * tca_prefill_part: as tca_prefill, restricted to TCA_PART_WINDOW (the dense keys of each query's
 * window; idx, Kg, Vg, n_rows are not read and need not be filled yet) or TCA_PART_GLOBAL (the
 * global rows with idx <= i-w); TCA_PART_ALL is tca_prefill.  O holds the attention normalised
 * over that subset, lse (required for a part) the log-sum-exp of its scaled logits; a query
 * that sees nothing of the subset gets zeros and lse = -inf.
 * tca_prefill_merge: O_a <- (e^{lse_a} O_a + e^{lse_b} O_b) / (e^{lse_a} + e^{lse_b}), row by row:
 * the one softmax of Eq. 2 over the union of two disjoint key sets.  O_a, O_b: device
 * [Hq, n_queries, d]; lse_a, lse_b: device float [Hq, n_queries]; lse_out: the same or NULL. */
#define TCA_PART_ALL    0
#define TCA_PART_WINDOW 1
#define TCA_PART_GLOBAL 2
int tca_prefill_part(const tca_params* prm, int part, const void* Q, int64_t q_pos0, int64_t n_queries,
                     const void* K, const void* V, int64_t kv_stride,
                     const int32_t* idx, const void* Kg, const void* Vg,
                     const int64_t* offs, const int32_t* n_rows,
                     void* O, float* lse, void* ws, size_t ws_bytes, void* stream);
int tca_prefill_merge(const tca_params* prm, int64_t n_queries, void* O_a, const float* lse_a,
                      const void* O_b, const float* lse_b, float* lse_out, void* stream);

/* tca_select followed by tca_prefill over the same tokens [pos0, pos0 + n_tokens), with the
 * window part of the attention overlapped with the selection (App. C names this overlap as a
 * further optimisation): the window part runs on side_stream from the point `stream` has reached
 * at the call, the selection and the global part on `stream`, which then waits for the window
 * part and merges.  Arguments as for tca_select (q_last .. Vg) and tca_prefill (Q with q_pos0 =
 * pos0, O); O_part: device scratch shaped like O; lse_parts: device float [2][Hq][n_tokens];
 * the two workspaces as for tca_select and tca_prefill (one prefill workspace serves both parts).
 * Results equal tca_select + tca_prefill up to the rounding of the two partial outputs to the
 * storage type.  Creates and destroys two events; does not synchronise. */
int tca_select_prefill_overlapped(const tca_params* prm, const void* q_last, const void* Q,
                                  const void* K, const void* V, int64_t kv_stride, int64_t pos0,
                                  int64_t n_tokens, const double* p, const int64_t* offs,
                                  int32_t* n_rows, int32_t* idx, void* Kg, void* Vg, void* O,
                                  void* O_part, float* lse_parts, void* ws_select, size_t ws_select_bytes,
                                  void* ws_prefill, size_t ws_prefill_bytes, void* stream, void* side_stream);

/* Storage of the rows of the decode cache.  TCA_KV_NATIVE: rows of tca_params.dtype.
 * TCA_KV_FP8 (an extension, not in the paper; requires dtype TCA_BF16): a row x of d numbers is
 * kept as d FP8 E4M3 codes (OCP 8-bit floating point: bias 7, largest finite value 448, no
 * infinities) and one float scale:
 *     amax = max_i |x_i|,   scale = amax / 448  (1 if amax = 0),   code_i = RNE_e4m3(x_i / scale)
 * with both divisions in float32; what decode reads back is code_i * scale.  The cache then
 * takes 1 + 4/d bytes per element instead of 2. */
#define TCA_KV_NATIVE 0
#define TCA_KV_FP8    1

/* KV cache of a batch of sequences that share one set of per-head budgets
 * (budgets belong to the model, Sec. IV-A).  All pointers are device memory. */
typedef struct tca_cache {
  int32_t  batch;      /* B                                                            */
  int64_t  cap_rows;   /* rows of the flat global buffer per sequence (= offs[Hs])      */
  int32_t* idx;        /* [B, cap_rows]     positions of the global rows                */
  void*    Kg;         /* [B, cap_rows, d]  (TCA_KV_FP8: one byte per element)          */
  void*    Vg;         /* [B, cap_rows, d]                                              */
  int32_t* n_rows;     /* [B, Hs]           rows filled per head (updated by the library) */
  void*    ringK;      /* [B, Hkv, w, d]    last w dense rows, position P at slot P mod w */
  void*    ringV;      /* [B, Hkv, w, d]                                                */
  int64_t* length;     /* [B]               tokens seen so far (updated by the library)  */
  int32_t  kv_format;  /* TCA_KV_NATIVE or TCA_KV_FP8                                    */
  float*   Kg_scale;   /* [B, cap_rows]     TCA_KV_FP8 only (else ignored, may be NULL)  */
  float*   Vg_scale;   /* [B, cap_rows]                                                  */
  float*   ringK_scale;/* [B, Hkv, w]                                                    */
  float*   ringV_scale;/* [B, Hkv, w]                                                    */
} tca_cache;

/* Hand a prefilled sequence over to the decode cache: copies dense rows
 * [max(0,L-w), L) of K and V into sequence `seq`'s ring (slot = position mod w;
 * TCA_KV_FP8: as codes and scales) and sets length[seq] = L.  With TCA_KV_NATIVE
 * the global region of that sequence is whatever tca_select wrote there (pass
 * idx + seq*cap_rows etc. to tca_select); with TCA_KV_FP8 see tca_cache_load_global.
 * K, V: device [Hkv, kv_stride, d].  Does not synchronise. */
int tca_cache_load_window(const tca_params* prm, const tca_cache* cache, int seq,
                          const void* K, const void* V, int64_t kv_stride, int64_t L, void* stream);

/* Copies the global subset of one prefilled sequence, as tca_select left it in buffers of
 * tca_params.dtype, into sequence `seq` of the cache in the cache's storage format (the way
 * into a TCA_KV_FP8 cache; a plain copy with TCA_KV_NATIVE): rows offs[n] .. offs[n] +
 * n_rows[n] - 1 of every selection head n, their positions, and n_rows.
 *   idx, Kg, Vg : device, [offs[Hs]] / [offs[Hs], d], as written by tca_select
 *   offs        : host [Hs+1], offs[Hs] == cache->cap_rows;  n_rows: device int32 [Hs]
 * Does not synchronise. */
int tca_cache_load_global(const tca_params* prm, const tca_cache* cache, int seq,
                          const int32_t* idx, const void* Kg, const void* Vg,
                          const int64_t* offs, const int32_t* n_rows, void* stream);

/* One decode step for every sequence of the batch (Sec. IV-B, last paragraph).
 *
 * For sequence s with T = length[s]: the new row (k_new[s], v_new[s]) becomes
 * position T (ring slot T mod w); query q[s,h] attends to the head's global
 * rows with idx <= T-w and to dense positions max(0,T-w+1) .. T (Eq. 2 for one
 * query); if T+1 is a multiple of b, block T/b is complete: its b rows are
 * scored with this step's query (Eq. 5 restricted to the block) and the
 * t = floor(sum_k k p_k) best (ties: lower position), in ascending position
 * order, are appended to the head's global region (dropped beyond capacity);
 * finally length[s] = T+1.
 * TCA_SHARE_GROUP: the block's rows are ranked by the mean over the group's query heads of
 * their scores, each normalised over the block, and appended once per KV head.
 *
 *   q      : device [B, Hq, d];  k_new, v_new: device [B, Hkv, d];  O: device [B, Hq, d]
 *   offs   : host [Hs+1] (capacity prefix sums, offs[Hs] == cache->cap_rows)
 *   p      : host [Hs][nk]
 * Does not synchronise; lengths live on the device, so steps can be queued back to back.
 * The call only launches kernels on `stream` (no memset, no allocation, no read-back), so a
 * step may be captured into a HIP graph and replayed.
 * TCA_KV_FP8: the new rows are stored as codes and scales first; attention and the scoring of
 * a completed block read the rows back as code * scale; rows kept from a completed block are
 * copied as stored. */
int tca_decode(const tca_params* prm, const tca_cache* cache, const int64_t* offs,
               const void* q, const void* k_new, const void* v_new, const double* p,
               void* O, void* ws, size_t ws_bytes, void* stream);

/* tca_decode for callers that cannot allocate or hand over scratch memory: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, checks, kernels
 * and results as tca_decode, minus (ws, ws_bytes): the split-K partials go to an array of
 * TCA_DECODE_STATIC_BYTES bytes that is part of the library itself (each GPU the library runs on
 * holds it until the process ends).  The call allocates and frees nothing.  A step whose
 * tca_decode_workspace_bytes() exceeds TCA_DECODE_STATIC_BYTES is rejected with
 * TCA_ERR_WORKSPACE and nothing is launched (32 MiB covers batch 16 x 32 query heads x 128K
 * tokens at budgets up to 50 %).  Every call on one GPU uses the same array: nothing in it has
 * to be cleared between calls (each step writes what it reads), but calls that overlap in time
 * on one GPU - different streams, or a graph replay beside an eager call - race on it. */
#define TCA_DECODE_STATIC_BYTES (32u << 20)
int tca_decode_static(const tca_params* prm, const tca_cache* cache, const int64_t* offs,
                      const void* q, const void* k_new, const void* v_new, const double* p,
                      void* O, void* stream);

/* Offline head-specific sparsity determination (Alg. 1) on one calibration sequence.
 *
 * For every query head: column means of the dense causal attention matrix
 * A = softmax(scale * Q K^T) (mean of column k over the L_cal - k rows that can
 * see it; Eq. 4 inner term), the selection S_i of each of the M candidates of
 * Eq. 3 (same procedure as tca_select, scored by the last query of the sample),
 * a_i = sum over S_i of the column means (Eq. 4), and the valid candidate
 * (a_i >= tau) that keeps the fewest rows (ties: lower i).  If none is valid the
 * last candidate is returned and fallback[h] = 1.
 * TCA_SHARE_GROUP: one result per KV head; the candidates' sets come from the shared
 * selection and a_i sums the mean over the group's query heads of their column means.
 *
 *   Qcal : device [Hq, L_cal, d];  Kcal: device [Hkv, L_cal, d]
 *   p_star   : host [Hs][nk]   chosen configuration
 *   cand_idx : host [Hs]       its 0-based index
 *   a_out    : host [Hs][M] or NULL: a_i;  n_out: host int64 [Hs][M] or NULL: |S_i|
 *   fallback : host [Hs] or NULL
 * Waits for `stream` before returning (results are host arrays). */
int tca_calibrate_budgets(const tca_params* prm, const void* Qcal, const void* Kcal, int64_t L_cal,
                          int M, double sigma, double tau,
                          double* p_star, int32_t* cand_idx, double* a_out, int64_t* n_out,
                          int32_t* fallback, void* ws, size_t ws_bytes, void* stream);

/* Alg. 1 for every layer of a model (the determination is made once per model and covers all
 * heads of all layers, Sec. IV and IV-A): tca_calibrate_budgets once per layer, on that layer's
 * sample, results layer-major.
 *   Qcal, Kcal : host arrays of n_layers device pointers, [Hq, L_cal, d] and [Hkv, L_cal, d] each
 *   p_star [n_layers][Hs][nk], cand_idx [n_layers][Hs], a_out [n_layers][Hs][M] or NULL,
 *   n_out [n_layers][Hs][M] or NULL, fallback [n_layers][Hs] or NULL: host
 *   ws : as for tca_calibrate_budgets (reused by every layer).
 * Waits for `stream` before returning.  Stops at the first layer that fails. */
int tca_calibrate_layers(const tca_params* prm, int n_layers, const void* const* Qcal,
                         const void* const* Kcal, int64_t L_cal, int M, double sigma, double tau,
                         double* p_star, int32_t* cand_idx, double* a_out, int64_t* n_out,
                         int32_t* fallback, void* ws, size_t ws_bytes, void* stream);

/* Rotary position embedding of Q or K rows in place, the step that precedes this path in a
 * model layer (an extension: the paper takes Q and K as given, after position encoding).
 * Row r of every head sits at position pos0 + r; its pair i, (x_i, x_{i+d/2}) with
 * TCA_ROPE_HALF (the layout of Llama-family checkpoints) or (x_{2i}, x_{2i+1}) with
 * TCA_ROPE_INTERLEAVED, is turned by the angle (pos0 + r) * base^(-2i/d) (the RoFormer rotation).
 *   X : device [n_heads, n_rows, d] of tca_params.dtype (n_heads: Hq for Q, Hkv for K)
 * Angles and products are fp64, rounded once to the storage type.  Does not synchronise. */
#define TCA_ROPE_HALF        0
#define TCA_ROPE_INTERLEAVED 1
int tca_rope(const tca_params* prm, void* X, int n_heads, int64_t n_rows, int64_t pos0, double base,
             int pairing, void* stream);

/* The projections that produce what the method takes as given (Sec. III: Q = X W_Q, K = X W_K,
 * V = X W_V for every head), the step of a model layer that precedes tca_rope (an extension: the
 * paper's method starts from Q, K, V).  All heads in one call; the results are written in the
 * layout the next call reads, described by two strides per output, in elements: element e of head
 * h of token t lands at  out + h * head_stride + t * token_stride + e.
 *   head-major [H, n, d], what tca_select / tca_prefill / tca_rope read: token_stride = d,
 *     head_stride = n d (n = the rows the buffer holds per head; point Q / K / V at the first row
 *     to be written);   token-major [n, H, d], what tca_decode reads: token_stride = H d, head_stride = d.
 *   X    : device [n_tokens, hidden], the layer's input rows, of tca_params.dtype
 *   W    : device [(Hq + 2 Hkv) d, hidden], one row per output feature: the query heads first, then
 *          the key heads, then the value heads, d rows each (the concatenated q/k/v projection weights)
 *   bias : device [(Hq + 2 Hkv) d] or NULL, added to the features
 *   Q    : device, Hq heads;  K, V : device, Hkv heads each, sharing kv_token_stride / kv_head_stride
 * bf16: products are exact, sums fp32, one rounding to bf16; hidden must be a multiple of 64, the
 * strides multiples of 4, X and W 16-byte and the outputs 8-byte aligned.  fp32: fp32 multiply-adds
 * in the order of the hidden index; at most 65535 tokens per call.  Does not synchronise, takes no
 * workspace.  Errors: TCA_ERR_INVALID (NULL pointer, negative size, stride below d, alignment),
 * TCA_ERR_UNSUPPORTED (the limits above). */
int tca_qkv_project(const tca_params* prm, const void* X, int64_t n_tokens, int hidden, const void* W,
                    const void* bias, void* Q, int64_t q_token_stride, int64_t q_head_stride, void* K,
                    void* V, int64_t kv_token_stride, int64_t kv_head_stride, void* stream);

const char* tca_strerror(int code);
const char* tca_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* TCA_H */
