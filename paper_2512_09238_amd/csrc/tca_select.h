// Internal interface of the selection stages (Eq. 5-7), shared with calibration.
#pragma once

#include <hip/hip_runtime.h>

#include "tca_common.h"

namespace tca {

// Hs = selection heads (query heads, or KV heads when the group shares one selection); nbt = blocks
// including a ragged tail.
struct SelectWs {
  uint8_t* tokrank;   // [Hs][n_blocks*b]  rank of each token inside its block (0 = highest score); calibration only
  uint64_t* keys;     // [Hs][n_blocks*b]  ranking key of each token (ordered score bits, position in the low byte)
  double* stats;      // [Hq][nbt][4]      per block and query head: max logit M, sum e^(x-M), sum e^(2(x-M)), sum e^(x-M) (x-M)
  double* sel_stats;  // [Hs][nbt][4]      the same four of the score that ranks tokens: `stats` itself, or those of the group score y
  double* xlog;       // [Hq][nbt*b]       logits of every query head (shared selection only)
  double* lse;        // [Hq]              log of the Eq. 5 normaliser of every query head (shared selection only)
  int32_t* blk_t;     // [Hs][n_blocks]    budget t_j of each block (Eq. 7)
  int32_t* blk_dst;   // [Hs][n_blocks]    first destination row of each block inside the head's region
  size_t bytes;
};

SelectWs carve_select_ws(void* ws, const tca_params* prm, int64_t n_tokens);

void select_score_stage(const tca_params* prm, const void* q_last, const void* K, int64_t kv_stride,
                        int64_t n_tokens, const SelectWs& w, hipStream_t st);

// p, cap, n_rows: one entry per selection head; stats: SelectWs::sel_stats.
void select_assign_stage(const tca_params* prm, int64_t n_tokens, const double* p, const int64_t* cap,
                         const double* stats, int32_t* n_rows, int32_t* blk_t, int32_t* blk_dst,
                         hipStream_t st);

}  // namespace tca
