// Internal interface of the selection stages (Eq. 5-7), shared with calibration.
#pragma once

#include <hip/hip_runtime.h>

#include "tca_common.h"

namespace tca {

struct SelectWs {
  uint8_t* tokrank;   // [Hq][n_blocks*b]  rank of each token inside its block (0 = highest logit); calibration only
  uint64_t* keys;     // [Hq][n_blocks*b]  ranking key of each token (ordered logit bits, position in the low byte)
  double* stats;      // [Hq][nbt][4]      per block: max logit M, sum e^(x-M), sum e^(2(x-M)), sum e^(x-M) (x-M)
  int32_t* blk_t;     // [Hq][n_blocks]    budget t_j of each block (Eq. 7)
  int32_t* blk_dst;   // [Hq][n_blocks]    first destination row of each block inside the head's region
  size_t bytes;
};

SelectWs carve_select_ws(void* ws, int Hq, int b, int64_t n_tokens);

void select_score_stage(const tca_params* prm, const void* q_last, const void* K, int64_t kv_stride,
                        int64_t n_tokens, const SelectWs& w, hipStream_t st);

void select_assign_stage(const tca_params* prm, int64_t n_tokens, const double* p, const int64_t* cap,
                         const double* stats, int32_t* n_rows, int32_t* blk_t, int32_t* blk_dst,
                         hipStream_t st);

}  // namespace tca
