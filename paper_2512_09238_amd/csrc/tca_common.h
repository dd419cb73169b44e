// Internal helpers shared by the translation units of libtca: error reporting,
// argument validation and the host-side fp64 bookkeeping of Eq. 3 / Eq. 7.
#pragma once

#include <cstdarg>
#include <cstdint>
#include <cstdio>

#include "tca.h"

namespace tca {

// Thread-local description of the last failure (returned by tca_last_error()).
void set_error(const char* fmt, ...);
int fail(int code, const char* fmt, ...);

// log2 of a supported block size, or -1.
int block_log2(int b);

// Checks every field of prm against the documented limits.
int check_params(const tca_params* prm);

// Eq. 3 for one mu; p has nk entries.
void config_from_mu(int nk, double mu, double sigma, double* p);

// Checks that p is a distribution over nk entries (>= 0, sums to 1 within 1e-9).
bool valid_config(const double* p, int nk);

// Eq. 7 counts; the deficit goes to the k=1 group.
void psi_counts(int nk, int64_t m, const double* p, int64_t* c);

// Diagnostics switches (tca_diag.h): whether tca_prefill records its shader clock, and which
// workgroup shape the bf16 prefill kernel takes (0 = chosen by the call's size).
bool diag_prefill_clocks();
int prefill_variant();

inline double logit_scale(const tca_params* prm) {
  return prm->scale != 0.0 ? prm->scale : 1.0 / __builtin_sqrt((double)prm->head_dim);
}
// Selections kept per layer, and query heads served by each of them.
inline int sel_heads(const tca_params* prm) { return prm->share == TCA_SHARE_GROUP ? prm->n_kv_heads : prm->n_q_heads; }
inline int sel_group(const tca_params* prm) { return prm->share == TCA_SHARE_GROUP ? prm->n_q_heads / prm->n_kv_heads : 1; }
inline size_t elem_bytes(const tca_params* prm) { return prm->dtype == TCA_BF16 ? 2 : 4; }
inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

}  // namespace tca

#define TCA_HIP_CHECK(expr)                                                              \
  do {                                                                                   \
    hipError_t e_ = (expr);                                                              \
    if (e_ != hipSuccess)                                                                \
      return tca::fail(TCA_ERR_HIP, "%s failed: %s (%s:%d)", #expr, hipGetErrorString(e_), \
                       __FILE__, __LINE__);                                              \
  } while (0)
