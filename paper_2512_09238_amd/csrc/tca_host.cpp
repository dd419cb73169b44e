// Host-side part of libtca: configurations (Eq. 3), the rank->budget map
// (Eq. 7), derived sizes, argument validation and error strings.  fp64, no GPU.
#include <cmath>
#include <cstring>

#include "tca_common.h"

namespace tca {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
}

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

int block_log2(int b) {
  if (b < 2 || b > 256 || (b & (b - 1)) != 0) return -1;
  int l = 0;
  while ((1 << l) < b) ++l;
  return l;
}

int check_params(const tca_params* prm) {
  if (!prm) return fail(TCA_ERR_INVALID, "params is NULL");
  if (prm->n_q_heads < 1 || prm->n_kv_heads < 1 || prm->n_q_heads % prm->n_kv_heads != 0)
    return fail(TCA_ERR_INVALID, "n_q_heads=%d must be a positive multiple of n_kv_heads=%d",
                prm->n_q_heads, prm->n_kv_heads);
  if (prm->n_q_heads > TCA_MAX_HEADS)
    return fail(TCA_ERR_UNSUPPORTED, "n_q_heads=%d exceeds %d", prm->n_q_heads, TCA_MAX_HEADS);
  if (prm->n_q_heads / prm->n_kv_heads > TCA_MAX_GROUP)
    return fail(TCA_ERR_UNSUPPORTED, "group size %d exceeds %d", prm->n_q_heads / prm->n_kv_heads,
                TCA_MAX_GROUP);
  if (prm->head_dim != 64 && prm->head_dim != 128)
    return fail(TCA_ERR_UNSUPPORTED, "head_dim=%d (supported: 64, 128)", prm->head_dim);
  if (block_log2(prm->block) < 0)
    return fail(TCA_ERR_UNSUPPORTED, "block=%d (supported: powers of two in [2,256])", prm->block);
  if (prm->window < prm->block || prm->window % prm->block != 0)
    return fail(TCA_ERR_INVALID, "window=%d must be a multiple of block=%d and >= it", prm->window,
                prm->block);
  if (prm->dtype != TCA_BF16 && prm->dtype != TCA_F32)
    return fail(TCA_ERR_UNSUPPORTED, "dtype=%d", prm->dtype);
  if (!(prm->alpha >= 0.0 && prm->alpha <= 1.0))
    return fail(TCA_ERR_INVALID, "alpha=%g outside [0,1]", prm->alpha);
  if (!(prm->scale >= 0.0) || !std::isfinite(prm->scale))
    return fail(TCA_ERR_INVALID, "scale=%g must be finite and >= 0", prm->scale);
  if (prm->metric != TCA_METRIC_HHI && prm->metric != TCA_METRIC_ENTROPY)
    return fail(TCA_ERR_UNSUPPORTED, "metric=%d", prm->metric);
  if (prm->share != TCA_SHARE_HEAD && prm->share != TCA_SHARE_GROUP)
    return fail(TCA_ERR_UNSUPPORTED, "share=%d", prm->share);
  return TCA_OK;
}

void config_from_mu(int nk, double mu, double sigma, double* p) {
  // Phi[log2 k] = exp(-(log2 k - mu)^2 / (2 sigma^2)), k = 2^0 .. 2^(nk-1).
  // The largest exponent is factored out before exponentiation (it cancels in
  // the ratio) so that very small sigma cannot produce 0/0.
  double ex[TCA_MAX_COUNTS];
  double top = -INFINITY;
  for (int e = 0; e < nk; ++e) {
    double dlt = (double)e - mu;
    ex[e] = -(dlt * dlt) / (2.0 * sigma * sigma);
    if (ex[e] > top) top = ex[e];
  }
  double sum = 0.0;
  for (int e = 0; e < nk; ++e) {
    p[e] = std::exp(ex[e] - top);
    sum += p[e];
  }
  for (int e = 0; e < nk; ++e) p[e] /= sum;
}

static double mean_budget(int nk, const double* p) {
  double s = 0.0;
  for (int e = 0; e < nk; ++e) s += (double)(1 << e) * p[e];
  return s;
}

bool valid_config(const double* p, int nk) {
  double s = 0.0;
  for (int e = 0; e < nk; ++e) {
    if (!(p[e] >= 0.0) || !std::isfinite(p[e])) return false;
    s += p[e];
  }
  return std::fabs(s - 1.0) <= 1e-9;
}

void psi_counts(int nk, int64_t m, const double* p, int64_t* c) {
  int64_t total = 0;
  for (int e = 0; e < nk; ++e) {
    c[e] = (int64_t)std::floor((double)m * p[e] + 1e-9);
    total += c[e];
  }
  c[0] += m - total;
}

}  // namespace tca

using namespace tca;

extern "C" {

int tca_selection_heads(const tca_params* prm) {
  int rc = check_params(prm);
  if (rc) return rc;
  return sel_heads(prm);
}

int tca_num_counts(int b) {
  int l = block_log2(b);
  if (l < 0) return fail(TCA_ERR_UNSUPPORTED, "block=%d (supported: powers of two in [2,256])", b);
  return l + 1;
}

int tca_make_candidates(int b, int M, double sigma, double* p_out) {
  int nk = tca_num_counts(b);
  if (nk < 0) return nk;
  if (!p_out || M < 1 || !(sigma > 0.0)) return fail(TCA_ERR_INVALID, "bad candidate arguments");
  for (int i = 0; i < M; ++i) {
    double mu = (M == 1) ? 0.0 : std::log2(1.0 + (double)i * (double)(b - 1) / (double)(M - 1));
    config_from_mu(nk, mu, sigma, p_out + (size_t)i * nk);
  }
  return TCA_OK;
}

int tca_config_from_budget(int b, double sigma, double frac, double* p_out) {
  int nk = tca_num_counts(b);
  if (nk < 0) return nk;
  if (!p_out || !(sigma > 0.0) || !(frac >= 0.0)) return fail(TCA_ERR_INVALID, "bad budget arguments");
  double target = frac * (double)b;
  double lo = 0.0, hi = (double)(nk - 1);
  if (frac >= 1.0) {
    for (int e = 0; e < nk; ++e) p_out[e] = (e == nk - 1) ? 1.0 : 0.0;
    return TCA_OK;
  }
  config_from_mu(nk, hi, sigma, p_out);
  if (target >= mean_budget(nk, p_out)) return TCA_OK;
  config_from_mu(nk, lo, sigma, p_out);
  if (target < mean_budget(nk, p_out)) {
    for (int e = 0; e < nk; ++e) p_out[e] = (e == 0) ? 1.0 : 0.0;
    return TCA_OK;
  }
  for (int it = 0; it < 200; ++it) {
    double mid = 0.5 * (lo + hi);
    config_from_mu(nk, mid, sigma, p_out);
    if (mean_budget(nk, p_out) < target) lo = mid; else hi = mid;
  }
  config_from_mu(nk, 0.5 * (lo + hi), sigma, p_out);
  return TCA_OK;
}

int tca_psi_counts(int b, int64_t m, const double* p, int64_t* counts_out) {
  int nk = tca_num_counts(b);
  if (nk < 0) return nk;
  if (!p || !counts_out || m < 0) return fail(TCA_ERR_INVALID, "bad psi arguments");
  if (!valid_config(p, nk)) return fail(TCA_ERR_INVALID, "p is not a distribution over %d counts", nk);
  psi_counts(nk, m, p, counts_out);
  return TCA_OK;
}

int64_t tca_select_rows(const tca_params* prm, int64_t n_blocks, const double* p, int64_t* rows_out) {
  int rc = check_params(prm);
  if (rc) return rc;
  if (!p || n_blocks < 0) return fail(TCA_ERR_INVALID, "bad select_rows arguments");
  int nk = block_log2(prm->block) + 1;
  int64_t total = 0;
  for (int h = 0; h < sel_heads(prm); ++h) {
    const double* ph = p + (size_t)h * nk;
    if (!valid_config(ph, nk)) return fail(TCA_ERR_INVALID, "p[%d] is not a distribution", h);
    int64_t c[TCA_MAX_COUNTS];
    psi_counts(nk, n_blocks, ph, c);
    int64_t rows = 0;
    for (int e = 0; e < nk; ++e) rows += c[e] << e;
    if (rows_out) rows_out[h] = rows;
    total += rows;
  }
  return total;
}

int tca_decode_budget(int b, const double* p) {
  int nk = tca_num_counts(b);
  if (nk < 0) return nk;
  if (!p || !valid_config(p, nk)) return fail(TCA_ERR_INVALID, "p is not a distribution over %d counts", nk);
  return (int)std::floor(mean_budget(nk, p) + 1e-9);
}

const char* tca_strerror(int code) {
  switch (code) {
    case TCA_OK: return "ok";
    case TCA_ERR_INVALID: return "invalid argument";
    case TCA_ERR_UNSUPPORTED: return "unsupported configuration";
    case TCA_ERR_WORKSPACE: return "workspace too small or misaligned";
    case TCA_ERR_HIP: return "HIP runtime error";
    default: return "unknown error";
  }
}

const char* tca_last_error(void) { return g_err; }

}  // extern "C"
