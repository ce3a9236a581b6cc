// Host-side state around the verification step: the stride selection and acceptance-rate average of Alg. 2
// (steps 1 and 3, Sec. IV-B objective) and the page bookkeeping of the per-user KV sessions (Sec. IV-C).
// No device work: scalar arithmetic and a free list.
#include <math.h>
#include <new>
#include <vector>

#include "flexverify.h"

struct fsv_pager {
  int32_t page_size = 16, max_pages_per_session = 0;
  std::vector<int32_t> free_list;                 // stack: the lowest ids are handed out first
  std::vector<std::vector<int32_t>> owned;        // per session, in logical order
};

extern "C" {

int fsv_policy_stride(const fsv_latency_model *m, double rate, double gamma_hat, int32_t k_max, int32_t tau_model,
                      double *objective_out) {
  if (!m || !(rate > 0.0) || k_max < 1 || !(gamma_hat >= 0.0) || (tau_model != FSV_TAU_LINEAR && tau_model != FSV_TAU_GEOMETRIC))
    return FSV_E_INVALID_ARG;
  const double t_fixed = m->t_prop + m->t_base + m->t_down + m->header_bits / rate + m->beta;
  const double t_marginal = m->alpha_edge + m->bits_per_token / rate + m->delta_cloud;
  int best_k = 1;
  double best = -1.0, tokens = 1.0, pw = 1.0;
  for (int k = 1; k <= k_max; ++k) {
    if (tau_model == FSV_TAU_LINEAR) {
      tokens = 1.0 + gamma_hat * k;
    } else {
      pw *= gamma_hat;
      tokens += pw;
    }
    const double f = tokens / (t_fixed + k * t_marginal);
    if (f > best) { best = f; best_k = k; }   // strict: ties go to the smallest K
  }
  if (objective_out) *objective_out = best;
  return best_k;
}

double fsv_policy_step_time(const fsv_latency_model *m, double rate, int32_t k, double cloud_seconds) {
  if (!m || !(rate > 0.0) || k < 0) return -1.0;
  const double t_cloud = (cloud_seconds >= 0.0) ? cloud_seconds : m->t_base + k * m->delta_cloud;
  return (m->alpha_edge * k + m->beta) + (m->t_prop + (k * m->bits_per_token + m->header_bits) / rate) + t_cloud + m->t_down;
}

double fsv_policy_ema(double gamma_hat, int32_t tau, int32_t k, double mu) {
  if (k <= 0) return gamma_hat;
  return (1.0 - mu) * gamma_hat + mu * ((double)tau / (double)k);
}

int fsv_pager_create(int32_t num_pages, int32_t max_sessions, int32_t max_pages_per_session, fsv_pager **out) {
  if (!out) return FSV_E_INVALID_ARG;
  *out = nullptr;
  if (num_pages <= 0 || max_sessions <= 0 || max_pages_per_session <= 0) return FSV_E_INVALID_ARG;
  fsv_pager *p = new (std::nothrow) fsv_pager();
  if (!p) return FSV_E_HIP;
  p->max_pages_per_session = max_pages_per_session;
  p->free_list.resize(num_pages);
  for (int32_t i = 0; i < num_pages; ++i) p->free_list[i] = num_pages - 1 - i;
  p->owned.resize(max_sessions);
  *out = p;
  return FSV_OK;
}

void fsv_pager_destroy(fsv_pager *p) { delete p; }

int fsv_pager_reserve(fsv_pager *p, int32_t session, int32_t n_positions, int32_t *page_table_row) {
  if (!p || session < 0 || session >= (int32_t)p->owned.size() || n_positions < 0) return FSV_E_INVALID_ARG;
  std::vector<int32_t> &have = p->owned[session];
  const int32_t need = (n_positions + p->page_size - 1) / p->page_size;
  if (need > p->max_pages_per_session) return FSV_E_CAPACITY;
  if (need - (int32_t)have.size() > (int32_t)p->free_list.size()) return FSV_E_CAPACITY;   // nothing is taken on failure
  while ((int32_t)have.size() < need) {
    have.push_back(p->free_list.back());
    p->free_list.pop_back();
  }
  if (page_table_row)
    for (size_t i = 0; i < have.size(); ++i) page_table_row[i] = have[i];
  return FSV_OK;
}

int fsv_pager_trim(fsv_pager *p, int32_t session, int32_t n_positions) {
  if (!p || session < 0 || session >= (int32_t)p->owned.size() || n_positions < 0) return FSV_E_INVALID_ARG;
  std::vector<int32_t> &have = p->owned[session];
  const int32_t keep = (n_positions + p->page_size - 1) / p->page_size;
  int released = 0;
  while ((int32_t)have.size() > keep) {
    p->free_list.push_back(have.back());
    have.pop_back();
    ++released;
  }
  return released;
}

int32_t fsv_pager_free_pages(const fsv_pager *p) { return p ? (int32_t)p->free_list.size() : 0; }

int32_t fsv_pager_session_pages(const fsv_pager *p, int32_t session) {
  if (!p || session < 0 || session >= (int32_t)p->owned.size()) return 0;
  return (int32_t)p->owned[session].size();
}

}  // extern "C"
