// Host-side decision policy of a verifier: Tukey fences with the adaptive multiplier of
// Alg. adaptive_iqr, and the per-stage bookkeeping of Alg. activation_verification /
// Alg. gradient_verification (violation counters with forgiveness, bans, the history of clean
// deviations, the per-iteration tainted set and its ">50 % flagged" reset).  The inputs are the few
// scalar statistics per submission that the GPU kernels emit, so this is plain double-precision C++
// with no device work; it can be called without a GPU.
#include <math.h>
#include <stdint.h>

#include <algorithm>
#include <limits>
#include <new>
#include <vector>

#include "stageverify.h"

namespace {

struct Quartiles { double q1, q2, q3; };

// 25th / 50th / 75th percentile with linear interpolation between order statistics.
Quartiles quartiles(std::vector<double> h) {
  std::sort(h.begin(), h.end());
  const size_t n = h.size();
  auto at = [&](double p) {
    const double pos = (double)(n - 1) * p;
    const size_t lo = (size_t)floor(pos);
    const size_t hi = std::min(lo + 1, n - 1);
    return h[lo] + (h[hi] - h[lo]) * (pos - (double)lo);
  };
  return Quartiles{at(0.25), at(0.5), at(0.75)};
}

double outside_fraction(const std::vector<double>& h, double lower, double upper) {
  size_t cnt = 0;
  for (double x : h) cnt += (x < lower) || (x > upper);
  return (double)cnt / (double)h.size();
}

struct Fences { double lower, upper, k, q2, iqr; };

Fences adapt(const std::vector<double>& h, double k_prev, const sv_policy_cfg& cfg) {
  const Quartiles q = quartiles(h);
  const double iqr = std::max(q.q3 - q.q1, cfg.eps);
  double k = k_prev;
  double lower = q.q2 - k * iqr, upper = q.q2 + k * iqr;
  double fp = outside_fraction(h, lower, upper);
  for (int it = 0; fp > cfg.alpha && it < cfg.n_max; ++it) {          // too many benign values outside: widen
    k *= cfg.grow;
    lower = q.q2 - k * iqr; upper = q.q2 + k * iqr;
    fp = outside_fraction(h, lower, upper);
  }
  for (int it = 0; fp < cfg.alpha / 10.0 && it < cfg.n_max; ++it) {   // far fewer than the target: narrow
    k *= cfg.shrink;
    lower = q.q2 - k * iqr; upper = q.q2 + k * iqr;
    fp = outside_fraction(h, lower, upper);
  }
  const double d_min = fabs(q.q2) * cfg.min_dist_mult;
  lower = std::min(lower, q.q2 - d_min);
  upper = std::max(upper, q.q2 + d_min);
  return Fences{lower, upper, k, q.q2, iqr};
}

bool cfg_ok(const sv_policy_cfg* c) {
  return c && c->c >= 1 && c->t_forgive >= 1 && c->window >= 1 && c->n_max >= 0 && c->k0 > 0.0 && c->alpha >= 0.0 && c->grow >= 1.0 &&
         c->shrink > 0.0 && c->shrink <= 1.0 && c->min_dist_mult >= 0.0 && c->eps > 0.0 && c->severe > 0.0;
}

}  // namespace

struct sv_policy {
  int d, m;
  sv_policy_cfg cfg;
  std::vector<int32_t> v, streak;
  std::vector<uint8_t> banned;
  std::vector<std::vector<double>> hist;
  std::vector<Fences> f;

  void update_fences() {
    for (int i = 0; i < m; ++i) {
      auto& h = hist[i];
      if ((int64_t)h.size() > cfg.window) h.erase(h.begin(), h.end() - cfg.window);
      if (h.empty()) continue;
      f[i] = adapt(h, f[i].k, cfg);
    }
  }
};

extern "C" {

sv_status sv_adaptive_iqr(const double* history, int32_t n, double k_prev, const sv_policy_cfg* cfg, double* lower, double* upper,
                          double* k_out) {
  if (!history || n < 1 || !cfg_ok(cfg) || !(k_prev > 0.0) || !lower || !upper || !k_out) return SV_EINVAL;
  const Fences f = adapt(std::vector<double>(history, history + n), k_prev, *cfg);
  *lower = f.lower; *upper = f.upper; *k_out = f.k;
  return SV_OK;
}

sv_status sv_policy_create(int32_t n_workers, int32_t n_metrics, const sv_policy_cfg* cfg, sv_policy** out) {
  if (!out) return SV_EINVAL;
  *out = nullptr;
  if (n_workers < 1 || n_metrics < 1 || !cfg_ok(cfg)) return SV_EINVAL;
  sv_policy* p = new (std::nothrow) sv_policy();
  if (!p) return SV_ENOMEM;
  p->d = n_workers; p->m = n_metrics; p->cfg = *cfg;
  p->v.assign(n_workers, 0); p->streak.assign(n_workers, 0); p->banned.assign(n_workers, 0);
  p->hist.resize(n_metrics);
  const double inf = std::numeric_limits<double>::infinity();
  p->f.assign(n_metrics, Fences{-inf, inf, cfg->k0, 0.0, inf});
  *out = p;
  return SV_OK;
}

void sv_policy_destroy(sv_policy* p) { delete p; }

sv_status sv_policy_warmup(sv_policy* p, const double* gamma) {
  if (!p || !gamma) return SV_EINVAL;
  for (int r = 0; r < p->d; ++r)
    for (int i = 0; i < p->m; ++i) p->hist[i].push_back(gamma[(size_t)r * p->m + i]);
  p->update_fences();
  return SV_OK;
}

sv_status sv_policy_step(sv_policy* p, const double* gamma, const uint8_t* skip, const uint8_t* pre_tainted, uint8_t* tainted_out) {
  if (!p || !gamma || !tainted_out) return SV_EINVAL;
  int n_tainted = 0;
  for (int r = 0; r < p->d; ++r) {
    tainted_out[r] = 0;
    if (p->banned[r]) continue;
    if (pre_tainted && pre_tainted[r]) { tainted_out[r] = 1; ++n_tainted; continue; }
    if (skip && skip[r]) continue;
    const double* g = gamma + (size_t)r * p->m;
    bool violated = false, severe = false;
    for (int i = 0; i < p->m; ++i) {
      violated |= !(g[i] > p->f[i].lower) || !(g[i] < p->f[i].upper);         // on the fence counts; NaN counts
      severe |= fabs(g[i] - p->f[i].q2) >= p->cfg.severe * p->f[i].k * p->f[i].iqr;
    }
    if (violated) {
      p->v[r] += 1;
      p->streak[r] = 0;
      tainted_out[r] = 1;
      ++n_tainted;
      if (p->v[r] >= p->cfg.c || severe) p->banned[r] = 1;
    } else {
      for (int i = 0; i < p->m; ++i) p->hist[i].push_back(g[i]);
      p->streak[r] += 1;
      if (p->streak[r] >= p->cfg.t_forgive) {
        p->v[r] = std::max(0, p->v[r] - 1);
        p->streak[r] = 0;
      }
    }
  }
  p->update_fences();
  int active = 0;
  for (int r = 0; r < p->d; ++r) active += !p->banned[r];
  if ((double)n_tainted > 0.5 * (double)active)                               // read as a natural shift of the statistic
    for (int r = 0; r < p->d; ++r) tainted_out[r] = 0;
  return SV_OK;
}

sv_status sv_policy_state(const sv_policy* p, int32_t* violations, uint8_t* banned, double* lower, double* upper, double* k,
                          int32_t* history_len) {
  if (!p) return SV_EINVAL;
  for (int r = 0; r < p->d; ++r) {
    if (violations) violations[r] = p->v[r];
    if (banned) banned[r] = p->banned[r];
  }
  for (int i = 0; i < p->m; ++i) {
    if (lower) lower[i] = p->f[i].lower;
    if (upper) upper[i] = p->f[i].upper;
    if (k) k[i] = p->f[i].k;
    if (history_len) history_len[i] = (int32_t)p->hist[i].size();
  }
  return SV_OK;
}

}  // extern "C"
