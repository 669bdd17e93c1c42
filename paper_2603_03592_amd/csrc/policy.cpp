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
#include <utility>
#include <vector>

#include "stageverify.h"

namespace {

// A history window sorted once: order statistics and "how many values lie outside an interval" are then index
// arithmetic and two binary searches, whatever the number of multipliers tried.
struct SortedWindow {
  std::vector<double> v;
  explicit SortedWindow(std::vector<double> h) : v(std::move(h)) { std::sort(v.begin(), v.end()); }
  // percentile p in [0, 1], linear interpolation between the order statistics around position (n - 1) p
  double percentile(double p) const {
    const double pos = (double)(v.size() - 1) * p;
    const size_t lo = (size_t)floor(pos);
    const size_t hi = std::min(lo + 1, v.size() - 1);
    return v[lo] + (v[hi] - v[lo]) * (pos - (double)lo);
  }
  // fraction of the window strictly below `lower` or strictly above `upper`
  double outside(double lower, double upper) const {
    const size_t below = (size_t)(std::lower_bound(v.begin(), v.end(), lower) - v.begin());
    const size_t above = (size_t)(v.end() - std::upper_bound(v.begin(), v.end(), upper));
    return (double)(below + above) / (double)v.size();
  }
};

struct Fences { double lower, upper, k, q2, iqr; };

// Alg. adaptive_iqr.  The widening and the narrowing search are the same walk along k <- k * factor with a different
// factor and stopping test, so they are one routine called twice; the fences follow k as median -/+ k * IQR.
Fences adapt(const std::vector<double>& h, double k_prev, const sv_policy_cfg& cfg) {
  const SortedWindow w(h);
  const double q1 = w.percentile(0.25), q2 = w.percentile(0.5), q3 = w.percentile(0.75);
  const double iqr = std::max(q3 - q1, cfg.eps);
  Fences f{0.0, 0.0, k_prev, q2, iqr};
  double frac = 0.0;
  auto place = [&]() {
    f.lower = q2 - f.k * iqr; f.upper = q2 + f.k * iqr;
    frac = w.outside(f.lower, f.upper);
  };
  enum Dir { kWiden, kNarrow };
  auto walk = [&](Dir dir) {
    const double factor = dir == kWiden ? cfg.grow : cfg.shrink;
    for (int it = 0; it < cfg.n_max; ++it) {
      // widen while more than the target fraction of (benign) history lies outside; narrow while far fewer do
      const bool go = dir == kWiden ? frac > cfg.alpha : frac < cfg.alpha / 10.0;
      if (!go) break;
      f.k *= factor;
      place();
    }
  };
  place();
  walk(kWiden);
  walk(kNarrow);
  // optional floor on the fences' distance from the median (Lambda of the metric)
  const double d_min = fabs(q2) * cfg.min_dist_mult;
  f.lower = std::min(f.lower, q2 - d_min);
  f.upper = std::max(f.upper, q2 + d_min);
  return f;
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

  // keep the last `window` values of every history
  void truncate() {
    for (auto& h : hist)
      if ((int64_t)h.size() > cfg.window) h.erase(h.begin(), h.end() - cfg.window);
  }
  void update_fences() {
    for (int i = 0; i < m; ++i)
      if (!hist[i].empty()) f[i] = adapt(hist[i], f[i].k, cfg);
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
  p->truncate();        // the warm-up listing has no later call that would cut for it
  p->update_fences();
  return SV_OK;
}

sv_status sv_policy_step(sv_policy* p, const double* gamma, const uint8_t* skip, const uint8_t* pre_tainted, uint8_t* tainted_out) {
  if (!p || !gamma || !tainted_out) return SV_EINVAL;
  int n_tainted = 0;
  // Alg. activation_verification / Alg. gradient_verification cut the window before anybody is examined; the fences
  // adapted at the end of the call therefore see the kept values plus this call's clean ones (up to window + d)
  p->truncate();
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
