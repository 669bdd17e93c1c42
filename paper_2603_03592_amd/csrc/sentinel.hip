// Alg. momentum_verification end to end for the verifiers of p pipeline stages with d workers each
// (worker r of every stage belongs to data-parallel pipe r).  The device work -- the statistics of every
// worker's signal against the stage's EMA, the gradient replacement, the EMA update over the clean set --
// goes through the library's own C entry points on the caller's stream; the decisions in between are the
// host-side policy (sv_policy_*).  Each forward / backward call therefore waits once for the stream: the
// few scalars per worker have to reach the host before the policy can decide who enters the EMA.
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <limits>
#include <vector>

#include <hip/hip_runtime.h>

#include "stageverify.h"

struct sv_sentinel {
  sv_ctx* ctx = nullptr;
  sv_sentinel_cfg cfg;
  int n_metrics = 0;
  int metric_bit[5];                       // mask bit of column i of Gamma
  std::vector<float*> m[2];                // [kind][stage] device fp32 [T, D]; kind 0 = activations, 1 = gradients
  std::vector<sv_policy*> pol[2];
  std::vector<uint8_t> tainted;            // [stage * d + r] of the current iteration
  bool warm = true;
  sv_result* res_dev = nullptr;
  float* sw_dev = nullptr;
  uint8_t* mask_dev = nullptr;             // two rows of d bytes: replacement mask, EMA exclusion mask
  float* sum_dev = nullptr;                // [T, D]: sum over the signals not excluded beforehand, written by the score pass
  // sliced Wasserstein against the EMA without projecting the EMA: its projections follow from the signals' (linearity)
  std::vector<float*> pm[2];               // [kind][stage] device fp32 [n_dirs, Tpad]: <u_l, m_t>, kept up to date with m
  float* cproj = nullptr;                  // [d, n_dirs, Tpad]: the current signals' projections
  int64_t n_calls = 0, n_from_sum = 0, n_from_signals = 0, n_sw_carried = 0;
  // pinned staging
  sv_result* res_host = nullptr;
  float* sw_host = nullptr;
  uint8_t* mask_host = nullptr;
  char err[256] = "";
};

namespace {

void set_err(sv_sentinel* s, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(s->err, sizeof(s->err), fmt, ap);
  va_end(ap);
}

#define SN_HIP(s, call)                                                         \
  do {                                                                          \
    hipError_t e_ = (call);                                                     \
    if (e_ != hipSuccess) { set_err(s, "%s failed: %s", #call, hipGetErrorString(e_)); return SV_EHIP; } \
  } while (0)
#define SN_SV(s, call)                                                          \
  do {                                                                          \
    sv_status st_ = (call);                                                     \
    if (st_ != SV_OK) { set_err(s, "%s: %s", #call, sv_last_error((s)->ctx)); return st_; } \
  } while (0)

// Gamma [d, n_metrics] of the d signals against the reference point m, on the host (waits for the stream).
// `skip` [d]: the signals known to be excluded from the EMA before they are scored.  Where the score pass can do it,
// it also leaves the sum over the others in sum_dev (*summed = true), which saves the EMA update its own pass over the
// signals whenever the verdicts exclude nobody else.
sv_status gamma_of(sv_sentinel* s, const void* signals, int dtype, const float* m, const float* pm, const uint8_t* skip, bool* summed,
                   std::vector<double>& gamma, hipStream_t st) {
  const sv_sentinel_cfg& c = s->cfg;
  const int d = c.n_workers;
  const int64_t stride = c.T * c.D;
  const float inf = std::numeric_limits<float>::infinity();
  const float tau[4] = {inf, inf, inf, inf};      // nothing is decided on the device here: the fences live in the policy
  sv_status sum_st = s->sum_dev ? sv_score_and_sum(s->ctx, signals, stride, d, m, dtype, SV_F32, c.T, c.D, c.metric_mask & 15u, tau,
                                                   SV_REDUCE_GLOBAL, nullptr, s->res_dev, skip, s->sum_dev, st)
                                : SV_EUNSUPPORTED;
  *summed = sum_st == SV_OK;
  if (sum_st == SV_EUNSUPPORTED)                  // shapes the summing pass does not take: the plain one
    SN_SV(s, sv_score_and_flag(s->ctx, signals, stride, d, m, 0, dtype, SV_F32, c.T, c.D, c.metric_mask & 15u, tau, SV_REDUCE_GLOBAL, nullptr,
                               s->res_dev, st));
  else if (sum_st != SV_OK) { set_err(s, "sv_score_and_sum: %s", sv_last_error(s->ctx)); return sum_st; }
  SN_HIP(s, hipMemcpyAsync(s->res_host, s->res_dev, sizeof(sv_result) * d, hipMemcpyDeviceToHost, st));
  if (c.metric_mask & SV_M_SW) {
    if (pm) ++s->n_sw_carried;
    if (pm)
      SN_SV(s, sv_sw_against_projection(s->ctx, signals, stride, d, dtype, c.T, c.D, c.directions, c.n_dirs, pm, s->cproj, inf, s->sw_dev,
                                        nullptr, st));
    else
      SN_SV(s, sv_sliced_wasserstein(s->ctx, signals, stride, d, m, 0, dtype, SV_F32, c.T, c.D, c.directions, c.n_dirs, inf, s->sw_dev,
                                     nullptr, st));
    SN_HIP(s, hipMemcpyAsync(s->sw_host, s->sw_dev, sizeof(float) * d, hipMemcpyDeviceToHost, st));
  }
  SN_HIP(s, hipStreamSynchronize(st));
  gamma.assign((size_t)d * s->n_metrics, 0.0);
  for (int r = 0; r < d; ++r)
    for (int i = 0; i < s->n_metrics; ++i) {
      const int bit = s->metric_bit[i];
      double v;
      if (bit == SV_M_SW) v = s->sw_host[r];
      else v = s->res_host[r].score[bit == SV_M_RELL2 ? SV_IDX_RELL2 : bit == SV_M_L1 ? SV_IDX_L1 : bit == SV_M_ZL2 ? SV_IDX_ZL2 : SV_IDX_SFR];
      gamma[(size_t)r * s->n_metrics + i] = v;
    }
  return SV_OK;
}

// Eq. momentum_def over the signals with excl[r] == 0.  If the score pass has left the sum over the signals with
// skip[r] == 0 and the verdicts excluded nobody beyond those, the update is one pass over m and that sum; otherwise
// the update reads the signals itself.
sv_status update_ema(sv_sentinel* s, float* m, float* pm, const void* signals, int dtype, const uint8_t* excl, const uint8_t* skip,
                     bool summed, float beta, hipStream_t hs, bool mask_uploaded = false) {
  const int d = s->cfg.n_workers;
  if (pm) SN_SV(s, sv_sw_projection_ema(s->ctx, pm, s->cproj, d, excl, s->cfg.T, s->cfg.n_dirs, beta, hs));
  bool same = summed;
  int n = 0;
  for (int r = 0; r < d; ++r) { same = same && (excl[r] != 0) == (skip[r] != 0); n += excl[r] == 0; }
  ++s->n_calls;
  if (same) {
    ++s->n_from_sum;
    SN_SV(s, sv_ema_from_sum(s->ctx, m, s->sum_dev, n, s->cfg.T, s->cfg.D, beta, hs));
    return SV_OK;
  }
  ++s->n_from_signals;
  if (!mask_uploaded) SN_HIP(s, hipMemcpyAsync(s->mask_dev + d, excl, (size_t)d, hipMemcpyHostToDevice, hs));
  SN_SV(s, sv_ema_update(s->ctx, m, signals, s->cfg.T * s->cfg.D, d, dtype, s->mask_dev + d, s->cfg.T, s->cfg.D, beta, hs));
  return SV_OK;
}

sv_status check_stage(sv_sentinel* s, int stage, const void* sig, int dtype, uint8_t* tainted_out) {
  if (stage < 0 || stage >= s->cfg.n_stages) { set_err(s, "stage %d out of range", stage); return SV_EINVAL; }
  if (!sig || !tainted_out) { set_err(s, "signals and tainted_out must be non-NULL"); return SV_EINVAL; }
  if (dtype != SV_F32 && dtype != SV_BF16) { set_err(s, "unknown dtype"); return SV_EINVAL; }
  return SV_OK;
}

}  // namespace

extern "C" {

sv_status sv_sentinel_create(sv_ctx* ctx, const sv_sentinel_cfg* cfg, sv_sentinel** out) {
  if (!out) return SV_EINVAL;
  *out = nullptr;
  if (!ctx || !cfg || cfg->n_stages < 1 || cfg->n_workers < 1 || cfg->n_workers > 1024 || cfg->T < 1 || cfg->D < 1 || cfg->D % 8) return SV_EINVAL;
  if (!(cfg->metric_mask & 31u) || (cfg->metric_mask & ~31u)) return SV_EINVAL;
  if ((cfg->metric_mask & SV_M_SW) && (!cfg->directions || cfg->n_dirs < 1)) return SV_EINVAL;
  if (!(cfg->beta_h >= 0.0f && cfg->beta_h < 1.0f && cfg->beta_g >= 0.0f && cfg->beta_g < 1.0f)) return SV_EINVAL;
  sv_sentinel* s = new sv_sentinel();
  s->ctx = ctx; s->cfg = *cfg;
  for (int bit = 1; bit <= 16; bit <<= 1)
    if (cfg->metric_mask & (uint32_t)bit) s->metric_bit[s->n_metrics++] = bit;
  const int d = cfg->n_workers;
  sv_status st = SV_OK;
  for (int kind = 0; kind < 2 && st == SV_OK; ++kind)
    for (int i = 0; i < cfg->n_stages && st == SV_OK; ++i) {
      sv_policy* p = nullptr;
      st = sv_policy_create(d, s->n_metrics, kind == 0 ? &cfg->policy_h : &cfg->policy_g, &p);
      if (st == SV_OK) s->pol[kind].push_back(p);
    }
  const size_t m_bytes = (size_t)cfg->T * cfg->D * sizeof(float);
  hipError_t e = hipSuccess;
  for (int kind = 0; kind < 2 && st == SV_OK && e == hipSuccess; ++kind)
    for (int i = 0; i < cfg->n_stages && e == hipSuccess; ++i) {
      float* p = nullptr;
      e = hipMalloc(&p, m_bytes);
      if (e == hipSuccess) { s->m[kind].push_back(p); e = hipMemset(p, 0, m_bytes); }     // m_0 = 0
    }
  if (st == SV_OK && e == hipSuccess) e = hipMalloc(&s->res_dev, sizeof(sv_result) * d);
  if (st == SV_OK && e == hipSuccess) e = hipMalloc(&s->sw_dev, sizeof(float) * d);
  if (st == SV_OK && e == hipSuccess) e = hipMalloc(&s->mask_dev, 2 * (size_t)d);
  if (st == SV_OK && e == hipSuccess && (cfg->metric_mask & SV_M_SW) && d <= 32 && cfg->n_dirs % 32 == 0 && cfg->D % 64 == 0 &&
      sv_sw_row_len(cfg->T) <= 16384) {               // optional: without them the EMA itself is projected in every check
    const size_t p_bytes = (size_t)cfg->n_dirs * (size_t)sv_sw_row_len(cfg->T) * sizeof(float);
    bool ok = hipMalloc(&s->cproj, p_bytes * d) == hipSuccess;
    for (int kind = 0; kind < 2 && ok; ++kind)
      for (int i = 0; i < cfg->n_stages && ok; ++i) {
        float* p = nullptr;
        ok = hipMalloc(&p, p_bytes) == hipSuccess;
        if (ok) { s->pm[kind].push_back(p); ok = hipMemset(p, 0, p_bytes) == hipSuccess; }     // projections of m_0 = 0
      }
    if (!ok) {
      (void)hipGetLastError();
      for (int kind = 0; kind < 2; ++kind) { for (float* p : s->pm[kind]) (void)hipFree(p); s->pm[kind].clear(); }
      if (s->cproj) { (void)hipFree(s->cproj); s->cproj = nullptr; }
    }
  }
  if (st == SV_OK && e == hipSuccess && d <= 32) {  // optional: without it the EMA update reads the signals itself
    if (hipMalloc(&s->sum_dev, m_bytes) != hipSuccess) { s->sum_dev = nullptr; (void)hipGetLastError(); }
  }
  if (st == SV_OK && e == hipSuccess) e = hipHostMalloc((void**)&s->res_host, sizeof(sv_result) * d, hipHostMallocDefault);
  if (st == SV_OK && e == hipSuccess) e = hipHostMalloc((void**)&s->sw_host, sizeof(float) * d, hipHostMallocDefault);
  if (st == SV_OK && e == hipSuccess) e = hipHostMalloc((void**)&s->mask_host, 2 * (size_t)d, hipHostMallocDefault);
  if (st != SV_OK || e != hipSuccess) {
    sv_sentinel_destroy(s);
    return st != SV_OK ? st : (e == hipErrorOutOfMemory ? SV_ENOMEM : SV_EHIP);
  }
  s->tainted.assign((size_t)cfg->n_stages * d, 0);
  *out = s;
  return SV_OK;
}

void sv_sentinel_destroy(sv_sentinel* s) {
  if (!s) return;
  for (int kind = 0; kind < 2; ++kind) {
    for (float* p : s->m[kind]) (void)hipFree(p);
    for (sv_policy* p : s->pol[kind]) sv_policy_destroy(p);
  }
  if (s->res_dev) (void)hipFree(s->res_dev);
  if (s->sw_dev) (void)hipFree(s->sw_dev);
  if (s->mask_dev) (void)hipFree(s->mask_dev);
  if (s->sum_dev) (void)hipFree(s->sum_dev);
  for (int kind = 0; kind < 2; ++kind)
    for (float* p : s->pm[kind]) (void)hipFree(p);
  if (s->cproj) (void)hipFree(s->cproj);
  if (s->res_host) (void)hipHostFree(s->res_host);
  if (s->sw_host) (void)hipHostFree(s->sw_host);
  if (s->mask_host) (void)hipHostFree(s->mask_host);
  delete s;
}

const char* sv_sentinel_last_error(const sv_sentinel* s) { return s ? s->err : "sentinel is NULL"; }

sv_status sv_sentinel_begin_iteration(sv_sentinel* s, int32_t warmup) {
  if (!s) return SV_EINVAL;
  std::fill(s->tainted.begin(), s->tainted.end(), (uint8_t)0);
  s->warm = warmup != 0;
  return SV_OK;
}

sv_status sv_sentinel_forward(sv_sentinel* s, int32_t stage, const void* h, int32_t dtype, uint8_t* tainted_out, double* gamma_out,
                              void* stream) {
  if (!s) return SV_EINVAL;
  sv_status st = check_stage(s, stage, h, dtype, tainted_out);
  if (st != SV_OK) return st;
  hipStream_t hs = (hipStream_t)stream;
  const int d = s->cfg.n_workers, p = s->cfg.n_stages;
  std::vector<double> gamma;
  sv_policy* pol = s->pol[0][stage];
  std::vector<uint8_t> upstream(d, 0), banned(d, 0), skip(d, 0);
  if (!s->warm) {                                  // excluded whatever this check says: banned or tainted upstream
    for (int r = 0; r < d; ++r)
      for (int s2 = 0; s2 < p; ++s2) upstream[r] |= s->tainted[(size_t)s2 * d + r];
    SN_SV(s, sv_policy_state(pol, nullptr, banned.data(), nullptr, nullptr, nullptr, nullptr));
    for (int r = 0; r < d; ++r) skip[r] = banned[r] | upstream[r];
  }
  bool summed = false;
  float* pm = s->pm[0].empty() ? nullptr : s->pm[0][stage];
  st = gamma_of(s, h, dtype, s->m[0][stage], pm, skip.data(), &summed, gamma, hs);
  if (st != SV_OK) return st;
  if (gamma_out) memcpy(gamma_out, gamma.data(), gamma.size() * sizeof(double));
  uint8_t* excl = s->mask_host + d;
  if (s->warm) {
    SN_SV(s, sv_policy_warmup(pol, gamma.data()));
    for (int r = 0; r < d; ++r) { tainted_out[r] = 0; excl[r] = 0; }
  } else {
    SN_SV(s, sv_policy_step(pol, gamma.data(), upstream.data(), nullptr, tainted_out));
    SN_SV(s, sv_policy_state(pol, nullptr, banned.data(), nullptr, nullptr, nullptr, nullptr));
    for (int r = 0; r < d; ++r) {
      if (tainted_out[r]) s->tainted[(size_t)stage * d + r] = 1;
      excl[r] = banned[r] | upstream[r] | tainted_out[r];
    }
  }
  return update_ema(s, s->m[0][stage], pm, h, dtype, excl, skip.data(), summed, s->cfg.beta_h, hs);
}

sv_status sv_sentinel_backward(sv_sentinel* s, int32_t stage, void* g, int32_t dtype, uint8_t* tainted_out, double* gamma_out, void* stream) {
  if (!s) return SV_EINVAL;
  sv_status st = check_stage(s, stage, g, dtype, tainted_out);
  if (st != SV_OK) return st;
  hipStream_t hs = (hipStream_t)stream;
  const int d = s->cfg.n_workers, p = s->cfg.n_stages;
  std::vector<double> gamma;
  sv_policy* pol = s->pol[1][stage];
  std::vector<uint8_t> down(d, 0), banned(d, 0), skip(d, 0);
  if (!s->warm) {                                  // excluded whatever this check says (short of a majority reset): banned,
                                                   // tainted here on the way forward, or tainted at a later stage
    for (int r = 0; r < d; ++r)
      for (int s2 = stage + 1; s2 < p; ++s2) down[r] |= s->tainted[(size_t)s2 * d + r];
    SN_SV(s, sv_policy_state(pol, nullptr, banned.data(), nullptr, nullptr, nullptr, nullptr));
    for (int r = 0; r < d; ++r) skip[r] = banned[r] | s->tainted[(size_t)stage * d + r] | down[r];
  }
  bool summed = false;
  float* pm = s->pm[1].empty() ? nullptr : s->pm[1][stage];
  st = gamma_of(s, g, dtype, s->m[1][stage], pm, skip.data(), &summed, gamma, hs);
  if (st != SV_OK) return st;
  if (gamma_out) memcpy(gamma_out, gamma.data(), gamma.size() * sizeof(double));
  uint8_t* repl = s->mask_host;
  uint8_t* excl = s->mask_host + d;
  if (s->warm) {
    SN_SV(s, sv_policy_warmup(pol, gamma.data()));
    for (int r = 0; r < d; ++r) { tainted_out[r] = 0; repl[r] = 0; excl[r] = 0; }
  } else {
    SN_SV(s, sv_policy_step(pol, gamma.data(), nullptr, down.data(), tainted_out));
    SN_SV(s, sv_policy_state(pol, nullptr, banned.data(), nullptr, nullptr, nullptr, nullptr));
    for (int r = 0; r < d; ++r) {
      if (tainted_out[r]) s->tainted[(size_t)stage * d + r] = 1;
      repl[r] = s->tainted[(size_t)stage * d + r];           // includes a forward-pass taint at this very stage
      excl[r] = banned[r] | repl[r];
    }
  }
  SN_HIP(s, hipMemcpyAsync(s->mask_dev, s->mask_host, 2 * (size_t)d, hipMemcpyHostToDevice, hs));
  // the EMA reads only signals that are not replaced, and the replacement reads m before it is updated
  bool any_repl = false;
  for (int r = 0; r < d; ++r) any_repl |= repl[r] != 0;
  if (any_repl) SN_SV(s, sv_replace_with_ema(s->ctx, g, s->cfg.T * s->cfg.D, d, dtype, s->mask_dev, s->m[1][stage], s->cfg.T, s->cfg.D, hs));
  // (the sum the score pass left was taken before the replacement, over signals that are not replaced)
  return update_ema(s, s->m[1][stage], pm, g, dtype, excl, skip.data(), summed, s->cfg.beta_g, hs, /*mask_uploaded=*/true);
}

sv_status sv_sentinel_state(const sv_sentinel* s, int32_t stage, int32_t kind, const float** ema_dev, int32_t* violations, uint8_t* banned,
                            double* lower, double* upper, double* k) {
  if (!s || stage < 0 || stage >= s->cfg.n_stages || (kind != 0 && kind != 1)) return SV_EINVAL;
  if (ema_dev) *ema_dev = s->m[kind][stage];
  return sv_policy_state(s->pol[kind][stage], violations, banned, lower, upper, k, nullptr);
}

sv_status sv_sentinel_counters(const sv_sentinel* s, int64_t* counts) {
  if (!s || !counts) return SV_EINVAL;
  counts[0] = s->n_calls; counts[1] = s->n_from_sum; counts[2] = s->n_from_signals; counts[3] = s->n_sw_carried;
  return SV_OK;
}

sv_status sv_sentinel_read_ema(sv_sentinel* s, int32_t stage, int32_t kind, float* out_host, void* stream) {
  if (!s || stage < 0 || stage >= s->cfg.n_stages || (kind != 0 && kind != 1) || !out_host) return SV_EINVAL;
  hipStream_t hs = (hipStream_t)stream;
  SN_HIP(s, hipMemcpyAsync(out_host, s->m[kind][stage], (size_t)s->cfg.T * s->cfg.D * sizeof(float), hipMemcpyDeviceToHost, hs));
  SN_HIP(s, hipStreamSynchronize(hs));
  return SV_OK;
}

}  // extern "C"
