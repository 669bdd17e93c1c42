"""CPU oracle for the verifier's remaining statistic and its decision policy -- TEST
INFRASTRUCTURE, not a product path.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this file.
It shares no code with the HIP / C++ library.

What it defines (float64, plain numpy, one function per passage):

* sliced_wasserstein      -- Omega_SW of the paragraph "Choice of Distance Measure": the mean
                             over random unit directions u of the 1-Wasserstein distance
                             between the projections of the two signals onto u.
* percentiles / tukey_flag-- q1, q2, q3 of a history window and the fence test of
                             Eq. tukey_fences (flag iff |Gamma - q2| >= k (q3 - q1)).
* adaptive_iqr            -- Alg. adaptive_iqr: widen / narrow the multiplier k until the
                             fraction of the history outside the fences matches the target
                             false-positive rate, then enforce a minimum distance from the median.
* SentinelStream          -- Alg. momentum_verification end to end on a stream of per-stage signals:
                             warm-up, Gamma against the EMA, the policy, taint propagation between
                             stages, gradient replacement (Alg. gradient_replacement), EMA updates
                             over the clean set.
* StagePolicy             -- the bookkeeping of Alg. activation_verification /
                             Alg. gradient_verification for one stage: violation counters with
                             forgiveness, bans (after c violations, or at once for a deviation
                             100 times the fence half-width), the history of clean deviations,
                             the per-iteration tainted set and its ">50 % flagged" reset.

Readings where the paper is silent or at odds with itself (the same list is in the design notes):
  - the samples of the two distributions are the T token vectors in R^D; L directions are an
    input (drawn by the caller from N(0, I) and normalised); with equal sample counts the
    1-Wasserstein distance of two empirical distributions on the line is the mean absolute
    difference of the sorted samples;
  - percentiles use linear interpolation between order statistics (position (n-1) p);
  - "outside [lower, upper]" is strict (x < lower or x > upper);
  - "FP-rate << alpha" is read as FP-rate < alpha / 10;
  - the multiplier carried into a call is the one the previous call returned (k_0 on the first);
  - the history is cut to its last l VALUES (the algorithm's slice), not l iterations, and it is cut
    where Alg. activation_verification / Alg. gradient_verification cut it: at the START of a
    verified call, so that Alg. adaptive_iqr at the end of the call sees the l kept values plus
    this call's clean ones (up to l + d values).  The warm-up listing neither cuts nor adapts; here
    a warm-up iteration appends its values, keeps the last l, and adapts, so that fences exist
    when the first verified call tests against them;
  - the flag test uses the bounds Alg. adaptive_iqr returned: flagged iff
    Gamma <= lower or Gamma >= upper (the ">=" of Eq. tukey_fences); before any history exists
    nothing is flagged;
  - ">>" in the ban rule: |Gamma - q2| >= 100 k IQR for some metric;
  - forgiveness: after T_forgiveness consecutive clean steps the counter drops by one and the
    streak starts again.

Pins: tests/test_oracle_sentinel.py.  Parts with no pin ("parity unpinned"): none.
"""
from __future__ import annotations

import numpy as np

F64 = np.float64


# ------------------------------------------------------------------ sliced Wasserstein
def sliced_wasserstein(claim, ref, directions):
    """Omega_SW(claim, ref).  claim, ref: [T, D] (leading dims are flattened into T);
    directions: [L, D].  Returns the mean over the L directions of W1 between the projected
    sample sets."""
    d = np.asarray(directions, dtype=F64)
    c = np.asarray(claim, dtype=F64).reshape(-1, d.shape[1])
    r = np.asarray(ref, dtype=F64).reshape(-1, d.shape[1])
    pc = c @ d.T                                  # [T, L]: sample t projected on direction l
    pr = r @ d.T
    w1 = np.mean(np.abs(np.sort(pc, axis=0) - np.sort(pr, axis=0)), axis=0)
    return float(np.mean(w1))


# ------------------------------------------------------------------ Tukey fences
def percentiles(history):
    """25th, 50th and 75th percentiles with linear interpolation between order statistics."""
    h = np.sort(np.asarray(history, dtype=F64))
    n = h.shape[0]
    out = []
    for p in (0.25, 0.5, 0.75):
        pos = (n - 1) * p
        lo = int(np.floor(pos))
        hi = min(lo + 1, n - 1)
        out.append(h[lo] + (h[hi] - h[lo]) * (pos - lo))
    return tuple(out)


def tukey_flag(gamma, q1, q2, q3, k):
    """Eq. tukey_fences."""
    return bool(abs(gamma - q2) >= k * (q3 - q1))


def _fp_rate(h, lower, upper):
    return float(np.mean((h < lower) | (h > upper)))


def adaptive_iqr(history, k_prev, alpha, grow, shrink, n_max, min_dist_mult, eps):
    """Alg. adaptive_iqr.  Returns (lower, upper, k)."""
    h = np.asarray(history, dtype=F64)
    q1, q2, q3 = percentiles(h)
    iqr = max(q3 - q1, eps)
    k = float(k_prev)
    lower, upper = q2 - k * iqr, q2 + k * iqr
    fp = _fp_rate(h, lower, upper)
    it = 0
    while fp > alpha and it < n_max:              # too many benign values outside: widen
        k *= grow
        lower, upper = q2 - k * iqr, q2 + k * iqr
        fp = _fp_rate(h, lower, upper)
        it += 1
    it = 0
    while fp < alpha / 10.0 and it < n_max:       # far fewer than the target: narrow
        k *= shrink
        lower, upper = q2 - k * iqr, q2 + k * iqr
        fp = _fp_rate(h, lower, upper)
        it += 1
    d_min = abs(q2) * min_dist_mult
    lower = min(lower, q2 - d_min)
    upper = max(upper, q2 + d_min)
    return lower, upper, k


# ------------------------------------------------------------------ per-stage policy
class StagePolicy:
    """State one verifier keeps for one stage and one signal kind (Alg. momentum_verification's
    v_r, B_s, H_l plus the fences of every metric)."""

    def __init__(self, n_workers, n_metrics, *, c=5, t_forgive=100, window=100, k0=1.5, alpha=0.01,
                 grow=1.1, shrink=0.9, n_max=10, min_dist_mult=0.0, eps=1e-3, severe=100.0):
        self.d, self.m = n_workers, n_metrics
        self.c, self.t_forgive, self.window = c, t_forgive, window
        self.alpha, self.grow, self.shrink, self.n_max = alpha, grow, shrink, n_max
        self.min_dist_mult, self.eps, self.severe = min_dist_mult, eps, severe
        self.v = [0] * n_workers
        self.streak = [0] * n_workers
        self.banned = [False] * n_workers
        self.hist = [[] for _ in range(n_metrics)]
        self.k = [float(k0)] * n_metrics
        self.lower = [-np.inf] * n_metrics
        self.upper = [np.inf] * n_metrics
        self.q2 = [0.0] * n_metrics
        self.iqr = [np.inf] * n_metrics

    def _truncate(self):
        for i in range(self.m):
            self.hist[i] = self.hist[i][-self.window:]

    def _update_fences(self):
        for i in range(self.m):
            if not self.hist[i]:
                continue
            lo, up, k = adaptive_iqr(self.hist[i], self.k[i], self.alpha, self.grow, self.shrink,
                                     self.n_max, self.min_dist_mult, self.eps)
            q1, q2, q3 = percentiles(self.hist[i])
            self.lower[i], self.upper[i], self.k[i] = lo, up, k
            self.q2[i], self.iqr[i] = q2, max(q3 - q1, self.eps)

    def warmup(self, gamma):
        """Warm-up iteration: every worker's deviation enters the history, nothing is flagged."""
        g = np.asarray(gamma, dtype=F64)
        for r in range(self.d):
            for i in range(self.m):
                self.hist[i].append(float(g[r, i]))
        self._truncate()
        self._update_fences()

    def step(self, gamma, skip=None, pre_tainted=None):
        """One verified iteration.  gamma [d, m]; skip[r] true for workers that are not examined
        (already tainted by another stage in this iteration, or absent); pre_tainted[r] true for
        workers that enter this stage's tainted set without being examined (tainted downstream, in
        the backward pass).  Returns the list of workers tainted at this stage."""
        g = np.asarray(gamma, dtype=F64)
        tainted = []
        self._truncate()                               # the listing's second line: before anything is examined
        for r in range(self.d):
            if self.banned[r]:
                continue
            if pre_tainted is not None and pre_tainted[r]:
                tainted.append(r)
                continue
            if skip is not None and skip[r]:
                continue
            violated = any((not (g[r, i] > self.lower[i])) or (not (g[r, i] < self.upper[i])) for i in range(self.m))
            if violated:
                self.v[r] += 1
                self.streak[r] = 0
                tainted.append(r)
                severe = any(abs(g[r, i] - self.q2[i]) >= self.severe * self.k[i] * self.iqr[i] for i in range(self.m))
                if self.v[r] >= self.c or severe:
                    self.banned[r] = True
            else:
                for i in range(self.m):
                    self.hist[i].append(float(g[r, i]))
                self.streak[r] += 1
                if self.streak[r] >= self.t_forgive:
                    self.v[r] = max(0, self.v[r] - 1)
                    self.streak[r] = 0
        self._update_fences()
        active = self.d - sum(self.banned)
        if len(tainted) > 0.5 * active:
            tainted = []
        return tainted


# ------------------------------------------------------------------ the whole verifier loop
def _sgn(a):
    return (a > 0).astype(np.int8) - (a < 0).astype(np.int8)


def global_scores(x, m):
    """The paper's statistics of one signal against the reference point, each over the whole
    flattened signal: relative L2, mean absolute difference, z-scored squared distance, sign flip
    ratio (sign(0) = 0).  A constant side has no z-score: both constant -> 0, one -> 2."""
    c, r = np.asarray(x, F64).ravel(), np.asarray(m, F64).ravel()
    out = {"rel_l2": float(np.sqrt(np.sum((c - r) ** 2)) / max(np.sqrt(np.sum(r * r)), 1e-30)),
           "l1": float(np.mean(np.abs(c - r)))}
    cc, cr = bool(np.max(c) == np.min(c)), bool(np.max(r) == np.min(r))
    if cc and cr:
        out["zl2"] = 0.0
    elif cc or cr:
        out["zl2"] = 2.0
    else:
        out["zl2"] = float(np.mean(((c - c.mean()) / c.std() - (r - r.mean()) / r.std()) ** 2))
    out["sfr"] = float(np.mean(_sgn(c) != _sgn(r)))
    return out


class SentinelStream:
    """Alg. momentum_verification with its three sub-procedures, for p stages and d workers per
    stage (worker r of every stage belongs to the same data-parallel pipe).  Signals are handed in
    stage by stage: forward(s, h) for s = 0 .. p-1, then backward(s, g) for s = p-1 .. 0.

    Readings: Gamma uses the whole-signal form of every statistic; in the forward pass a worker whose
    pipe was tainted at an earlier stage of this iteration is neither examined nor allowed into the
    EMA (the text's "pause their deviation statistics"; the listing's R_clean alone would let it in);
    in the backward pass R_clean is the listing's: everything not tainted at this stage; banned
    workers are never examined and never enter an EMA; m_0 = 0."""

    METRICS = ("rel_l2", "l1", "zl2", "sfr", "sw")

    def __init__(self, n_stages, n_workers, shape, metrics, directions, beta_h, beta_g, policy_h, policy_g):
        self.p, self.d, self.shape = n_stages, n_workers, tuple(shape)
        self.metrics = [m for m in self.METRICS if m in metrics]
        self.dirs = directions
        self.beta = {"h": beta_h, "g": beta_g}
        self.m = {k: [np.zeros(self.shape, F64) for _ in range(n_stages)] for k in "hg"}
        self.pol = {"h": [StagePolicy(n_workers, len(self.metrics), **policy_h) for _ in range(n_stages)],
                    "g": [StagePolicy(n_workers, len(self.metrics), **policy_g) for _ in range(n_stages)]}
        self.tainted = set()          # (stage, worker) pairs of the current iteration
        self.warm = True

    def begin_iteration(self, warmup):
        self.tainted = set()
        self.warm = bool(warmup)

    def gamma(self, signals, m):
        out = np.zeros((self.d, len(self.metrics)), F64)
        for r, x in enumerate(signals):
            sc = global_scores(x, m)
            if "sw" in self.metrics:
                sc["sw"] = sliced_wasserstein(x, m, self.dirs)
            out[r] = [sc[k] for k in self.metrics]
        return out

    def _ema(self, kind, s, signals, excluded):
        clean = [np.asarray(x, F64).reshape(self.shape) for x, e in zip(signals, excluded) if not e]
        if clean:
            b = self.beta[kind]
            self.m[kind][s] = b * self.m[kind][s] + (1.0 - b) * sum(clean) / len(clean)

    def forward(self, s, h):
        """Alg. activation_verification + the EMA update of the main loop.  Returns (tainted here, Gamma)."""
        pol, g = self.pol["h"][s], self.gamma(h, self.m["h"][s])
        if self.warm:
            pol.warmup(g)
            self._ema("h", s, h, [False] * self.d)
            return [], g
        upstream = [any((s2, r) in self.tainted for s2 in range(self.p)) for r in range(self.d)]
        here = pol.step(g, skip=upstream)
        self.tainted |= {(s, r) for r in here}
        excluded = [pol.banned[r] or upstream[r] or r in here for r in range(self.d)]
        self._ema("h", s, h, excluded)
        return here, g

    def backward(self, s, grads):
        """Alg. gradient_verification + Alg. gradient_replacement + the EMA update.  grads: list of d
        arrays; returns (tainted here, Gamma, grads with the tainted ones replaced by m_{t-1}(g))."""
        pol, g = self.pol["g"][s], self.gamma(grads, self.m["g"][s])
        if self.warm:
            pol.warmup(g)
            self._ema("g", s, grads, [False] * self.d)
            return [], g, list(grads)
        down = [any((s2, r) in self.tainted for s2 in range(s + 1, self.p)) for r in range(self.d)]
        here = pol.step(g, pre_tainted=down)
        self.tainted |= {(s, r) for r in here}
        at_stage = [(s, r) in self.tainted for r in range(self.d)]
        out = [self.m["g"][s].copy() if at_stage[r] else grads[r] for r in range(self.d)]
        excluded = [pol.banned[r] or at_stage[r] for r in range(self.d)]
        self._ema("g", s, grads, excluded)
        return here, g, out
