"""CPU oracle for the stage verifier -- TEST INFRASTRUCTURE, not a product path.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this
file.  It shares no code with the HIP library and is never used to produce a result
the library returns.

What it defines, slowly and in float64 throughout (inputs are widened, nothing is
rounded in between):

* the stage map  h^(s) = f_s(h^(s-1); theta^(s))  and the activation gradient
  g^(s) = d L / d h^(s-1)  of the paper's threat model (Problem Statement, "Threat
  Model" paragraph).  The paper does not print f_s; it trains Llama-3 and NanoGPT
  decoder stacks, so f_s is n_blocks pre-norm decoder blocks:
      x1 = x + Attn(Norm1(x)) Wo^T ,   y = x1 + MLP(Norm2(x1))
  with RMSNorm + RoPE + SwiGLU (Llama style) or LayerNorm + exact-erf GELU (GPT style).
  This is what a duplicate-work verifier recomputes (the recompute-and-compare
  baseline of the paper's "Proposed Method" paragraph and FAQ Q9).
  The paper's "Alternative Architectures" paragraph also trains two mixture-of-experts
  stacks and Table model_config gives their expert count, shared-expert count and top-k,
  but no formula for the layer.  With desc.n_experts > 0 the MLP of a block is the generic
  routed layer those architectures share:
      l = n Wr^T,   s = sigmoid(l) or softmax(l),   S_t = the top_k experts of token t by s
      (decided on l, which orders the experts as s does; ties to the lower index),   g = s on S_t, divided by its sum over S_t if router_norm,
      MLP(n) = sum_{e in S_t} g_e SwiGLU_e(n) + sum_{shared experts} SwiGLU_sh(n),
  every expert a SwiGLU feed-forward of width ffn_hidden; no capacity limit, no token is
  dropped, no load-balancing term (none of them changes the forward value).
* the test statistic Gamma = Omega(signal, reference) and the flag rule Gamma > tau
  (Eq. test_statistic), with the distance family of the paragraph "Choice of Distance
  Measure": mean absolute difference, normalised (z-scored) Euclidean distance and sign
  flip ratio, plus the per-token relative L2 the benchmark thresholds are stated in.
  A submission is flagged when any enabled metric exceeds its threshold.
* the EMA reference update of Eq. momentum_def restricted to the un-flagged set
  R_clean as in Alg. momentum_verification (flagged signals never enter the EMA).

Parity pins live in tests/test_oracle_*.py: brute-force loops on tiny shapes, central
finite differences, adjoint identity, structural special cases and closed-form scores of
the attack variants.  Parts with no pin are listed as "parity unpinned": none here.

Array conventions: activations [B, S, D] (or [T, D] per sequence), weights [out, in].
`desc` is any object with attributes n_blocks, d_model, n_heads, n_kv_heads, ffn_hidden,
mlp ("swiglu"|"gelu"), norm ("rms"|"ln"), rope, causal, norm_eps, rope_theta and, optionally,
n_experts (0 = dense MLP), top_k, n_shared, router_score ("sigmoid"|"softmax"), router_norm.
Mixture-of-experts weights: w_router [E, D], w_gate / w_up [E, F, D], w_down [E, D, F] and, with
shared experts, ws_gate / ws_up [n_shared * F, D], ws_down [D, n_shared * F] (the shared experts
side by side: expert i owns rows / columns i*F .. (i+1)*F).
"""
from __future__ import annotations

import math

import numpy as np

try:  # exact erf for the GELU; scipy is a plain library primitive here
    from scipy.special import erf as _erf
except Exception:  # pragma: no cover
    _erf = np.vectorize(math.erf, otypes=[np.float64])

F64 = np.float64
METRICS = ("rel_l2", "l1", "zl2", "sfr")


def _f64(a):
    return None if a is None else np.asarray(a, dtype=F64)


# ----------------------------------------------------------------------------- norms
def norm_forward(x, gain, bias, kind, eps):
    """RMSNorm: x / sqrt(mean(x^2)+eps) * g.  LayerNorm: (x-mu)/sqrt(var_pop+eps) * g + b."""
    x = _f64(x)
    if kind == "rms":
        r = np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps)
        return x / r * gain
    mu = np.mean(x, axis=-1, keepdims=True)
    var = np.mean((x - mu) ** 2, axis=-1, keepdims=True)
    return (x - mu) / np.sqrt(var + eps) * gain + bias


def norm_backward(dn, x, gain, kind, eps):
    """Gradient of norm_forward with respect to x (gain/bias gradients are not needed)."""
    x, dn = _f64(x), _f64(dn)
    D = x.shape[-1]
    gd = dn * gain
    if kind == "rms":
        r = np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps)
        return gd / r - x * np.sum(gd * x, axis=-1, keepdims=True) / (D * r ** 3)
    mu = np.mean(x, axis=-1, keepdims=True)
    sd = np.sqrt(np.mean((x - mu) ** 2, axis=-1, keepdims=True) + eps)
    xh = (x - mu) / sd
    return (gd - np.mean(gd, axis=-1, keepdims=True) - xh * np.mean(gd * xh, axis=-1, keepdims=True)) / sd


# ----------------------------------------------------------------------------- RoPE
def rope_rotate(x, theta, inverse=False):
    """x [S, n_heads, hd]; token p, pair (2i, 2i+1) rotated by angle p * theta^(-2i/hd).
    inverse=True rotates by the negative angle (the transpose of the rotation)."""
    x = _f64(x)
    S, _, hd = x.shape
    i = np.arange(hd // 2, dtype=F64)
    ang = np.arange(S, dtype=F64)[:, None] * theta ** (-2.0 * i / hd)[None, :]      # [S, hd/2]
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    if inverse:
        s = -s
    a, b = x[..., 0::2], x[..., 1::2]
    out = np.empty_like(x)
    out[..., 0::2] = a * c - b * s
    out[..., 1::2] = a * s + b * c
    return out


# ----------------------------------------------------------------------------- attention
def _probabilities(qh, kh, causal):
    S, hd = qh.shape
    s = qh @ kh.T / math.sqrt(hd)
    if causal:
        s = np.where(np.tril(np.ones((S, S), dtype=bool)), s, -np.inf)
    s = s - np.max(s, axis=-1, keepdims=True)
    e = np.exp(s)
    return e / np.sum(e, axis=-1, keepdims=True)


def attention_forward(q, k, v, causal):
    """q [S, H, hd], k/v [S, Hkv, hd] of one sequence -> o [S, H, hd].
    Query head h reads kv head h // (H // Hkv)."""
    S, H, hd = q.shape
    G = H // k.shape[1]
    o = np.empty((S, H, hd), dtype=F64)
    for h in range(H):
        P = _probabilities(q[:, h], k[:, h // G], causal)
        o[:, h] = P @ v[:, h // G]
    return o


def attention_backward(do, q, k, v, causal):
    """Gradients (dq, dk, dv) of attention_forward; dk, dv sum over the query heads of a group."""
    S, H, hd = q.shape
    G = H // k.shape[1]
    dq, dk, dv = np.zeros_like(q), np.zeros_like(k), np.zeros_like(v)
    for h in range(H):
        kv = h // G
        P = _probabilities(q[:, h], k[:, kv], causal)
        dv[:, kv] += P.T @ do[:, h]
        dP = do[:, h] @ v[:, kv].T
        dS = P * (dP - np.sum(P * dP, axis=-1, keepdims=True))
        dq[:, h] = dS @ k[:, kv] / math.sqrt(hd)
        dk[:, kv] += dS.T @ q[:, h] / math.sqrt(hd)
    return dq, dk, dv


# ----------------------------------------------------------------------------- MLP pieces
def silu(z):
    return z / (1.0 + np.exp(-z))


def silu_grad(z):
    s = 1.0 / (1.0 + np.exp(-z))
    return s * (1.0 + z * (1.0 - s))


def gelu(z):
    return 0.5 * z * (1.0 + _erf(z / math.sqrt(2.0)))


def gelu_grad(z):
    return 0.5 * (1.0 + _erf(z / math.sqrt(2.0))) + z * np.exp(-0.5 * z * z) / math.sqrt(2.0 * math.pi)



# ----------------------------------------------------------------------------- mixture of experts
def router_scores_from_logits(logits, kind):
    if kind == "sigmoid":
        return 1.0 / (1.0 + np.exp(-logits))
    if kind == "softmax":
        e = np.exp(logits - np.max(logits, axis=-1, keepdims=True))
        return e / np.sum(e, axis=-1, keepdims=True)
    raise ValueError(kind)


def router_scores(n, w_router, kind):
    """Router scores [S, E] of the tokens n [S, D]: sigmoid or softmax of the logits n Wr^T."""
    return router_scores_from_logits(_f64(n) @ _f64(w_router).T, kind)


def moe_route(n, w_router, desc):
    """Which experts each token uses and with what weight.

    Returns (sel [S, k] expert indices in decreasing score order, gates [S, k], scores [S, E],
    margin [S], logits [S, E]).  Both score functions increase with the logit, so "the k highest
    scores" is decided on the logits (which do not saturate); ties go to the lower index.  margin is
    the gap between the k-th and (k+1)-th logit (inf when k = E): how far the token is from a
    different routing.  Everything is float64; a recomputation in a lower precision may legitimately
    choose differently for a token whose margin is within that precision's error of the logits --
    what counts as legitimate is for the comparing test to state, not for this function."""
    n = _f64(n)
    E, k = desc.n_experts, desc.top_k
    logits = n @ _f64(w_router).T
    scores = router_scores_from_logits(logits, desc.router_score)
    order = np.argsort(-logits, axis=-1, kind="stable")         # decreasing logit, ties to the lower index
    sel = order[:, :k]
    srt = np.take_along_axis(logits, order, axis=-1)
    margin = srt[:, k - 1] - srt[:, k] if k < E else np.full(n.shape[0], np.inf)
    gates = np.take_along_axis(scores, sel, axis=-1)
    if desc.router_norm:
        gates = gates / np.sum(gates, axis=-1, keepdims=True)
    return sel, gates, scores, margin, logits


def _shared_slices(w, desc):
    F = desc.ffn_hidden
    return [slice(i * F, (i + 1) * F) for i in range(getattr(desc, "n_shared", 0))]


def moe_forward(n, w, desc, keep=False):
    """The routed MLP of the tokens n [S, D] -> [S, D] (without the residual)."""
    n = _f64(n)
    sel, gates, scores, margin, logits = moe_route(n, w["w_router"], desc)
    Wg, Wu, Wd = _f64(w["w_gate"]), _f64(w["w_up"]), _f64(w["w_down"])
    out = np.zeros_like(n)
    for e in range(desc.n_experts):
        tok, slot = np.nonzero(sel == e)                       # the tokens routed to expert e
        if tok.size == 0:
            continue
        x = n[tok]
        y = (silu(x @ Wg[e].T) * (x @ Wu[e].T)) @ Wd[e].T
        np.add.at(out, tok, gates[tok, slot][:, None] * y)
    for sl in _shared_slices(w, desc):
        out += (silu(n @ _f64(w["ws_gate"])[sl].T) * (n @ _f64(w["ws_up"])[sl].T)) @ _f64(w["ws_down"])[:, sl].T
    if keep:
        return out, dict(n=n, sel=sel, gates=gates, scores=scores, margin=margin, logits=logits)
    return out


def moe_backward(dy, st, w, desc):
    """Gradient of moe_forward with respect to its input tokens, for the routing kept in `st`
    (the routing is piecewise constant; its decision carries no gradient, its gate values do)."""
    dy = _f64(dy)
    n, sel, gates, scores = st["n"], st["sel"], st["gates"], st["scores"]
    Wg, Wu, Wd, Wr = _f64(w["w_gate"]), _f64(w["w_up"]), _f64(w["w_down"]), _f64(w["w_router"])
    dn = np.zeros_like(n)
    dgates = np.zeros_like(gates)
    for e in range(desc.n_experts):
        tok, slot = np.nonzero(sel == e)
        if tok.size == 0:
            continue
        x, d = n[tok], dy[tok]
        gt, up = x @ Wg[e].T, x @ Wu[e].T
        y = (silu(gt) * up) @ Wd[e].T
        dgates[tok, slot] = np.sum(d * y, axis=-1)
        da = (gates[tok, slot][:, None] * d) @ Wd[e]
        np.add.at(dn, tok, (da * up * silu_grad(gt)) @ Wg[e] + (da * silu(gt)) @ Wu[e])
    # gate values -> selected scores
    ssel = np.take_along_axis(scores, sel, axis=-1)
    if desc.router_norm:
        z = np.sum(ssel, axis=-1, keepdims=True)
        dssel = (dgates - np.sum(dgates * gates, axis=-1, keepdims=True)) / z
    else:
        dssel = dgates
    dscores = np.zeros_like(scores)
    np.put_along_axis(dscores, sel, dssel, axis=-1)
    # scores -> logits
    if desc.router_score == "sigmoid":
        dlogits = dscores * scores * (1.0 - scores)
    else:
        dlogits = scores * (dscores - np.sum(dscores * scores, axis=-1, keepdims=True))
    dn += dlogits @ Wr
    for sl in _shared_slices(w, desc):
        Wsg, Wsu, Wsd = _f64(w["ws_gate"])[sl], _f64(w["ws_up"])[sl], _f64(w["ws_down"])[:, sl]
        gt, up = n @ Wsg.T, n @ Wsu.T
        da = dy @ Wsd
        dn += (da * up * silu_grad(gt)) @ Wsg + (da * silu(gt)) @ Wsu
    return dn


# ----------------------------------------------------------------------------- one block, one sequence
def block_forward(x, w, desc, keep=False):
    """x [S, D] of ONE sequence -> y [S, D]; with keep=True also the tensors backward needs."""
    x = _f64(x)
    S, D = x.shape
    H, Hkv = desc.n_heads, desc.n_kv_heads
    hd = D // H
    n1 = norm_forward(x, _f64(w["norm1_g"]), _f64(w["norm1_b"]), desc.norm, desc.norm_eps)
    q = (n1 @ _f64(w["wq"]).T).reshape(S, H, hd)
    k = (n1 @ _f64(w["wk"]).T).reshape(S, Hkv, hd)
    v = (n1 @ _f64(w["wv"]).T).reshape(S, Hkv, hd)
    if desc.rope:
        q, k = rope_rotate(q, desc.rope_theta), rope_rotate(k, desc.rope_theta)
    o = attention_forward(q, k, v, desc.causal).reshape(S, H * hd)
    x1 = x + o @ _f64(w["wo"]).T
    n2 = norm_forward(x1, _f64(w["norm2_g"]), _f64(w["norm2_b"]), desc.norm, desc.norm_eps)
    if getattr(desc, "n_experts", 0) > 0:
        mo = moe_forward(n2, w, desc, keep)
        if keep:
            return x1 + mo[0], dict(x=x, q=q, k=k, v=v, x1=x1, moe=mo[1])
        return x1 + mo
    u = n2 @ _f64(w["w_up"]).T
    if desc.mlp == "swiglu":
        gt = n2 @ _f64(w["w_gate"]).T
        a = silu(gt) * u
    else:
        gt = None
        a = gelu(u)
    y = x1 + a @ _f64(w["w_down"]).T
    if keep:
        return y, dict(x=x, q=q, k=k, v=v, x1=x1, gate=gt, up=u)
    return y


def block_backward(dy, st, w, desc):
    """dy = dL/dy [S, D] -> dL/dx [S, D] for one sequence (no weight gradients)."""
    dy = _f64(dy)
    S, D = dy.shape
    H, Hkv = desc.n_heads, desc.n_kv_heads
    hd = D // H
    if "moe" in st:
        dn2 = moe_backward(dy, st["moe"], w, desc)
    elif desc.mlp == "swiglu":
        da = dy @ _f64(w["w_down"])
        dgate = da * st["up"] * silu_grad(st["gate"])
        dup = da * silu(st["gate"])
        dn2 = dgate @ _f64(w["w_gate"]) + dup @ _f64(w["w_up"])
    else:
        da = dy @ _f64(w["w_down"])
        dn2 = (da * gelu_grad(st["up"])) @ _f64(w["w_up"])
    dx1 = dy + norm_backward(dn2, st["x1"], _f64(w["norm2_g"]), desc.norm, desc.norm_eps)
    do = (dx1 @ _f64(w["wo"])).reshape(S, H, hd)
    dq, dk, dv = attention_backward(do, st["q"], st["k"], st["v"], desc.causal)
    if desc.rope:
        dq = rope_rotate(dq, desc.rope_theta, inverse=True)
        dk = rope_rotate(dk, desc.rope_theta, inverse=True)
    dn1 = (dq.reshape(S, H * hd) @ _f64(w["wq"]) + dk.reshape(S, Hkv * hd) @ _f64(w["wk"])
           + dv.reshape(S, Hkv * hd) @ _f64(w["wv"]))
    return dx1 + norm_backward(dn1, st["x"], _f64(w["norm1_g"]), desc.norm, desc.norm_eps)


# ----------------------------------------------------------------------------- the stage
def stage_forward(h, weights, desc):
    """h^(s-1) [B, S, D] -> h^(s) [B, S, D]: n_blocks blocks applied to each sequence."""
    h = _f64(h)
    out = np.empty_like(h)
    for b in range(h.shape[0]):
        x = h[b]
        for w in weights:
            x = block_forward(x, w, desc)
        out[b] = x
    return out


def stage_routing_margin(h, weights, desc):
    """Mixture-of-experts stages: per token [B, S], the smallest routing margin over the blocks of
    the stage (see moe_route).  Tokens with a small margin are those whose expert set a
    recomputation in another precision may legitimately choose differently."""
    h = _f64(h)
    out = np.empty(h.shape[:2], dtype=F64)
    for b in range(h.shape[0]):
        x, m = h[b], np.full(h.shape[1], np.inf)
        for w in weights:
            x, st = block_forward(x, w, desc, keep=True)
            m = np.minimum(m, st["moe"]["margin"])
        out[b] = m
    return out


def stage_backward(h, g_next, weights, desc):
    """(h^(s-1), dL/dh^(s)) -> (h^(s), g^(s) = dL/dh^(s-1)); the forward is recomputed and
    kept per sequence, then the blocks are walked in reverse."""
    h, g_next = _f64(h), _f64(g_next)
    h_out, g = np.empty_like(h), np.empty_like(h)
    for b in range(h.shape[0]):
        x, kept = h[b], []
        for w in weights:
            x, st = block_forward(x, w, desc, keep=True)
            kept.append(st)
        h_out[b] = x
        d = g_next[b]
        for w, st in zip(reversed(weights), reversed(kept)):
            d = block_backward(d, st, w, desc)
        g[b] = d
    return h_out, g


# ----------------------------------------------------------------------------- the check
def _sgn(a):
    return (a > 0).astype(np.int8) - (a < 0).astype(np.int8)


def token_rel_l2(claim, ref):
    """Per-token ||c_t - r_t||_2 / max(||r_t||_2, 1e-30) over the feature axis -> [T]."""
    c = _f64(claim).reshape(-1, np.shape(claim)[-1])
    r = _f64(ref).reshape(c.shape)
    return np.sqrt(np.sum((c - r) ** 2, axis=1)) / np.maximum(np.sqrt(np.sum(r * r, axis=1)), 1e-30)


def scores(claim, ref, reduce="max_token"):
    """All four statistics between one submission and its reference point.

    rel_l2 : max over tokens of the per-token relative L2 (reduce="max_token"), or
             ||c - r||_F / ||r||_F over the whole signal (reduce="global").
    l1     : mean |c - r| over all elements.
    zl2    : mean squared difference of the z-scored signals (scalar mean / population std
             over the flattened tensor); equals 2 (1 - corr(c, r)).  A constant signal has
             no z-score: both constant -> 0, exactly one constant -> 2.
    sfr    : fraction of elements whose signs differ, with sign(0) = 0.
    """
    c, r = _f64(claim).ravel(), _f64(ref).ravel()
    n = c.size
    out = {}
    if reduce == "max_token":
        out["rel_l2"] = float(np.max(token_rel_l2(claim, ref)))
    elif reduce == "global":
        out["rel_l2"] = float(np.sqrt(np.sum((c - r) ** 2)) / max(np.sqrt(np.sum(r * r)), 1e-30))
    else:
        raise ValueError(reduce)
    out["l1"] = float(np.sum(np.abs(c - r)) / n)
    const_c, const_r = bool(np.max(c) == np.min(c)), bool(np.max(r) == np.min(r))
    if const_c and const_r:
        out["zl2"] = 0.0
    elif const_c or const_r:
        out["zl2"] = 2.0
    else:
        out["zl2"] = float(np.mean(((c - np.mean(c)) / np.std(c) - (r - np.mean(r)) / np.std(r)) ** 2))
    out["sfr"] = float(np.count_nonzero(_sgn(c) != _sgn(r)) / n)
    return out


def flag(score_by_metric, tau_by_metric):
    """Flag when any enabled metric is strictly above its threshold.  A score that is not a
    number (a submission carrying NaN/inf) cannot be shown to be within the threshold and is
    flagged too: the rule is "not (Gamma <= tau)", which equals "Gamma > tau" on the reals."""
    return any(not (score_by_metric[m] <= tau_by_metric[m]) for m in tau_by_metric)


def ema_update(m, signals, flags, beta):
    """m_t = beta m_{t-1} + (1-beta) * mean of the un-flagged signals; unchanged if none is clean."""
    m = _f64(m)
    clean = [_f64(x) for x, f in zip(signals, flags) if not f]
    if not clean:
        return m.copy()
    acc = np.zeros_like(m)
    for x in clean:
        acc += x.reshape(m.shape)
    return beta * m + (1.0 - beta) * acc / len(clean)
