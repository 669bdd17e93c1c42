"""Seeded synthetic inputs for the stage-verifier tests and benchmark.

This module only *generates inputs*: stage descriptors, random weights, activations,
loss gradients, and the corrupted submissions ("attacks") that a dishonest stage
worker would send.  It holds none of the verifier's arithmetic (no block forward or
backward, no distance statistic, no flag rule) so that the CPU oracle and the HIP
library can both be fed from it without sharing any of the method's code.

Attack shapes follow the paper's "Attack Variants" paragraph (Problem Statement):
scaling x -> alpha*x, random sign flips, bias (additive Gaussian noise) and the
constant (zeros) attack.  Workload shapes are the five benchmark configurations of
this repository (tiny / small / medium / large / sweep).

Everything is numpy; values destined for a bf16 stage are rounded to
bf16-representable fp32 here so that both consumers see bit-identical inputs.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Dict, List, Optional, Tuple

import numpy as np


# --------------------------------------------------------------------------- descriptors
@dataclasses.dataclass(frozen=True)
class StageDesc:
    """Hyper-parameters of one pipeline stage (n_blocks identical pre-norm blocks)."""
    n_blocks: int
    d_model: int
    n_heads: int
    n_kv_heads: int
    ffn_hidden: int
    mlp: str = "swiglu"          # "swiglu" | "gelu"
    norm: str = "rms"            # "rms" | "ln"
    rope: bool = True
    causal: bool = True
    norm_eps: float = 1e-5
    rope_theta: float = 500000.0
    dtype: str = "bf16"          # "bf16" | "f32"
    # mixture-of-experts MLP (n_experts = 0: dense).  Every expert, routed or shared, is a SwiGLU
    # feed-forward of width ffn_hidden; each token uses its top_k routed experts and all shared ones.
    n_experts: int = 0
    top_k: int = 0
    n_shared: int = 0
    router_score: str = "sigmoid"   # "sigmoid" | "softmax"
    router_norm: bool = False       # divide the selected scores by their sum

    @property
    def head_dim(self) -> int:
        return self.d_model // self.n_heads


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    desc: StageDesc
    batch: int
    seq: int
    tau: float
    n_claims: int
    backward: bool = False


TINY = Workload("tiny", StageDesc(1, 128, 4, 4, 512, mlp="gelu", norm="ln", rope=False,
                                  causal=True, dtype="f32"), batch=2, seq=64, tau=1e-3, n_claims=8)
SMALL = Workload("small", StageDesc(2, 1024, 16, 16, 2816), batch=8, seq=512, tau=2e-2, n_claims=64)
MEDIUM = Workload("medium", StageDesc(4, 2048, 16, 16, 5632), batch=8, seq=1024, tau=2e-2,
                  n_claims=10, backward=True)
LARGE = Workload("large", StageDesc(4, 4096, 32, 8, 14336), batch=4, seq=2048, tau=2e-2, n_claims=32)
# The two mixture-of-experts shapes of the paper's Table model_config (hidden size, heads, KV heads, experts, shared
# experts, top-k as printed; expert width from its "multiplier 1.3, multiple of 1024" rule; the table gives the second
# model no KV-head count, so it gets one KV head per query head).  One block per stage and sequence length 1024 as in
# the paper's setup; the micro-batch is ours.
MOE_TOP1 = Workload("moe_top1", StageDesc(1, 512, 32, 8, 2048, n_experts=8, top_k=1, n_shared=1), batch=8, seq=1024,
                    tau=2e-2, n_claims=8, backward=True)
MOE_TOP6 = Workload("moe_top6", StageDesc(1, 1024, 16, 16, 4096, n_experts=8, top_k=6, n_shared=2, router_norm=True),
                    batch=8, seq=1024, tau=2e-2, n_claims=8, backward=True)


def sweep_point(seq: int, batch: int) -> Workload:
    return Workload(f"sweep_s{seq}_b{batch}", StageDesc(1, 4096, 32, 8, 14336), batch=batch, seq=seq,
                    tau=2e-2, n_claims=128, backward=True)


WORKLOADS: Dict[str, Workload] = {w.name: w for w in (TINY, SMALL, MEDIUM, LARGE, MOE_TOP1, MOE_TOP6)}


# --------------------------------------------------------------------------- bf16 helpers
def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bf16 (ties to even); result stays fp32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    u = (u + 0x7FFF + lsb) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(x.shape)


def to_stage_dtype(x: np.ndarray, dtype: str) -> np.ndarray:
    x = np.asarray(x, dtype=np.float32)
    return round_to_bf16(x) if dtype == "bf16" else x


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of already bf16-representable fp32 values."""
    return (np.ascontiguousarray(x, dtype=np.float32).view(np.uint32) >> 16).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


# --------------------------------------------------------------------------- generators
def _rng(seed: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[int(seed), int(stream)]))


def make_weights(desc: StageDesc, seed: int = 0) -> List[Dict[str, Optional[np.ndarray]]]:
    """Per-block weights.  Matrices ~ N(0, 0.02^2) stored [out, in]; norm gains
    1 + 0.1 N(0,1) and LayerNorm biases 0.02 N(0,1) so that they are exercised."""
    D, hd = desc.d_model, desc.head_dim
    Hq, Hkv, F = desc.n_heads * hd, desc.n_kv_heads * hd, desc.ffn_hidden
    blocks = []
    for b in range(desc.n_blocks):
        g = _rng(seed, 1000 + b)

        def mat(o, i):
            return to_stage_dtype(0.02 * g.standard_normal((o, i), dtype=np.float32), desc.dtype)

        def vec(n, mean, std):
            return to_stage_dtype(mean + std * g.standard_normal(n, dtype=np.float32), desc.dtype)

        w = dict(wq=mat(Hq, D), wk=mat(Hkv, D), wv=mat(Hkv, D), wo=mat(D, Hq))
        if desc.n_experts > 0:
            E, Fs = desc.n_experts, desc.n_shared * F
            w.update(w_gate=mat(E * F, D).reshape(E, F, D), w_up=mat(E * F, D).reshape(E, F, D),
                     w_down=mat(E * D, F).reshape(E, D, F), w_router=mat(E, D))
            if Fs:
                w.update(ws_gate=mat(Fs, D), ws_up=mat(Fs, D), ws_down=mat(D, Fs))
        elif desc.mlp == "swiglu":
            w.update(w_gate=mat(F, D), w_up=mat(F, D), w_down=mat(D, F))
        else:
            w.update(w_gate=None, w_up=mat(F, D), w_down=mat(D, F))
        w.update(norm1_g=vec(D, 1.0, 0.1), norm2_g=vec(D, 1.0, 0.1))
        if desc.norm == "ln":
            w.update(norm1_b=vec(D, 0.0, 0.02), norm2_b=vec(D, 0.0, 0.02))
        else:
            w.update(norm1_b=None, norm2_b=None)
        blocks.append(w)
    return blocks


def make_activations(desc: StageDesc, batch: int, seq: int, seed: int, micro_batch: int = 0) -> np.ndarray:
    """Stage input h_s ~ N(0,1), shape [batch, seq, d_model]."""
    g = _rng(seed, 2000 + micro_batch)
    return to_stage_dtype(g.standard_normal((batch, seq, desc.d_model), dtype=np.float32), desc.dtype)


def make_output_grad(desc: StageDesc, batch: int, seq: int, seed: int, micro_batch: int = 0,
                     std: float = 1e-3) -> np.ndarray:
    """Loss gradient at the stage output, g_{s+1} ~ N(0, std^2)."""
    g = _rng(seed, 3000 + micro_batch)
    return to_stage_dtype(std * g.standard_normal((batch, seq, desc.d_model), dtype=np.float32), desc.dtype)


def make_moe_case_with_routing_features(desc: StageDesc, batch: int, seq: int, seed: int, level: float = 0.5,
                                        mlp_gain: float = 1.0):
    """A mixture-of-experts stage and its input whose routing is decided far from any tie, BY CONSTRUCTION of the inputs
    (no arithmetic of the layer happens here): the first E features of the residual stream are "routing features".

    * input: token t carries in features 0 .. E-1 the values level * (1 .. E) in a seeded order of its own; the other
      features are the usual N(0, 1) draws.  Multiples of 0.5 up to 8 are exact in bf16.
    * every block: the rows of Wo, of every expert's down projection and of the shared experts' down projection that
      write features 0 .. E-1 are zero, so those features pass through every block unchanged (the residual adds an
      exact zero); the second norm's gain is 1 on them; router row e is the unit vector of feature p_l(e), with p_l a
      seeded permutation per block (so the blocks of a stage route the same token differently).

    With these inputs the router logit of expert e for token t is (its routing feature) / rms(x1_t): the token's E
    logits are level * (1 .. E) / rms_t in some order, neighbouring logits are level / rms_t apart, every expert is
    used equally often, and the gate values differ from token to token.  Returns (weights, h)."""
    E = desc.n_experts
    assert E > 0 and E * level <= 8.0 and desc.d_model > E
    w = make_weights(desc, seed)
    g = _rng(seed, 8000)
    for l, b in enumerate(w):
        for k in ("w_gate", "w_up", "w_down", "ws_gate", "ws_up", "ws_down"):
            if b.get(k) is not None and mlp_gain != 1.0:
                b[k] = to_stage_dtype(b[k] * np.float32(mlp_gain), desc.dtype)
        b["wo"][:E, :] = 0.0
        b["w_down"][:, :E, :] = 0.0
        if b.get("ws_down") is not None:
            b["ws_down"][:E, :] = 0.0
        b["norm2_g"][:E] = 1.0
        r = np.zeros((E, desc.d_model), dtype=np.float32)
        r[np.arange(E), g.permutation(E)] = 1.0
        b["w_router"] = r
    h = make_activations(desc, batch, seq, seed)
    ranks = np.argsort(g.random((batch, seq, E)), axis=-1)              # a permutation of 0 .. E-1 per token
    h[..., :E] = np.float32(level) * (ranks + 1).astype(np.float32)
    return w, to_stage_dtype(h, desc.dtype)


# --------------------------------------------------------------------------- submissions
def make_directions(d_model: int, n_dirs: int, seed: int = 0) -> np.ndarray:
    """Projection directions for the sliced Wasserstein statistic: n_dirs draws from N(0, I_D),
    scaled to unit length, then rounded to bf16 (the library takes them in bf16; both consumers see
    the same rounded values, whose length differs from 1 by at most 2^-9 relative)."""
    u = _rng(seed, 50).standard_normal((n_dirs, d_model))
    u /= np.linalg.norm(u, axis=1, keepdims=True)
    return round_to_bf16(u.astype(np.float32))


def stream_signal(kind: str, stage: int, worker: int, t: int, T: int, D: int, dtype: str, seed: int = 0,
                  drift: float = 1e-3) -> np.ndarray:
    """Synthetic stand-in for what worker `worker` of pipeline stage `stage` sends at iteration t: a
    per-stage mean signal that drifts slowly with t plus an independent mini-batch component of
    half its scale.  kind "h": activations of unit scale; "g": activation gradients of scale 1e-3."""
    scale = 1.0 if kind == "h" else 1e-3
    base = _rng(seed, 1000 + 2 * stage + (kind == "g")).standard_normal((T, D))
    own = _rng(seed, 100_000 + ((t * 64 + stage) * 1024 + worker) * 2 + (kind == "g")).standard_normal((T, D))
    x = scale * ((1.0 + drift * t) * base + 0.5 * own)
    return to_stage_dtype(x.astype(np.float32), dtype)


def honest_claim(reference: np.ndarray, dtype: str) -> np.ndarray:
    """What an honest worker sends: the true signal in the stage's storage dtype."""
    return to_stage_dtype(np.asarray(reference, dtype=np.float32), dtype)


def attack_scale(x: np.ndarray, alpha: float, dtype: str) -> np.ndarray:
    return to_stage_dtype(np.float32(alpha) * np.asarray(x, np.float32), dtype)


def attack_noise(x: np.ndarray, rel_std: float, seed: int, dtype: str) -> np.ndarray:
    """Bias-addition attack with sigma = rel_std * RMS(x)."""
    x = np.asarray(x, np.float32)
    rms = float(np.sqrt(np.mean(np.square(x, dtype=np.float64))))
    eps = _rng(seed, 4000).standard_normal(x.shape, dtype=np.float32)
    return to_stage_dtype(x + np.float32(rel_std * rms) * eps, dtype)


def attack_sign_channels(x: np.ndarray, frac: float, seed: int, dtype: str) -> Tuple[np.ndarray, np.ndarray]:
    """Flip the sign of ceil(frac*D) feature channels (chosen without replacement) on every token."""
    x = np.array(x, dtype=np.float32, copy=True)
    D = x.shape[-1]
    n = int(math.ceil(frac * D))
    ch = np.sort(_rng(seed, 5000).permutation(D)[:n])
    x[..., ch] = -x[..., ch]
    return to_stage_dtype(x, dtype), ch


def attack_zero(x: np.ndarray, dtype: str) -> np.ndarray:
    return np.zeros_like(np.asarray(x, np.float32))


def attack_tokens(x: np.ndarray, frac: float, kind: str, seed: int, dtype: str) -> Tuple[np.ndarray, np.ndarray]:
    """Corrupt only ceil(frac*T) random tokens of x [.., D] (flattened token index returned).
    kind: "noise" (0.1 * token RMS), "scale" (x1.5), "neg" (x-1), "zero"."""
    x = np.array(x, dtype=np.float32, copy=True)
    flat = x.reshape(-1, x.shape[-1])
    T = flat.shape[0]
    n = int(math.ceil(frac * T))
    g = _rng(seed, 6000)
    tok = np.sort(g.permutation(T)[:n])
    if kind == "noise":
        rms = np.sqrt(np.mean(np.square(flat[tok], dtype=np.float64), axis=1, keepdims=True)).astype(np.float32)
        flat[tok] += 0.1 * rms * g.standard_normal((n, flat.shape[1]), dtype=np.float32)
    elif kind == "scale":
        flat[tok] *= np.float32(1.5)
    elif kind == "neg":
        flat[tok] *= np.float32(-1.0)
    elif kind == "zero":
        flat[tok] = 0.0
    else:
        raise ValueError(kind)
    return to_stage_dtype(x, dtype), tok


# --- the remaining attack variants of the paper's "Attack Variants" paragraph and its adaptive attack --------------
def attack_constant(x: np.ndarray, value: float, dtype: str) -> np.ndarray:
    """Constant attack: every element is `value` (the paper names zeros and negative ones)."""
    return to_stage_dtype(np.full_like(x, value, dtype=np.float32), dtype)


def attack_random_value(x: np.ndarray, seed: int, dtype: str) -> np.ndarray:
    """Random value attack: every element drawn from N(0, 1)."""
    return to_stage_dtype(_rng(seed, 23).standard_normal(x.shape).astype(np.float32), dtype)


def attack_sign_elements(x: np.ndarray, p: float, seed: int, dtype: str) -> np.ndarray:
    """Random sign attack: each element's sign is flipped with probability p."""
    flip = _rng(seed, 24).random(x.shape) < p
    return to_stage_dtype(np.where(flip, -x, x).astype(np.float32), dtype)


def invisible_noise_zmax(p: float) -> float:
    """z_max = sqrt(2) erfinv(2 p - 1): the p-quantile of the standard normal."""
    from scipy.special import erfinv
    return float(math.sqrt(2.0) * erfinv(2.0 * p - 1.0))


def attack_invisible_noise(x: np.ndarray, p: float, seed: int, dtype: str) -> np.ndarray:
    """Invisible noise attack: mu + z_max (sigma * eps) with mu, sigma the per-feature mean and standard deviation of
    the signal over its tokens (the element-wise statistics a single signal [.., D] offers) and eps ~ N(0, I)."""
    x2 = x.reshape(-1, x.shape[-1]).astype(np.float64)
    mu, sd = x2.mean(axis=0), x2.std(axis=0)
    eps = _rng(seed, 25).standard_normal(x2.shape)
    return to_stage_dtype((mu + invisible_noise_zmax(p) * sd * eps).reshape(x.shape).astype(np.float32), dtype)


def attack_drift(m_stale: np.ndarray, target: np.ndarray, alpha: float, sigma: float, seed: int, dtype: str) -> np.ndarray:
    """Adaptive attack: m + alpha (target - m) / ||m|| + eps, with m the attacker's stale EMA of the signals it sent
    and eps ~ N(0, sigma^2)."""
    m = m_stale.astype(np.float64)
    out = m + alpha * (target.astype(np.float64) - m) / max(float(np.linalg.norm(m)), 1e-30)
    out = out + sigma * _rng(seed, 26).standard_normal(m.shape)
    return to_stage_dtype(out.astype(np.float32), dtype)


def drift_delay(beta: float) -> int:
    """delta = ceil(log 0.1 / log beta): how stale the attacker's EMA is."""
    return int(math.ceil(math.log(0.1) / math.log(beta)))


def small_claim_plan(n_claims: int = 64, seed: int = 0) -> List[str]:
    """Small config: 10 % scaled by 1.5, 10 % sign-flipped on 5 % of channels, rest honest."""
    n_bad = int(round(0.1 * n_claims))
    kinds = ["honest"] * n_claims
    order = _rng(seed, 7000).permutation(n_claims)
    for i in order[:n_bad]:
        kinds[int(i)] = "scale"
    for i in order[n_bad:2 * n_bad]:
        kinds[int(i)] = "sign"
    return kinds


def make_claim(kind: str, reference: np.ndarray, dtype: str, seed: int) -> np.ndarray:
    """One submission of the given kind manufactured from the true signal `reference`."""
    if kind == "honest":
        return honest_claim(reference, dtype)
    if kind == "scale":
        return attack_scale(reference, 1.5, dtype)
    if kind == "noise":
        return attack_noise(reference, 0.1, seed, dtype)
    if kind == "sign":
        return attack_sign_channels(reference, 0.05, seed, dtype)[0]
    if kind == "zero":
        return attack_zero(reference, dtype)
    if kind.startswith("tok_"):
        return attack_tokens(reference, 0.01, kind[4:], seed, dtype)[0]
    if kind == "const_neg1":
        return attack_constant(reference, -1.0, dtype)
    if kind == "random":
        return attack_random_value(reference, seed, dtype)
    if kind == "sign_p":
        return attack_sign_elements(reference, 0.1, seed, dtype)
    if kind == "invisible":
        return attack_invisible_noise(reference, 0.99, seed, dtype)
    raise ValueError(kind)
