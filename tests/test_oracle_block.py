"""Pins for the oracle's stage map and its input gradient (CPU only).

Nothing here compares the oracle with itself: every check is against a scalar-loop
brute force, an independent library routine (torch CPU float64 primitives and
autograd), central finite differences, or a structural fact of the operation.
"""
import cmath
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import stage_oracle as so
from stage_inputs import StageDesc, make_activations, make_output_grad, make_weights

LLAMA = StageDesc(2, 32, 4, 2, 48, mlp="swiglu", norm="rms", rope=True, causal=True, dtype="f32")
GPT = StageDesc(1, 24, 3, 3, 40, mlp="gelu", norm="ln", rope=False, causal=True, dtype="f32")
BIDIR = StageDesc(1, 16, 2, 1, 24, mlp="swiglu", norm="rms", rope=True, causal=False, dtype="f32")


def rng(seed):
    return np.random.default_rng(seed)


# ------------------------------------------------------------------ norms
def test_rmsnorm_properties_and_library():
    g = rng(1)
    x = g.standard_normal((6, 64)) * 3.0
    n = so.norm_forward(x, np.ones(64), None, "rms", 0.0)
    np.testing.assert_allclose(np.mean(n * n, axis=-1), 1.0, rtol=1e-12)
    np.testing.assert_allclose(so.norm_forward(7.5 * x, np.ones(64), None, "rms", 0.0), n, rtol=1e-12)
    gain = g.standard_normal(64)
    lib = F.rms_norm(torch.from_numpy(x), (64,), torch.from_numpy(gain), eps=1e-5).numpy()
    np.testing.assert_allclose(so.norm_forward(x, gain, None, "rms", 1e-5), lib, rtol=1e-12)


def test_layernorm_properties_and_library():
    g = rng(2)
    x = g.standard_normal((6, 48)) * 2.0 + 1.0
    n = so.norm_forward(x, np.ones(48), np.zeros(48), "ln", 0.0)
    np.testing.assert_allclose(n.mean(-1), 0.0, atol=1e-13)
    np.testing.assert_allclose(n.var(-1), 1.0, rtol=1e-12)
    gain, bias = g.standard_normal(48), g.standard_normal(48)
    lib = F.layer_norm(torch.from_numpy(x), (48,), torch.from_numpy(gain), torch.from_numpy(bias), eps=1e-5).numpy()
    np.testing.assert_allclose(so.norm_forward(x, gain, bias, "ln", 1e-5), lib, rtol=1e-11, atol=1e-13)


@pytest.mark.parametrize("kind", ["rms", "ln"])
def test_norm_backward_finite_differences(kind):
    g = rng(3)
    x, dn, gain = g.standard_normal((3, 20)), g.standard_normal((3, 20)), 1 + 0.3 * g.standard_normal(20)
    bias = g.standard_normal(20) if kind == "ln" else None
    dx = so.norm_backward(dn, x, gain, kind, 1e-5)
    for _ in range(4):
        v = g.standard_normal(x.shape)
        e = 1e-6
        fd = (np.sum(dn * so.norm_forward(x + e * v, gain, bias, kind, 1e-5))
              - np.sum(dn * so.norm_forward(x - e * v, gain, bias, kind, 1e-5))) / (2 * e)
        assert abs(fd - np.sum(dx * v)) <= 1e-7 * max(1.0, abs(fd))


# ------------------------------------------------------------------ RoPE
def test_rope_is_complex_rotation():
    g = rng(4)
    S, nh, hd, theta = 9, 2, 8, 500000.0
    x = g.standard_normal((S, nh, hd))
    got = so.rope_rotate(x, theta)
    for p in range(S):
        for h in range(nh):
            for i in range(hd // 2):
                z = complex(x[p, h, 2 * i], x[p, h, 2 * i + 1]) * cmath.exp(1j * p * theta ** (-2.0 * i / hd))
                assert abs(got[p, h, 2 * i] - z.real) < 1e-12 and abs(got[p, h, 2 * i + 1] - z.imag) < 1e-12


def test_rope_identity_norm_relative_and_inverse():
    g = rng(5)
    S, hd, theta = 12, 16, 10000.0
    q, k = g.standard_normal((S, 1, hd)), g.standard_normal((S, 1, hd))
    rq = so.rope_rotate(q, theta)
    np.testing.assert_array_equal(rq[0], q[0])                                   # position 0 untouched
    np.testing.assert_allclose(np.linalg.norm(rq, axis=-1), np.linalg.norm(q, axis=-1), rtol=1e-13)
    np.testing.assert_allclose(so.rope_rotate(rq, theta, inverse=True), q, atol=1e-13)
    # <R_m a, R_n b> depends only on m - n: same vectors placed at (7,3) and (10,6)
    a, b = g.standard_normal(hd), g.standard_normal(hd)
    qa = np.tile(a, (S, 1, 1)).reshape(S, 1, hd)
    kb = np.tile(b, (S, 1, 1)).reshape(S, 1, hd)
    ra, rb = so.rope_rotate(qa, theta), so.rope_rotate(kb, theta)
    assert abs(ra[7, 0] @ rb[3, 0] - ra[10, 0] @ rb[6, 0]) < 1e-12
    assert abs(ra[7, 0] @ rb[3, 0] - ra[8, 0] @ rb[3, 0]) > 1e-6                 # and does depend on it


# ------------------------------------------------------------------ attention
def _attention_loops(q, k, v, causal):
    S, H, hd = q.shape
    G = H // k.shape[1]
    o = np.zeros((S, H, hd))
    for h in range(H):
        for i in range(S):
            last = i if causal else S - 1
            sc = [sum(q[i, h, d] * k[j, h // G, d] for d in range(hd)) / math.sqrt(hd) for j in range(last + 1)]
            mx = max(sc)
            e = [math.exp(s - mx) for s in sc]
            z = sum(e)
            for j in range(last + 1):
                for d in range(hd):
                    o[i, h, d] += e[j] / z * v[j, h // G, d]
    return o


@pytest.mark.parametrize("causal", [True, False])
def test_attention_bruteforce_and_library(causal):
    g = rng(6)
    S, H, Hkv, hd = 7, 4, 2, 6
    q, k, v = g.standard_normal((S, H, hd)), g.standard_normal((S, Hkv, hd)), g.standard_normal((S, Hkv, hd))
    got = so.attention_forward(q, k, v, causal)
    np.testing.assert_allclose(got, _attention_loops(q, k, v, causal), rtol=1e-12, atol=1e-14)
    tq = torch.from_numpy(q).permute(1, 0, 2)[None]
    tk = torch.from_numpy(np.repeat(k, H // Hkv, axis=1)).permute(1, 0, 2)[None]
    tv = torch.from_numpy(np.repeat(v, H // Hkv, axis=1)).permute(1, 0, 2)[None]
    lib = F.scaled_dot_product_attention(tq, tk, tv, is_causal=causal)[0].permute(1, 0, 2).numpy()
    np.testing.assert_allclose(got, lib, rtol=1e-10, atol=1e-12)


def test_attention_special_cases():
    g = rng(7)
    S, H, hd = 10, 2, 4
    q, k, v = g.standard_normal((S, H, hd)), g.standard_normal((S, H, hd)), g.standard_normal((S, H, hd))
    # a single token attends to itself
    np.testing.assert_allclose(so.attention_forward(q[:1], k[:1], v[:1], True), v[:1], rtol=1e-14)
    # q = 0: uniform weights -> causal running mean of v
    run = np.cumsum(v, axis=0) / np.arange(1, S + 1)[:, None, None]
    np.testing.assert_allclose(so.attention_forward(np.zeros_like(q), k, v, True), run, rtol=1e-13)
    # causality: changing tokens > i leaves outputs <= i bit-identical
    k2, v2, q2 = k.copy(), v.copy(), q.copy()
    k2[6:], v2[6:], q2[6:] = 9.0, -3.0, 2.0
    a, b = so.attention_forward(q, k, v, True), so.attention_forward(q2, k2, v2, True)
    np.testing.assert_array_equal(a[:6], b[:6])
    assert np.abs(a[6:] - b[6:]).max() > 1e-3


def test_gqa_equals_mha_with_replicated_kv():
    g = rng(8)
    S, H, Hkv, hd = 6, 6, 2, 4
    q, k, v = g.standard_normal((S, H, hd)), g.standard_normal((S, Hkv, hd)), g.standard_normal((S, Hkv, hd))
    mha = so.attention_forward(q, np.repeat(k, 3, axis=1), np.repeat(v, 3, axis=1), True)
    np.testing.assert_allclose(so.attention_forward(q, k, v, True), mha, rtol=1e-14)


# ------------------------------------------------------------------ MLP nonlinearities
def test_activations_against_library_and_fd():
    z = np.linspace(-6, 6, 41)
    np.testing.assert_allclose(so.silu(z), F.silu(torch.from_numpy(z)).numpy(), rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(so.gelu(z), F.gelu(torch.from_numpy(z)).numpy(), rtol=1e-12, atol=1e-15)
    e = 1e-6
    np.testing.assert_allclose(so.silu_grad(z), (so.silu(z + e) - so.silu(z - e)) / (2 * e), rtol=1e-8, atol=1e-9)
    np.testing.assert_allclose(so.gelu_grad(z), (so.gelu(z + e) - so.gelu(z - e)) / (2 * e), rtol=1e-8, atol=1e-9)


# ------------------------------------------------------------------ whole stage vs torch primitives + autograd
def _torch_stage(h, weights, d):
    """Independent construction from library primitives (float64 CPU), differentiable."""
    B, S, D = h.shape
    H, Hkv, hd = d.n_heads, d.n_kv_heads, d.d_model // d.n_heads
    x = h
    for w in weights:
        t = {k_: (None if v_ is None else torch.from_numpy(np.asarray(v_, np.float64))) for k_, v_ in w.items()}

        def norm(a, gname, bname):
            if d.norm == "rms":
                return F.rms_norm(a, (D,), t[gname], eps=d.norm_eps)
            return F.layer_norm(a, (D,), t[gname], t[bname], eps=d.norm_eps)

        n1 = norm(x, "norm1_g", "norm1_b")
        q = F.linear(n1, t["wq"]).view(B, S, H, hd)
        k = F.linear(n1, t["wk"]).view(B, S, Hkv, hd)
        v = F.linear(n1, t["wv"]).view(B, S, Hkv, hd)
        if d.rope:
            freqs = d.rope_theta ** (-torch.arange(0, hd, 2, dtype=torch.float64) / hd)
            cis = torch.polar(torch.ones(S, hd // 2, dtype=torch.float64),
                              torch.outer(torch.arange(S, dtype=torch.float64), freqs))[None, :, None, :]
            q = torch.view_as_real(torch.view_as_complex(q.reshape(B, S, H, hd // 2, 2)) * cis).reshape(B, S, H, hd)
            k = torch.view_as_real(torch.view_as_complex(k.reshape(B, S, Hkv, hd // 2, 2)) * cis).reshape(B, S, Hkv, hd)
        k = k.repeat_interleave(H // Hkv, dim=2)
        v = v.repeat_interleave(H // Hkv, dim=2)
        o = F.scaled_dot_product_attention(q.transpose(1, 2), k.transpose(1, 2), v.transpose(1, 2),
                                           is_causal=d.causal).transpose(1, 2).reshape(B, S, D)
        x1 = x + F.linear(o, t["wo"])
        n2 = norm(x1, "norm2_g", "norm2_b")
        if d.mlp == "swiglu":
            a = F.silu(F.linear(n2, t["w_gate"])) * F.linear(n2, t["w_up"])
        else:
            a = F.gelu(F.linear(n2, t["w_up"]))
        x = x1 + F.linear(a, t["w_down"])
    return x


@pytest.mark.parametrize("desc", [LLAMA, GPT, BIDIR], ids=["llama_gqa", "gpt_ln_gelu", "bidirectional"])
def test_stage_forward_and_input_gradient_match_library_autograd(desc):
    weights = make_weights(desc, seed=11)
    # larger weights than the benchmark init so that every branch matters in the comparison
    for w in weights:
        for k_ in ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down"):
            if w[k_] is not None:
                w[k_] = w[k_] * 12.0
    h = make_activations(desc, 2, 9, seed=11).astype(np.float64)
    gn = make_output_grad(desc, 2, 9, seed=11, std=1.0).astype(np.float64)
    th = torch.from_numpy(h).requires_grad_(True)
    ty = _torch_stage(th, weights, desc)
    (ty * torch.from_numpy(gn)).sum().backward()
    y, g = so.stage_backward(h, gn, weights, desc)
    np.testing.assert_allclose(y, ty.detach().numpy(), rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(g, th.grad.numpy(), rtol=1e-8, atol=1e-10)
    np.testing.assert_allclose(so.stage_forward(h, weights, desc), y, rtol=0, atol=0)
    assert np.abs(y - h).max() > 0.1            # the stage is not close to the identity


@pytest.mark.parametrize("desc", [LLAMA, GPT], ids=["llama_gqa", "gpt_ln_gelu"])
def test_input_gradient_central_finite_differences(desc):
    weights = make_weights(desc, seed=5)
    for w in weights:
        for k_ in ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down"):
            if w[k_] is not None:
                w[k_] = w[k_] * 10.0
    h = make_activations(desc, 1, 6, seed=5).astype(np.float64)
    gn = make_output_grad(desc, 1, 6, seed=5, std=1.0).astype(np.float64)
    _, g = so.stage_backward(h, gn, weights, desc)
    r = rng(9)
    for _ in range(3):
        v = r.standard_normal(h.shape)
        e = 1e-5
        fd = (np.sum(gn * so.stage_forward(h + e * v, weights, desc))
              - np.sum(gn * so.stage_forward(h - e * v, weights, desc))) / (2 * e)
        assert abs(fd - np.sum(g * v)) <= 1e-6 * max(abs(fd), 1e-3)


def test_adjoint_identity():
    """<J v, u> = <v, J^T u>: J v by finite differences, J^T u from the oracle's backward."""
    desc = LLAMA
    weights = make_weights(desc, seed=2)
    for w in weights:
        for k_ in ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down"):
            w[k_] = w[k_] * 10.0
    h = make_activations(desc, 1, 5, seed=2).astype(np.float64)
    r = rng(10)
    u, v = r.standard_normal(h.shape), r.standard_normal(h.shape)
    e = 1e-6
    jv = (so.stage_forward(h + e * v, weights, desc) - so.stage_forward(h - e * v, weights, desc)) / (2 * e)
    _, jtu = so.stage_backward(h, u, weights, desc)
    assert abs(np.sum(jv * u) - np.sum(v * jtu)) <= 1e-6 * abs(np.sum(jv * u))


def test_zero_output_projections_make_the_stage_an_identity():
    desc = LLAMA
    weights = make_weights(desc, seed=3)
    for w in weights:
        w["wo"] = np.zeros_like(w["wo"])
        w["w_down"] = np.zeros_like(w["w_down"])
    h = make_activations(desc, 2, 8, seed=3)
    gn = make_output_grad(desc, 2, 8, seed=3)
    y, g = so.stage_backward(h, gn, weights, desc)
    np.testing.assert_array_equal(y, h.astype(np.float64))
    np.testing.assert_array_equal(g, gn.astype(np.float64))


def test_composition_and_sequence_independence():
    desc = LLAMA
    weights = make_weights(desc, seed=4)
    h = make_activations(desc, 3, 8, seed=4)
    one = dataclass_replace(desc, n_blocks=1)
    two_step = so.stage_forward(so.stage_forward(h, weights[:1], one), weights[1:], one)
    full = so.stage_forward(h, weights, desc)
    np.testing.assert_array_equal(full, two_step)
    for b in range(3):
        np.testing.assert_array_equal(full[b:b + 1], so.stage_forward(h[b:b + 1], weights, desc))


def dataclass_replace(d, **kw):
    import dataclasses
    return dataclasses.replace(d, **kw)
