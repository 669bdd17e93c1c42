"""Pins of the oracle's mixture-of-experts layer (the second workload family of the paper's "Alternative
Architectures" paragraph; expert / shared-expert / top-k counts from Table model_config).  The paper prints no worked
example of the layer, so the pins are: reduction to the dense SwiGLU block the other pins already cover, a per-token
brute force written from the definition, a hand-worked two-expert example, the tie rule, and central finite
differences for the backward."""
import dataclasses
import math

import numpy as np
import pytest

import stage_inputs as si
from oracle import stage_oracle as so

MOE = si.StageDesc(1, 32, 4, 2, 24, n_experts=4, top_k=2, n_shared=1, router_norm=True)


def _weights(desc, seed=3, router_gain=25.0):
    w = si.make_weights(desc, seed)
    for b in w:                                 # spread the router logits so that margins are not all tiny
        b["w_router"] = b["w_router"] * router_gain
        for k in ("w_gate", "w_up", "w_down", "ws_gate", "ws_up", "ws_down"):
            if b.get(k) is not None:
                b[k] = b[k] * 8.0               # make the MLP a visible part of the block output
    return w


def _tokens(S, D, seed=0):
    return np.random.default_rng(seed).standard_normal((S, D))


@pytest.mark.parametrize("score,norm", [("sigmoid", False), ("sigmoid", True), ("softmax", False), ("softmax", True)])
def test_moe_matches_per_token_brute_force(score, norm):
    desc = dataclasses.replace(MOE, router_score=score, router_norm=norm, dtype="f32")
    w = _weights(desc)[0]
    n = _tokens(11, desc.d_model)
    got = so.moe_forward(n, w, desc)
    F = desc.ffn_hidden
    for t in range(n.shape[0]):
        logit = [float(np.dot(w["w_router"][e].astype(np.float64), n[t])) for e in range(desc.n_experts)]
        if score == "sigmoid":
            s = [1.0 / (1.0 + math.exp(-v)) for v in logit]
        else:
            z = sum(math.exp(v) for v in logit)
            s = [math.exp(v) / z for v in logit]
        chosen = sorted(range(desc.n_experts), key=lambda e: (-s[e], e))[:desc.top_k]
        tot = sum(s[e] for e in chosen) if norm else 1.0
        acc = np.zeros(desc.d_model)
        experts = [(s[e] / tot, w["w_gate"][e], w["w_up"][e], w["w_down"][e]) for e in chosen]
        experts += [(1.0, w["ws_gate"][i * F:(i + 1) * F], w["ws_up"][i * F:(i + 1) * F], w["ws_down"][:, i * F:(i + 1) * F])
                    for i in range(desc.n_shared)]
        for gate, wg, wu, wd in experts:
            hidden = np.zeros(F)
            for f in range(F):
                a = float(np.dot(wg[f].astype(np.float64), n[t]))
                hidden[f] = a / (1.0 + math.exp(-a)) * float(np.dot(wu[f].astype(np.float64), n[t]))
            acc += gate * (wd.astype(np.float64) @ hidden)
        np.testing.assert_allclose(got[t], acc, rtol=1e-11, atol=1e-13)


def test_moe_hand_worked_two_expert_example():
    # D = 2, F = 1, two experts, top-1, sigmoid gate.  Token (1, 2): logits (1, 2)·(1, 0) = 1 and (1, 2)·(0, 1) = 2
    # -> expert 1, gate sigmoid(2).  Expert 1: gate proj (1, 1) -> 3, up proj (2, 0) -> 2, silu(3) * 2, down (1, -1).
    desc = si.StageDesc(1, 2, 1, 1, 1, n_experts=2, top_k=1, dtype="f32")
    w = dict(w_router=np.array([[1.0, 0.0], [0.0, 1.0]]),
             w_gate=np.array([[[5.0, 5.0]], [[1.0, 1.0]]]), w_up=np.array([[[7.0, 7.0]], [[2.0, 0.0]]]),
             w_down=np.array([[[9.0], [9.0]], [[1.0], [-1.0]]]))
    out = so.moe_forward(np.array([[1.0, 2.0]]), w, desc)
    sig = lambda v: 1.0 / (1.0 + math.exp(-v))
    a = sig(2.0) * (3.0 * sig(3.0)) * 2.0
    np.testing.assert_allclose(out, [[a, -a]], rtol=1e-14)
    # token (2, 1) goes to expert 0 instead: gate sigmoid(2), gate proj 15, up proj 21
    out = so.moe_forward(np.array([[2.0, 1.0]]), w, desc)
    b = sig(2.0) * (15.0 * sig(15.0)) * 21.0 * 9.0
    np.testing.assert_allclose(out, [[b, b]], rtol=1e-14)


def test_moe_reduces_to_the_dense_swiglu_block():
    # (a) identical experts with normalised gates, (b) one expert with a softmax router (its only score is 1),
    # (c) no routed contribution (zero down projections) and two shared experts = one dense MLP of twice the width
    dense = si.StageDesc(1, 32, 4, 2, 24, dtype="f32")
    wd = si.make_weights(dense, 5)[0]
    x = _tokens(9, 32, seed=1)
    want = so.block_forward(x, wd, dense)
    for E, k, score in ((4, 2, "sigmoid"), (1, 1, "softmax"), (4, 3, "softmax")):
        desc = dataclasses.replace(dense, n_experts=E, top_k=k, router_score=score, router_norm=True)
        w = dict(wd)
        w["w_router"] = np.random.default_rng(E).standard_normal((E, 32))
        w["w_gate"] = np.repeat(wd["w_gate"][None], E, 0)
        w["w_up"] = np.repeat(wd["w_up"][None], E, 0)
        w["w_down"] = np.repeat(wd["w_down"][None], E, 0)
        np.testing.assert_allclose(so.block_forward(x, w, desc), want, rtol=1e-12, atol=1e-14)
    wide = dataclasses.replace(dense, ffn_hidden=48)
    ww = si.make_weights(wide, 6)[0]
    desc = dataclasses.replace(dense, n_experts=2, top_k=1, n_shared=2)
    w = dict(ww)
    w.update(w_router=np.ones((2, 32)), w_gate=np.ones((2, 24, 32)), w_up=np.ones((2, 24, 32)), w_down=np.zeros((2, 32, 24)),
             ws_gate=ww["w_gate"], ws_up=ww["w_up"], ws_down=ww["w_down"])
    np.testing.assert_allclose(so.block_forward(x, w, desc), so.block_forward(x, ww, wide), rtol=1e-12, atol=1e-14)


def test_route_tie_rule_margin_and_gate_normalisation():
    desc = si.StageDesc(1, 4, 1, 1, 8, n_experts=4, top_k=2, router_norm=True, dtype="f32")
    wr = np.array([[1.0, 0, 0, 0], [1.0, 0, 0, 0], [0, 1.0, 0, 0], [0, 0, 1.0, 0]])
    n = np.array([[2.0, 1.0, 0.5, 0.0],      # experts 0 and 1 tie at the top: the lower indices win, in index order
                  [0.0, 3.0, 3.0, 0.0],      # experts 2 and 3 tie at the top
                  [1.0, 1.0, 1.0, 0.0]])     # all four tie
    sel, gates, scores, margin, logits = so.moe_route(n, wr, desc)
    assert sel.tolist() == [[0, 1], [2, 3], [0, 1]]
    np.testing.assert_allclose(gates.sum(-1), 1.0, rtol=1e-15)
    sig = lambda v: 1.0 / (1.0 + math.exp(-v))
    np.testing.assert_allclose(margin, [2.0 - 1.0, 3.0 - 0.0, 0.0], rtol=1e-13, atol=1e-16)       # in logits
    np.testing.assert_allclose(logits, [[2.0, 2.0, 1.0, 0.5], [0.0, 0.0, 3.0, 3.0], [1.0, 1.0, 1.0, 1.0]], rtol=1e-15)
    np.testing.assert_allclose(gates[0], [0.5, 0.5], rtol=1e-15)
    # without normalisation the gates are the scores themselves; top_k = E has no margin
    desc2 = dataclasses.replace(desc, router_norm=False, top_k=4)
    sel, gates, scores, margin, _ = so.moe_route(n, wr, desc2)
    np.testing.assert_allclose(gates[0], sorted([sig(2.0), sig(2.0), sig(1.0), sig(0.5)], reverse=True), rtol=1e-15)
    assert np.all(np.isinf(margin))
    # softmax scores sum to one over ALL experts
    desc3 = dataclasses.replace(desc, router_score="softmax", router_norm=False)
    _, _, scores, _, _ = so.moe_route(n, wr, desc3)
    np.testing.assert_allclose(scores.sum(-1), 1.0, rtol=1e-15)


@pytest.mark.parametrize("score,norm,k", [("sigmoid", False, 1), ("sigmoid", True, 3), ("softmax", False, 2), ("softmax", True, 2)])
def test_moe_block_backward_matches_central_differences(score, norm, k):
    desc = dataclasses.replace(MOE, router_score=score, router_norm=norm, top_k=k, dtype="f32")
    w = _weights(desc, seed=7)
    x = _tokens(6, desc.d_model, seed=2)[None]
    g_out = np.random.default_rng(4).standard_normal(x.shape)
    _, g = so.stage_backward(x, g_out, w, desc)
    margin = so.stage_routing_margin(x, w, desc)
    assert margin.min() > 1e-4                # the probe below must not cross a routing boundary
    eps = 1e-6
    rng = np.random.default_rng(9)
    for _ in range(12):
        d = rng.standard_normal(x.shape)
        fd = (np.sum(so.stage_forward(x + eps * d, w, desc) * g_out) - np.sum(so.stage_forward(x - eps * d, w, desc) * g_out)) / (2 * eps)
        assert abs(fd - np.sum(g * d)) <= 2e-7 * max(1.0, abs(fd))


def test_backward_gate_gradient_is_not_dropped():
    # with one expert selected per token and no normalisation the only path from the router weights' INPUT side to
    # the output is the gate value: zeroing the router logits' slope must change the input gradient
    desc = dataclasses.replace(MOE, top_k=1, router_norm=False, n_shared=0, dtype="f32")
    w = _weights(desc, seed=8)
    x = _tokens(5, desc.d_model, seed=3)[None]
    g_out = np.ones_like(x)
    _, g = so.stage_backward(x, g_out, w, desc)
    st = so.block_forward(x[0], w[0], desc, keep=True)[1]
    n2 = st["moe"]["n"]
    # the routed term alone, recomputed token by token from the definition d/dn [ s_e(n) y_e(n) ]
    e_sel = st["moe"]["sel"][:, 0]
    sc = st["moe"]["scores"][np.arange(5), e_sel]
    dn = so.moe_backward(g_out[0], st["moe"], w[0], desc)
    for t in range(5):
        e = e_sel[t]
        y = so.moe_forward(n2[t:t + 1], w[0], desc)[0] / sc[t]                 # expert output without its gate
        router_part = float(np.sum(g_out[0, t] * y)) * sc[t] * (1 - sc[t]) * w[0]["w_router"][e].astype(np.float64)
        eps = 1e-6
        num = np.zeros(desc.d_model)
        for i in range(desc.d_model):
            dvec = np.zeros(desc.d_model); dvec[i] = eps
            gt = lambda v: (so.silu(v @ w[0]["w_gate"][e].astype(np.float64).T) * (v @ w[0]["w_up"][e].astype(np.float64).T)) @ w[0]["w_down"][e].astype(np.float64).T
            num[i] = np.sum(g_out[0, t] * (gt(n2[t] + dvec) - gt(n2[t] - dvec))) / (2 * eps) * sc[t]
        np.testing.assert_allclose(dn[t], num + router_part, rtol=2e-6, atol=1e-9)
    assert np.linalg.norm(g) > 0


def test_routing_feature_inputs_decide_every_token_far_from_a_tie():
    """The constructed case the GPU parity tests use to compare ALL tokens (stage_inputs.make_moe_case_with_routing_features):
    in every block of the stage the oracle's logits of a token are level * (1 .. E) / rms(x1_t) in some order, so the
    routing margin is level / rms_t -- one E-th of the largest logit -- and every expert is chosen equally often."""
    desc = si.StageDesc(2, 64, 4, 2, 48, n_experts=8, top_k=3, n_shared=1, router_norm=True, dtype="bf16")
    w, h = si.make_moe_case_with_routing_features(desc, 3, 50, seed=4)
    counts = np.zeros((desc.n_blocks, desc.n_experts), dtype=int)
    for b in range(h.shape[0]):
        x = h[b].astype(np.float64)
        for l, blk in enumerate(w):
            y, st = so.block_forward(x, blk, desc, keep=True)
            m = st["moe"]
            rms = np.sqrt(np.mean(st["x1"] ** 2, axis=1) + desc.norm_eps)
            np.testing.assert_allclose(np.sort(m["logits"], axis=1), 0.5 * np.arange(1, 9)[None, :] / rms[:, None], rtol=1e-12)
            np.testing.assert_allclose(m["margin"], 0.5 / rms, rtol=1e-9)
            assert np.all(m["margin"] >= 0.124 * np.max(np.abs(m["logits"]), axis=1))       # 1/E of the largest logit
            assert np.array_equal(y[:, :8], x[:, :8])                                       # the features pass through unchanged
            counts[l] += np.bincount(m["sel"].ravel(), minlength=8)
            x = y
    assert counts.min() > 0.7 * counts.mean()                                               # every expert used about equally
    # the two blocks route the same token through different experts (their own permutations of the features)
    assert not np.array_equal(w[0]["w_router"], w[1]["w_router"])
