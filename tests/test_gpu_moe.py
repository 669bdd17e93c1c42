"""GPU parity of the mixture-of-experts recompute (the second workload family: the paper's "Alternative
Architectures" paragraph, shapes from Table model_config) against the CPU oracle.

The routing is an integer decision taken from floating-point logits; the oracle takes it in float64.  Two kinds of case:

1. CONSTRUCTED routing (stage_inputs.make_moe_case_with_routing_features): the inputs are built so that in every block
   every token's k-th and (k+1)-th logits are 1/E of its largest logit apart, far more than any rounding of the device
   path can move them (band below).  There is then one correct result: the chosen experts are compared exactly, in
   order, and ALL tokens of h and g at the stated tolerance (relative L2 <= 1e-4 fp32, <= 2e-2 bf16).
2. RANDOM router rows: near-ties exist, and a token whose margin is within the device's logit error may legitimately be
   routed to the other candidate.  Every token the device routed differently from the oracle must be such a valid
   near-tie (each chosen expert's oracle logit within the band of the k-th); sequences without any such token are
   compared whole at the stated tolerance; for the others only validity is checked (their values follow another,
   equally correct routing, which no float64 reference of this side can reproduce without reading the device's choice).

Band: the device computes a logit as sum_i n_i w_ei with n the bf16-rounded second norm of its own x1.  Per element n
carries the rounding of x1 and of n (2^-9 each) and the error of the attention branch (per-token relative L2 of the
recomputation, bounded by the tolerance this file asserts); a logit therefore moves by at most eps * sum_i |n_i w_ei|
with eps = 2^-7 (bf16) or 2^-20 (fp32), a gap between two logits by twice that.  For the constructed case a logit is
one routing feature (exact on both sides) over rms(x1): its relative error is the rms's, at most the tolerance 2e-2,
plus 2^-9; gaps of 1/E >= 1/16 of the largest logit exceed twice that (5e-2) by construction."""
import dataclasses

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import stage_inputs as si
from oracle import stage_oracle as so
from gpu_util import dev, dev_weights, host, rel_l2

TOL = {"f32": 1e-4, "bf16": 2e-2}
EPS = {"f32": 2.0 ** -20, "bf16": 2.0 ** -7}       # per-element relative error of the router's input on the device
REL_BAND = {"f32": 1e-3, "bf16": 5e-2}             # constructed case: gap error as a fraction of the largest |logit|


def moe_weights(desc, seed, router_gain=5.0, mlp_gain=4.0):
    w = si.make_weights(desc, seed)
    for b in w:
        b["w_router"] = si.to_stage_dtype(b["w_router"] * np.float32(router_gain), desc.dtype)
        for k in ("w_gate", "w_up", "w_down", "ws_gate", "ws_up", "ws_down"):
            if b.get(k) is not None:
                b[k] = si.to_stage_dtype(b[k] * np.float32(mlp_gain), desc.dtype)
    return w


def oracle_run(h, g, w, desc):
    """Oracle outputs plus, per block, the routing record of every sequence."""
    B = h.shape[0]
    out_h, out_g = np.empty(h.shape), (np.empty(h.shape) if g is not None else None)
    routes = [[None] * B for _ in w]
    for b in range(B):
        x, kept = h[b].astype(np.float64), []
        for l, blk in enumerate(w):
            x, st = so.block_forward(x, blk, desc, keep=True)
            kept.append(st)
            routes[l][b] = st["moe"]
        out_h[b] = x
        if g is not None:
            d = g[b].astype(np.float64)
            for blk, st in zip(reversed(w), reversed(kept)):
                d = so.block_backward(d, st, blk, desc)
            out_g[b] = d
    return out_h, out_g, routes


def _cat(routes, l, key):
    return np.concatenate([r[key] for r in routes[l]])


def device_routing(ver, desc, B, S, backward):
    """{block: (experts [T, k], gates [T, k])} for the blocks whose routing the context kept."""
    out = {}
    for l in (range(desc.n_blocks) if backward else [desc.n_blocks - 1]):
        ex, gt = ver.last_routing(l, B * S)
        ex, gt = ex.cpu().numpy(), gt.cpu().numpy().astype(np.float64)
        assert ex.min() >= 0 and ex.max() < desc.n_experts
        assert all(len(set(row)) == desc.top_k for row in ex.tolist())              # no expert twice
        out[l] = (ex, gt)
    return out


def run_device(desc, w, h, g, backward, plain, fuse=False):
    import paper_2603_03592_amd as sv
    B, S = h.shape[:2]
    ver = sv.Verifier(desc, B * S, S, backward=backward, plain_kernels=plain, fuse_norm=fuse)
    wc = ver.pack_weights(wd := dev_weights(w, desc.dtype))
    if backward:
        out = ver.verify_backward(wc, dev(h, desc.dtype), dev(g, desc.dtype), want_g_hat=True, want_h_hat=True)
        got_h, got_g = host(out["h_hat"]), host(out["g_hat"])
    else:
        out = ver.verify_forward(wc, dev(h, desc.dtype), want_h_hat=True)
        got_h, got_g = host(out["h_hat"]), None
    routing = device_routing(ver, desc, B, S, backward)
    ver.close()
    return got_h, got_g, routing


def run_constructed(desc, B, S, seed, backward, plain=False, grad_std=1.0, mlp_gain=4.0, visible=True, fuse=False):
    """Case 1: every token, every expert choice, the stated tolerance, no exclusions."""
    w, h = si.make_moe_case_with_routing_features(desc, B, S, seed, mlp_gain=mlp_gain)
    g = si.make_output_grad(desc, B, S, seed, std=grad_std) if backward else None
    got_h, got_g, routing = run_device(desc, w, h, g, backward, plain, fuse)
    want_h, want_g, routes = oracle_run(h, g, w, desc)
    D, tol = desc.d_model, TOL[desc.dtype]
    for l in range(desc.n_blocks):
        margin, logits = _cat(routes, l, "margin"), _cat(routes, l, "logits")
        assert np.all(margin >= REL_BAND[desc.dtype] * np.max(np.abs(logits), axis=1)), l     # far from a tie, by construction
    for l, (ex, gt) in routing.items():
        assert np.array_equal(ex, _cat(routes, l, "sel")), l                                  # same experts, same order, all tokens
        np.testing.assert_allclose(gt, _cat(routes, l, "gates"), rtol=3e-2 if desc.dtype == "bf16" else 1e-4, atol=1e-6)
        assert np.bincount(ex.ravel(), minlength=desc.n_experts).min() > 0                    # every expert's segment is exercised
    tok_h = so.token_rel_l2(got_h.reshape(-1, D), want_h.reshape(-1, D))
    print(f"constructed routing: relative L2 h {rel_l2(got_h, want_h):.3e} (worst token {tok_h.max():.3e})"
          + (f" g {rel_l2(got_g, want_g):.3e}" if backward else ""))
    assert rel_l2(got_h, want_h) <= tol
    assert tok_h.max() <= (2 * tol if desc.dtype == "f32" else tol)
    assert not visible or rel_l2(want_h[..., desc.n_experts:], h[..., desc.n_experts:]) > 0.05     # the mixture is a visible part
    if backward:
        assert rel_l2(got_g, want_g) <= tol
        for b in range(B):
            assert rel_l2(got_g[b], want_g[b]) <= tol, b
        assert so.token_rel_l2(got_g.reshape(-1, D), want_g.reshape(-1, D)).max() <= 2 * tol
    return got_h, want_h


def judge_random(desc, w, h, g, got_h, got_g, routing, max_rerouted=0.05, need_clean_sequence=True, visible=True):
    """Case 2: the device's result for random router rows against the oracle.  Returns (want_h, mask of tokens routed as
    the oracle routes them)."""
    B, S = h.shape[:2]
    want_h, want_g, routes = oracle_run(h, g, w, desc)
    tol, k = TOL[desc.dtype], desc.top_k
    same = np.ones(B * S, dtype=bool)                       # routed like the oracle in every block the context kept
    upstream_clean = np.ones(B, dtype=bool)                 # sequences without a re-routed token in an earlier block
    for l in sorted(routing):
        ex, gt = routing[l]
        sel, gates, logits, n, margin = (_cat(routes, l, key) for key in ("sel", "gates", "logits", "n", "margin"))
        # |device logit - oracle logit| <= eps sum_i |n_i w_ei| per expert; a gap moves by at most twice the largest of them
        band = 2.0 * EPS[desc.dtype] * np.max(np.abs(n) @ np.abs(w[l]["w_router"].astype(np.float64)).T, axis=1)
        kth = np.sort(logits, axis=1)[:, ::-1][:, k - 1]
        chosen = np.take_along_axis(logits, ex.astype(np.int64), axis=1)
        same_l = np.all(np.sort(ex, axis=1) == np.sort(sel, axis=1), axis=1)
        judged = np.repeat(upstream_clean, S)               # this block's inputs are the oracle's up to rounding
        # a token routed differently must be a near-tie: every expert the device chose is within the band of the k-th logit
        assert np.all((chosen >= (kth - band)[:, None])[judged]), l
        # ... and a token whose margin exceeds the band cannot have been routed differently
        assert np.all(same_l[judged & (margin > band)]), l
        order_same = np.all(ex == sel, axis=1) & judged
        np.testing.assert_allclose(gt[order_same], gates[order_same], rtol=3e-2 if desc.dtype == "bf16" else 1e-4, atol=1e-6)
        same &= same_l
        upstream_clean &= same_l.reshape(B, S).all(axis=1)
    seq_same = same.reshape(B, S).all(axis=1)
    print(f"random router: {np.mean(~same):.4f} of the tokens routed to the other candidate of a near-tie, "
          f"{int(seq_same.sum())} of {B} sequences without any; relative L2 over ALL tokens: h {rel_l2(got_h, want_h):.3e}"
          + (f" g {rel_l2(got_g, want_g):.3e}" if g is not None else ""))
    assert np.mean(~same) <= max_rerouted
    assert seq_same.any() or not need_clean_sequence, "no sequence is free of near-ties: use more, shorter sequences"
    assert not visible or rel_l2(want_h, h) > 0.05
    for b in np.nonzero(seq_same)[0]:
        assert rel_l2(got_h[b], want_h[b]) <= tol, b
        assert so.token_rel_l2(got_h[b], want_h[b]).max() <= (2 * tol if desc.dtype == "f32" else tol), b
        if g is not None:
            assert rel_l2(got_g[b], want_g[b]) <= tol, b
    return want_h, same


def run_random(desc, B, S, seed, backward, plain=False, grad_std=1.0, gains=(5.0, 4.0), **kw):
    w = moe_weights(desc, seed, *gains)
    h = si.make_activations(desc, B, S, seed)
    g = si.make_output_grad(desc, B, S, seed, std=grad_std) if backward else None
    got_h, got_g, routing = run_device(desc, w, h, g, backward, plain)
    want_h, same = judge_random(desc, w, h, g, got_h, got_g, routing, **kw)
    return got_h, want_h, same


F32 = si.StageDesc(2, 64, 4, 2, 96, dtype="f32", n_experts=4, top_k=2, n_shared=1, router_norm=True)
F32_VARIANTS = {
    "sigmoid_norm_shared": F32,
    "softmax_top1": dataclasses.replace(F32, router_score="softmax", top_k=1, router_norm=False, n_shared=0),
    "softmax_norm_top3": dataclasses.replace(F32, router_score="softmax", top_k=3, n_experts=5, n_shared=2),
    "sigmoid_all_experts": dataclasses.replace(F32, top_k=4, router_norm=False),
    "sixteen_experts_top8": dataclasses.replace(F32, n_experts=16, top_k=8, n_blocks=1),
}


@pytest.mark.parametrize("name", list(F32_VARIANTS))
@pytest.mark.parametrize("backward", [False, True], ids=["fwd", "bwd"])
def test_fp32_moe_stage_matches_oracle_on_every_token(name, backward):
    run_constructed(F32_VARIANTS[name], 3, 37, seed=11, backward=backward)


@pytest.mark.parametrize("name", list(F32_VARIANTS))
def test_fp32_moe_stage_with_random_router(name):
    run_random(F32_VARIANTS[name], 6, 37, seed=11, backward=True, max_rerouted=0.01)


def test_fp32_moe_several_sort_chunks_and_an_empty_expert():
    # 700 tokens x top-2 = 1400 (token, expert) pairs: two chunks of the counting sort.  Expert 3's router row is zero
    # (score exactly 0.5) while the others share a strong common direction on top of their own, so that nearly every
    # token scores them above 0.5 or far below it together: expert 3 gets few tokens or none, and its segment is ragged
    desc = dataclasses.replace(F32, n_blocks=1, n_experts=4, top_k=2)
    w = moe_weights(desc, 5)
    w[0]["w_router"][3] = 0.0
    h = si.make_activations(desc, 2, 350, 5)
    g = si.make_output_grad(desc, 2, 350, 5, std=1.0)
    got_h, got_g, routing = run_device(desc, w, h, g, True, False)
    want_h, same = judge_random(desc, w, h, g, got_h, got_g, routing, max_rerouted=0.01, need_clean_sequence=False)
    want_g = so.stage_backward(h, g, w, desc)[1]
    assert same.mean() > 0.99
    assert rel_l2(got_h.reshape(-1, 64)[same], want_h.reshape(-1, 64)[same]) <= TOL["f32"]
    if same.all():
        assert rel_l2(got_g, want_g) <= TOL["f32"]


def test_fp32_moe_expert_that_no_token_chooses():
    # top-1 of two experts with identical router rows: every token ties and the lower index wins, so expert 1's segment
    # is empty (zero rows, zero tiles) and expert 0 holds every token
    import paper_2603_03592_amd as sv
    desc = dataclasses.replace(F32, n_blocks=1, n_experts=2, top_k=1, n_shared=0, router_norm=False)
    w = moe_weights(desc, 6)
    w[0]["w_router"][1] = w[0]["w_router"][0]
    h = si.make_activations(desc, 2, 45, 6)
    ver = sv.Verifier(desc, 90, 45)
    wc = ver.pack_weights(wd := dev_weights(w, "f32"))
    out = ver.verify_forward(wc, dev(h, "f32"), want_h_hat=True)
    ex, _ = ver.last_routing(0, 90)
    ver.close()
    assert int(ex.max()) == 0
    assert rel_l2(host(out["h_hat"]), so.stage_forward(h, w, desc)) <= TOL["f32"]


BF16_SMALL = si.StageDesc(2, 256, 4, 2, 256, n_experts=8, top_k=2, n_shared=1, router_norm=True)       # 128-row tiles
BF16_TOP1 = si.StageDesc(1, 256, 4, 4, 1024, n_experts=4, top_k=1, n_shared=0)                           # 256x256 direct-to-LDS tiles
BF16_CASES = [(BF16_SMALL, 3, 100), (BF16_TOP1, 10, 512), (dataclasses.replace(F32, dtype="bf16"), 3, 37)]
BF16_IDS = ["small_tiles", "big_tiles", "plain_shapes"]


@pytest.mark.parametrize("desc,B,S", BF16_CASES, ids=BF16_IDS)
@pytest.mark.parametrize("backward", [False, True], ids=["fwd", "bwd"])
def test_bf16_moe_stage_matches_oracle_on_every_token(desc, B, S, backward):
    """Both tile paths, forward and forward + backward: chosen experts exact, every token of h and g within 2e-2."""
    run_constructed(desc, B, S, seed=12, backward=backward, grad_std=1e-3)


@pytest.mark.parametrize("desc,B,S", BF16_CASES[:2], ids=BF16_IDS[:2])
def test_bf16_moe_stage_with_the_first_norm_inside_the_products(desc, B, S):
    """SV_FLAG_FUSE_NORM on a mixture-of-experts stage: the norm before attention runs inside the q | k | v product, the one
    before the mixture (which also feeds the router) stays a pass of its own.  Same bar as without the flag."""
    run_constructed(desc, B, S, seed=12, backward=True, grad_std=1e-3, fuse=True)


@pytest.mark.parametrize("desc,B,S", [(BF16_SMALL, 16, 25), (BF16_TOP1, 80, 64), (dataclasses.replace(F32, dtype="bf16"), 8, 16)], ids=BF16_IDS)
def test_bf16_moe_stage_with_random_router(desc, B, S):
    """Near-ties included: tokens routed to the other candidate must be valid near-ties; sequences without any are compared whole."""
    run_random(desc, B, S, seed=12, backward=True, grad_std=1e-3)


def test_bf16_moe_plain_kernels_agree_with_matrix_core_path():
    got_a, _ = run_constructed(BF16_SMALL, 2, 96, seed=13, backward=False, plain=True)
    got_b, _ = run_constructed(BF16_SMALL, 2, 96, seed=13, backward=False, plain=False)
    assert rel_l2(got_a, got_b) <= TOL["bf16"]


@pytest.mark.parametrize("name", ["moe_top1", "moe_top6"])
def test_full_size_moe_workloads_on_every_token(name):
    """The two mixture-of-experts shapes of Table model_config at the size bench.py times (8 x 1024 tokens, forward and
    backward), with the constructed routing features: every token of every sequence against the oracle, experts exact."""
    wl = si.WORKLOADS[name]
    run_constructed(wl.desc, wl.batch, wl.seq, seed=0, backward=True, grad_std=1e-3, mlp_gain=1.0, visible=False)


@pytest.mark.parametrize("name", ["moe_top1", "moe_top6"])
def test_full_size_moe_workloads_as_generated(name):
    """The same shapes with the N(0, 0.02^2) router rows as generated (what bench.py times; logit standard deviation about
    0.45): sequences of 1024 tokens always hold a near-tie, so this checks that every differently routed token IS one,
    that tokens outside the band are routed as the oracle routes them, and that the whole-signal relative L2 -- which
    includes the differently routed tokens -- stays far below the threshold a verifier would use."""
    wl = si.WORKLOADS[name]
    desc, B, S = wl.desc, wl.batch, wl.seq
    w = si.make_weights(desc, 0)
    h = si.make_activations(desc, B, S, 0)
    g = si.make_output_grad(desc, B, S, 0, std=1e-3)
    got_h, got_g, routing = run_device(desc, w, h, g, True, False)
    want_h, same = judge_random(desc, w, h, g, got_h, got_g, routing, max_rerouted=0.08, need_clean_sequence=False, visible=False)
    want_g = so.stage_backward(h, g, w, desc)[1]
    D = desc.d_model
    assert rel_l2(got_h.reshape(-1, D)[same], want_h.reshape(-1, D)[same]) <= TOL["bf16"]     # one block: h of a token depends on its own routing only
    assert rel_l2(got_h, want_h) <= TOL["bf16"] and rel_l2(got_g, want_g) <= TOL["bf16"]      # whole signal, re-routed tokens included


def test_moe_context_reuse_with_shrinking_and_growing_batches():
    """One context, three checks of different sizes in a row (the routing tables, segment padding and expert-sorted
    buffers of an earlier, larger call must not leak into a later one)."""
    import paper_2603_03592_amd as sv
    desc = dataclasses.replace(F32, n_blocks=1)
    ver = sv.Verifier(desc, 4 * 300, 300, backward=True)
    for B, S in ((4, 300), (1, 5), (3, 129)):
        w, h = si.make_moe_case_with_routing_features(desc, B, S, seed=21 + S, mlp_gain=4.0)
        wc = ver.pack_weights(wd := dev_weights(w, "f32"))
        g = si.make_output_grad(desc, B, S, 21 + S, std=1.0)
        out = ver.verify_backward(wc, dev(h, "f32"), dev(g, "f32"), want_g_hat=True, want_h_hat=True)
        want_h, want_g, routes = oracle_run(h, g, w, desc)
        ex, _ = ver.last_routing(0, B * S)
        assert np.array_equal(ex.cpu().numpy(), _cat(routes, 0, "sel")), (B, S)
        assert rel_l2(host(out["h_hat"]), want_h) <= TOL["f32"], (B, S)
        assert rel_l2(host(out["g_hat"]), want_g) <= TOL["f32"], (B, S)
    ver.close()


def test_moe_forward_check_on_a_backward_context():
    """sv_verify_forward on a context created for backward checks: same result as on a forward-only context, and
    sv_last_routing then reports THIS call's routing for every block (not what an earlier backward call left)."""
    import paper_2603_03592_amd as sv
    for desc, B, S in ((dataclasses.replace(F32, n_blocks=2), 3, 37), (BF16_SMALL, 3, 100)):
        w, h = si.make_moe_case_with_routing_features(desc, B, S, seed=31, mlp_gain=4.0)
        w_old, h_old = si.make_moe_case_with_routing_features(desc, B, S, seed=32, mlp_gain=4.0)
        g = si.make_output_grad(desc, B, S, 31, std=1.0 if desc.dtype == "f32" else 1e-3)
        ver = sv.Verifier(desc, B * S, S, backward=True)
        ver.verify_backward(ver.pack_weights(wo := dev_weights(w_old, desc.dtype)), dev(h_old, desc.dtype), dev(g, desc.dtype))   # leaves another routing behind
        out = ver.verify_forward(ver.pack_weights(wd := dev_weights(w, desc.dtype)), dev(h, desc.dtype), want_h_hat=True)
        want_h, _, routes = oracle_run(h, None, w, desc)
        for l in range(desc.n_blocks):
            ex, _ = ver.last_routing(l, B * S)
            assert np.array_equal(ex.cpu().numpy(), _cat(routes, l, "sel")), l
        assert rel_l2(host(out["h_hat"]), want_h) <= TOL[desc.dtype]
        ver.close()
        fwd = sv.Verifier(desc, B * S, S)
        out2 = fwd.verify_forward(fwd.pack_weights(wd2 := dev_weights(w, desc.dtype)), dev(h, desc.dtype), want_h_hat=True)
        assert np.array_equal(host(out2["h_hat"]), host(out["h_hat"]))
        fwd.close()


def test_last_routing_errors():
    import paper_2603_03592_amd as sv
    desc = dataclasses.replace(F32, n_blocks=2)
    w = moe_weights(desc, 3)
    ver = sv.Verifier(desc, 64, 32)                                   # forward-only: keeps the last block's routing only
    wc = ver.pack_weights(wd := dev_weights(w, "f32"))
    with pytest.raises(sv.SVError):
        ver.last_routing(1, 64)                                       # nothing has run yet
    ver.verify_forward(wc, dev(si.make_activations(desc, 2, 32, 3), "f32"))
    ex, gt = ver.last_routing(1, 64)
    assert ex.shape == (64, 2) and float(gt.sum(dim=1).min()) > 0.999  # normalised gates
    with pytest.raises(sv.SVError):
        ver.last_routing(0, 64)
    with pytest.raises(sv.SVError):
        ver.last_routing(2, 64)
    ver.close()
    dense = sv.Verifier(si.TINY.desc, 64, 64)
    with pytest.raises(sv.SVError):
        dense.last_routing(0, 64)
    dense.close()


def test_moe_descriptor_checks():
    import paper_2603_03592_amd as sv
    ok = dataclasses.replace(F32)
    assert sv.sv_check_desc(ok)[0] == 0
    assert sv.sv_check_desc(dataclasses.replace(ok, top_k=5))[0] == 1                 # top_k > n_experts
    assert sv.sv_check_desc(dataclasses.replace(ok, n_experts=17, top_k=2))[0] == 2   # more experts than the kernels hold
    assert sv.sv_check_desc(dataclasses.replace(ok, mlp="gelu"))[0] == 2
