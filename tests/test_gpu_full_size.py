"""GPU parity at the benchmark configurations' full sizes, in the launch configuration bench.py
times (same context limits, same kernels): recomputed activations / gradients against the CPU
oracle, and the flag decisions for the configurations' claim mixes.

The oracle needs roughly 1 s (Small) to 90 s (Large) per distinct micro-batch on the GPU machine's
host cores, so each configuration uses few distinct micro-batches and manufactures all of its
submissions from the oracle's output for those:
  Small  : 8 micro-batches x 8 submissions = 64 (10 % scaled x1.5, 10 % sign-flipped on 5 % of channels)
  Medium : 2 micro-batches, forward + backward; on the first 10 gradient submissions, 2 corrupted (zeroed / noise)
  Large  : 1 micro-batch; 32 submissions, 8 corrupted on 1 % of the tokens only
  Sweep  : the S=512, B=1 point whole; at (S=2048, B=4) and (S=4096, B=16) the device runs the whole micro-batch and the
           oracle recomputes sampled sequences of it (the stage map acts on every sequence on its own: Problem Statement,
           "Threat Model" paragraph), forward + backward
  Loop   : one stage call of the verifier loop (16 workers x [8192, 4096]): statistics + sum, EMA, projections
"""
import dataclasses

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import stage_inputs as si
from oracle import stage_oracle as so
from gpu_util import assert_close, dev, dev_weights, host, rel_l2


def _flag_check(res, claim, ref, tau, expect_bad, tag):
    want = so.scores(claim, ref)["rel_l2"]
    assert so.flag({"rel_l2": want}, {"rel_l2": tau}) == expect_bad, (tag, want)
    if abs(want / tau - 1.0) > 0.05:                       # bit-exact outside the +-5 % band
        assert bool(res["flag"]) == expect_bad, (tag, res, want)
    return want


def test_small_config_64_submissions():
    import paper_2603_03592_amd as sv
    wl = si.SMALL
    w = si.make_weights(wl.desc, 0)
    assert sv.fuse_norm_pays(wl.desc)                       # as bench.py runs it: the norms inside the products
    ver = sv.Verifier(wl.desc, wl.batch * wl.seq, wl.seq, fuse_norm=True)
    wd = dev_weights(w, "bf16")
    wc = ver.pack_weights(wd)
    ver.prepare_weights(wc)
    kinds = si.small_claim_plan(64, seed=0)
    assert kinds.count("scale") == 6 and kinds.count("sign") == 6
    worst_honest, n = 0.0, 0
    for mb in range(8):
        h = si.make_activations(wl.desc, wl.batch, wl.seq, seed=0, micro_batch=mb)
        ref = so.stage_forward(h, w, wl.desc)
        hd = dev(h, "bf16")
        out = ver.verify_forward(wc, hd, want_h_hat=True)
        assert_close(host(out["h_hat"]), ref, 2e-2, ("small", mb))
        for j in range(8):
            kind = kinds[mb * 8 + j]
            claim = si.make_claim(kind, ref, "bf16", seed=mb * 8 + j)
            res = ver.read_results(ver.verify_forward(wc, hd, dev(claim, "bf16"), tau={"rel_l2": wl.tau})["result"])[0]
            _flag_check(res, claim, ref, wl.tau, kind != "honest", (mb, j, kind))
            if kind == "honest":
                worst_honest = max(worst_honest, float(res["score"][0]))
            n += 1
    assert n == 64
    assert worst_honest < 0.95 * wl.tau, worst_honest        # honest submissions keep clear of the band
    print(f"small: worst honest per-token score {worst_honest:.3e} (tau {wl.tau})")
    ver.close()


def test_medium_config_forward_backward():
    import paper_2603_03592_amd as sv
    wl = si.MEDIUM
    w = si.make_weights(wl.desc, 0)
    ver = sv.Verifier(wl.desc, wl.batch * wl.seq, wl.seq, backward=True, fuse_norm=True)
    wd = dev_weights(w, "bf16")
    wc = ver.pack_weights(wd)
    ver.prepare_weights(wc)
    for mb in (0, 1):                                      # two distinct micro-batches
        h = si.make_activations(wl.desc, wl.batch, wl.seq, seed=0, micro_batch=mb)
        g = si.make_output_grad(wl.desc, wl.batch, wl.seq, seed=0, micro_batch=mb)
        ref_h, ref_g = so.stage_backward(h, g, w, wl.desc)
        hd, gd = dev(h, "bf16"), dev(g, "bf16")
        out = ver.verify_backward(wc, hd, gd, want_g_hat=True, want_h_hat=True)
        eh = assert_close(host(out["h_hat"]), ref_h, 2e-2, ("medium h", mb))
        eg = assert_close(host(out["g_hat"]), ref_g, 2e-2, ("medium g", mb))
        print(f"medium[{mb}]: rel-L2 h {eh[0]:.3e} (worst token {eh[1]:.3e}, worst element {eh[2]:.2f} of its bound) "
              f"g {eg[0]:.3e} (worst token {eg[1]:.3e}, worst element {eg[2]:.2f})")
        # activation gradients are three orders of magnitude smaller than activations
        assert np.sqrt(np.mean(ref_g ** 2)) < 1e-2 * np.sqrt(np.mean(ref_h ** 2))
        if mb:
            continue
        kinds = ["honest"] * 10
        kinds[3], kinds[7] = "zero", "noise"
        for i, kind in enumerate(kinds):
            claim = si.make_claim(kind, ref_g, "bf16", seed=i)
            res = ver.read_results(ver.verify_backward(wc, hd, gd, dev(claim, "bf16"), tau={"rel_l2": wl.tau})["result"])[0]
            _flag_check(res, claim, ref_g, wl.tau, kind != "honest", (i, kind))
            if kind == "honest":
                assert res["score"][0] < 0.95 * wl.tau, res
        claim = si.make_claim("honest", ref_h, "bf16", 0)
        res = ver.read_results(ver.verify_forward(wc, hd, dev(claim, "bf16"), tau={"rel_l2": wl.tau})["result"])[0]
        _flag_check(res, claim, ref_h, wl.tau, False, "h honest")
    ver.close()


def test_norms_inside_the_products_with_a_ragged_row_tail_on_the_large_tile():
    """5 x 1257 = 6285 tokens against one block of the medium stage's width: every product runs on the 256 x 256 kernel
    (200 row-by-column tiles and more) and the last of the 25 row tiles has 141 rows, so the row factors are fetched and
    the rows' sums of squares are stored by the epilogue's row-checked form; two blocks, so that the second block's first
    norm takes its sums from the first block's down-projection.  Forward and backward."""
    import paper_2603_03592_amd as sv
    desc = dataclasses.replace(si.MEDIUM.desc, n_blocks=2)
    B, S = 5, 1257
    w = si.make_weights(desc, 4)
    h = si.make_activations(desc, B, S, seed=4)
    g = si.make_output_grad(desc, B, S, seed=4)
    ref_h, ref_g = so.stage_backward(h, g, w, desc)
    ver = sv.Verifier(desc, B * S, S, backward=True, fuse_norm=True)
    wc = ver.pack_weights(wd := dev_weights(w, "bf16"))
    ver.prepare_weights(wc)
    out = ver.verify_backward(wc, dev(h, "bf16"), dev(g, "bf16"), want_g_hat=True, want_h_hat=True)
    eh = assert_close(host(out["h_hat"]), ref_h, 2e-2, "ragged fused h")
    eg = assert_close(host(out["g_hat"]), ref_g, 2e-2, "ragged fused g")
    print(f"ragged rows, norms inside the products: h {eh[0]:.3e} / {eh[1]:.3e} / {eh[2]:.2f}   g {eg[0]:.3e} / {eg[1]:.3e} / {eg[2]:.2f}")
    prof_ops = None
    ver.profile_enable(True)
    ver.verify_forward(wc, dev(h, "bf16"))
    prof_ops = ver.profile_read()
    ver.profile_enable(False)
    # 2 blocks x 2 norms = 4 row-factor kernels, and no stand-alone norm pass ran
    assert prof_ops["norm_pieces"]["launches"] == 4 and prof_ops["norm"]["launches"] == 0, (prof_ops["norm_pieces"], prof_ops["norm"])
    ver.close()


def test_large_config_32_submissions_token_corruption():
    import paper_2603_03592_amd as sv
    wl = si.LARGE
    w = si.make_weights(wl.desc, 0)
    h = si.make_activations(wl.desc, wl.batch, wl.seq, seed=0)
    ref = so.stage_forward(h, w, wl.desc)
    wd = dev_weights(w, "bf16")
    hd = dev(h, "bf16")
    # the other form of the norms first (inside the products: row sums from the large tile's residual epilogue, the
    # one-launch q | k | v product and the gate / up product scaling their rows), then the one bench.py times here
    assert not sv.fuse_norm_pays(wl.desc)
    ver = sv.Verifier(wl.desc, wl.batch * wl.seq, wl.seq, fuse_norm=True)
    wc = ver.pack_weights(wd)
    ver.prepare_weights(wc)
    e = assert_close(host(ver.verify_forward(wc, hd, want_h_hat=True)["h_hat"]), ref, 2e-2, "large, norms inside the products")
    print(f"large, norms inside the products: rel-L2 {e[0]:.3e} worst token {e[1]:.3e} worst element {e[2]:.2f} of its bound")
    ver.close()
    ver = sv.Verifier(wl.desc, wl.batch * wl.seq, wl.seq)
    wc = ver.pack_weights(wd)
    got = host(ver.verify_forward(wc, hd, want_h_hat=True)["h_hat"])
    e = assert_close(got, ref, 2e-2, "large")
    print(f"large: rel-L2 {e[0]:.3e} worst token {e[1]:.3e} worst element {e[2]:.2f} of its bound")
    bad_kinds = ["tok_noise", "tok_scale", "tok_neg", "tok_zero"]
    kinds = ["honest"] * 32
    for i, slot in enumerate(range(1, 32, 4)):             # 8 of 32 corrupted
        kinds[slot] = bad_kinds[i % 4]
    worst_honest = 0.0
    for i, kind in enumerate(kinds):
        claim = si.make_claim(kind, ref, "bf16", seed=i)
        out = ver.verify_forward(wc, hd, dev(claim, "bf16"), tau={"rel_l2": wl.tau}, want_token_scores=True)
        res = ver.read_results(out["result"])[0]
        _flag_check(res, claim, ref, wl.tau, kind != "honest", (i, kind))
        if kind == "honest":
            worst_honest = max(worst_honest, float(res["score"][0]))
        else:
            # only the corrupted 1 % of the tokens stand out
            ts = host(out["token_scores"])
            n_bad = int(np.sum(ts > wl.tau))
            assert n_bad == 82, (kind, n_bad)
    assert worst_honest < 0.95 * wl.tau, worst_honest
    print(f"large: worst honest per-token score {worst_honest:.3e} (tau {wl.tau})")
    ver.close()


def test_sweep_point_forward_backward():
    import paper_2603_03592_amd as sv
    wl = si.sweep_point(512, 1)
    w = si.make_weights(wl.desc, 1)
    h = si.make_activations(wl.desc, wl.batch, wl.seq, seed=1)
    g = si.make_output_grad(wl.desc, wl.batch, wl.seq, seed=1)
    ref_h, ref_g = so.stage_backward(h, g, w, wl.desc)
    ver = sv.Verifier(wl.desc, wl.batch * wl.seq, wl.seq, backward=True, fuse_norm=sv.fuse_norm_pays(wl.desc))
    wd = dev_weights(w, "bf16")
    wc = ver.pack_weights(wd)
    ver.prepare_weights(wc)
    out = ver.verify_backward(wc, dev(h, "bf16"), dev(g, "bf16"), want_g_hat=True, want_h_hat=True)
    assert_close(host(out["h_hat"]), ref_h, 2e-2, "sweep 512x1 h")
    assert_close(host(out["g_hat"]), ref_g, 2e-2, "sweep 512x1 g")
    # 128 concurrent submissions scored in one call against the recomputation (shared reference)
    import torch
    kinds = (["honest"] * 5 + ["noise", "scale", "sign"]) * 16
    claims = torch.stack([dev(si.make_claim(k, ref_h, "bf16", i), "bf16") for i, k in enumerate(kinds)])
    res = ver.read_results(ver.score_and_flag(claims, out["h_hat"], tau={"rel_l2": wl.tau})["result"])
    assert [int(f) for f in res["flag"]] == [int(k != "honest") for k in kinds]
    ver.close()


@pytest.mark.parametrize("S,B,sampled", [(512, 4, (1,)), (512, 16, (0, 9)), (2048, 1, (0,)), (2048, 4, (0, 3)), (2048, 16, (7,)),
                                         (4096, 1, (0,)), (4096, 4, (2,)), (4096, 16, (15,))],
                         ids=["s512_b4", "s512_b16", "s2048_b1", "s2048_b4", "s2048_b16", "s4096_b1", "s4096_b4", "s4096_b16"])
def test_sweep_points_at_size_on_sampled_sequences(S, B, sampled):
    """The sweep's larger points in the launch configuration bench.py --sweep times (context sized for the point, whole
    micro-batch on the device, weights prepared once): the oracle recomputes the sampled sequences forward and backward
    and those rows of the device's h and g are compared like every other recompute (whole, per token, per element)."""
    import paper_2603_03592_amd as sv
    wl = si.sweep_point(S, B)
    w = si.make_weights(wl.desc, 1)
    h = si.make_activations(wl.desc, B, S, seed=2)
    g = si.make_output_grad(wl.desc, B, S, seed=2)
    refs = {b: so.stage_backward(h[b:b + 1], g[b:b + 1], w, wl.desc) for b in sampled}
    wd = dev_weights(w, "bf16")
    # one point also with the norms inside the products (forward and backward at the large tile's sizes), which
    # bench.py does not time at this width
    for fuse in ((sv.fuse_norm_pays(wl.desc), True) if (S, B) == (2048, 4) else (sv.fuse_norm_pays(wl.desc),)):
        ver = sv.Verifier(wl.desc, B * S, S, backward=True, fuse_norm=fuse)
        wc = ver.pack_weights(wd)
        ver.prepare_weights(wc)
        out = ver.verify_backward(wc, dev(h, "bf16"), dev(g, "bf16"), want_g_hat=True, want_h_hat=True)
        got_h, got_g = out["h_hat"], out["g_hat"]
        for b in sampled:
            ref_h, ref_g = refs[b]
            eh = assert_close(host(got_h[b:b + 1]), ref_h, 2e-2, (S, B, b, "h", fuse))
            eg = assert_close(host(got_g[b:b + 1]), ref_g, 2e-2, (S, B, b, "g", fuse))
            print(f"sweep S={S} B={B} sequence {b}{', norms inside the products' if fuse else ''}: h {eh[0]:.3e} / {eh[1]:.3e} / {eh[2]:.2f}"
                  f"   g {eg[0]:.3e} / {eg[1]:.3e} / {eg[2]:.2f}   (whole / worst token / worst element in units of its bound)")
        ver.close()


def test_large_shape_sliced_wasserstein_32_submissions():
    """Omega_SW at the large configuration's signal shape ([8192, 4096] bf16, 64 directions, 32 submissions against one
    shared reference): every value against the oracle.  The reference here is a synthetic signal of the stage
    output's shape (the statistic does not depend on where the reference came from)."""
    import torch
    import paper_2603_03592_amd as sv
    from oracle import sentinel_oracle as sn
    T, D, L, n = 8192, 4096, 64, 32
    ver = sv.Verifier(si.TINY.desc, T, 64, sliced_w=True)
    g = np.random.default_rng(0)
    ref = si.round_to_bf16((1.3 * g.standard_normal((T, D)) + 0.1).astype(np.float32))
    u = si.make_directions(D, L, 0)
    kinds = ["honest"] * n
    for i, slot in enumerate(range(1, n, 4)):
        kinds[slot] = ["tok_noise", "scale", "sign", "noise"][i % 4]
    claims_np = [si.make_claim(k, ref, "bf16", seed=i) for i, k in enumerate(kinds)]
    claims = torch.stack([dev(c, "bf16") for c in claims_np])
    sw = host(ver.sliced_wasserstein(claims, dev(ref, "bf16"), dev(u, "bf16"), 1e-2))
    scale = float(np.mean(np.abs(ref.astype(np.float64) @ u.astype(np.float64).T)))
    worst = 0.0
    for i, c in enumerate(claims_np):
        want = sn.sliced_wasserstein(c, ref, u)             # the oracle's routine for every compared value
        assert abs(sw[i] - want) <= 1e-3 * want + 1e-5 * scale, (i, kinds[i], sw[i], want)
        worst = max(worst, abs(sw[i] - want) / max(want, 1e-30))
    print(f"large-shape SW: worst relative difference {worst:.2e}; honest {sw[0]:.3e}, scaled {sw[5]:.3e}")
    ver.close()


def test_loop_shape_stage_call_16_workers():
    """One stage call of the verifier loop at the shape bench.py --loop-bench times (16 workers x [8192, 4096] bf16
    against an fp32 EMA, 64 directions): the statistics and the sum from one pass, the EMA from that sum, the sliced
    Wasserstein statistic against the EMA's projections and their update -- sampled submissions against the oracle,
    the sum and both updates element by element."""
    import torch
    import paper_2603_03592_amd as sv
    from oracle import sentinel_oracle as sn
    T, D, L, n, beta = 8192, 4096, 64, 16, 0.9
    ver = sv.Verifier(si.TINY.desc, T, 64, sliced_w=True)
    g = np.random.default_rng(7)
    m = (0.9 * g.standard_normal((T, D))).astype(np.float32)
    claims_np = []
    for r in range(n):                                     # workers scatter around the EMA; two of them attack
        x = m + 0.5 * g.standard_normal((T, D)).astype(np.float32)
        kind = {5: "scale", 11: "sign"}.get(r, "honest")
        claims_np.append(si.make_claim(kind, x, "bf16", seed=r))
    skip = [int(r == 3) for r in range(n)]
    claims = torch.stack([dev(c, "bf16") for c in claims_np])
    m_dev = dev(m, "f32")
    metrics = ("rel_l2", "l1", "zl2", "sfr")
    out = ver.score_and_sum(claims, m_dev, skip=skip, metrics=metrics, tau={k: 1e9 for k in metrics}, reduce="global")
    res = ver.read_results(out["result"])
    for i in (0, 5, 11, 15):
        want = so.scores(claims_np[i], m, "global")
        got = dict(zip(so.METRICS, res["score"][i]))
        for k in metrics:
            tol = dict(rel=1e-4, abs=5e-6) if k == "zl2" else dict(rel=3e-5, abs=2e-7)
            assert got[k] == pytest.approx(want[k], **tol), (i, k, got, want)
    total = np.zeros((T, D)); mag = np.zeros((T, D))
    for c, k in zip(claims_np, skip):
        if not k:
            c64 = np.asarray(c, np.float64); total += c64; mag += np.abs(c64)
    assert np.all(np.abs(host(out["sum"]) - total) <= 2e-7 * 15 * mag + 1e-30)
    # sliced Wasserstein against the EMA's projections
    u = si.make_directions(D, L, 0)
    uq = np.asarray(si.to_stage_dtype(u, "bf16"), np.float64)
    assert sv.lib.sv_sw_row_len(T) == T
    pm = (m.astype(np.float64) @ uq.T).T.astype(np.float32)
    pm_dev = dev(pm, "f32")
    sw, proj = ver.sw_against_projection(claims, pm_dev, dev(u, "bf16"), 1e9)
    sw = host(sw)
    scale = float(np.mean(np.abs(m.astype(np.float64) @ uq.T)))
    for i in (0, 5, 11):
        want = sn.sliced_wasserstein(claims_np[i], m, uq)
        assert abs(sw[i] - want) <= 1e-3 * want + 1e-5 * scale, (i, sw[i], want)
    # both updates over the 15 un-skipped workers: Eq. momentum_def by the oracle's routine
    ver.ema_from_sum(m_dev, out["sum"], 15, beta)
    m_new = so.ema_update(m, claims_np, skip, beta)
    np.testing.assert_allclose(host(m_dev), m_new, rtol=2e-6, atol=2e-6)
    ver.sw_projection_ema(pm_dev, proj, T, skip, beta)
    np.testing.assert_allclose(host(pm_dev), (m_new @ uq.T).T, rtol=1e-4, atol=1e-4 * scale)      # projections of the oracle's EMA
    ver.close()
