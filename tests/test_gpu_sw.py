"""GPU parity: sv_sliced_wasserstein against the CPU oracle.

Tolerance.  The oracle projects in float64; the library accumulates exact bf16 x bf16 (or split
fp32) products in fp32, so a projected value is off by at most ~sqrt(D) 2^-24 of the row's scale.
Sorting is 1-Lipschitz in the sup norm, hence |SW_gpu - SW_oracle| <= (error of claim projections)
+ (error of reference projections); the checks allow 1e-5 of the mean |projection| plus 1e-3
relative (the sums over T samples are fp32)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import stage_inputs as si
from oracle import sentinel_oracle as sn
from gpu_util import dev, host

KINDS = ["honest", "scale", "noise", "sign", "zero", "tok_scale"]


def _ver(max_tokens):
    import paper_2603_03592_amd as sv
    return sv, sv.Verifier(si.TINY.desc, max_tokens, 64, sliced_w=True)


def _signal(T, D, dtype, seed):
    g = np.random.default_rng(seed)
    return si.to_stage_dtype((1.3 * g.standard_normal((T, D)) + 0.1).astype(np.float32), dtype)


def _check(got, claims, refs, u, flags=None, tau=None):
    for i, c in enumerate(claims):
        r = refs[i] if len(refs) > 1 else refs[0]
        want = sn.sliced_wasserstein(c, r, u)
        scale = float(np.mean(np.abs(np.asarray(r, np.float64) @ np.asarray(u, np.float64).T)))
        assert abs(got[i] - want) <= 1e-3 * want + 1e-5 * scale, (i, got[i], want)
        if flags is not None and abs(want / tau - 1.0) > 0.05:
            assert bool(flags[i]) == (not want <= tau), (i, want, tau)


@pytest.mark.parametrize("cd,rd", [("bf16", "bf16"), ("bf16", "f32"), ("f32", "f32"), ("f32", "bf16")])
@pytest.mark.parametrize("shared", [True, False])
@pytest.mark.parametrize("T,L", [(300, 64), (128, 32), (1000, 96)])
def test_sw_matches_oracle_ragged(cd, rd, shared, T, L):
    sv, ver = _ver(1024)
    D = 192
    u = si.make_directions(D, L, seed=T)
    refs = [_signal(T, D, rd, 10 + i) for i in range(1 if shared else len(KINDS))]
    claims = [si.make_claim(k, refs[0 if shared else i].astype(np.float32), cd, seed=i) for i, k in enumerate(KINDS)]
    import torch
    cl = torch.stack([dev(c, cd) for c in claims])
    rf = dev(refs[0], rd) if shared else torch.stack([dev(r, rd) for r in refs])
    tau = 0.02
    res = ver.score_and_flag(cl, rf, tau={"rel_l2": 1e9})["result"]          # nothing flagged by the first statistic
    sw = ver.sliced_wasserstein(cl, rf, dev(u, "bf16"), tau, results=res)
    out = ver.read_results(res)
    _check(host(sw), claims, refs, u, flags=out["flag"], tau=tau)
    assert all(int(m) & sv.binding.SV_M_SW for m in out["metric_mask"])
    ver.close()


def test_sw_identical_and_permuted_tokens():
    sv, ver = _ver(512)
    T, D, L = 500, 128, 64
    u = si.make_directions(D, L, seed=1)
    r = _signal(T, D, "bf16", 0)
    perm = np.random.default_rng(3).permutation(T)
    import torch
    cl = torch.stack([dev(r, "bf16"), dev(r[perm], "bf16")])
    sw = host(ver.sliced_wasserstein(cl, dev(r, "bf16"), dev(u, "bf16"), 1.0))
    assert sw[0] == 0.0                                   # same inputs, same arithmetic, same order
    assert sw[1] <= 1e-6                                  # a distance between sample sets
    # an element-wise statistic sees the permuted submission as completely different
    res = ver.read_results(ver.score_and_flag(cl, dev(r, "bf16"), tau={"rel_l2": 0.5})["result"])
    assert list(res["flag"]) == [0, 1]
    ver.close()


def test_sw_long_rows_take_the_global_merge_steps():
    sv, ver = _ver(40000)
    T, D, L = 40000, 64, 32                               # padded to 65536 = 4 LDS chunks
    u = si.make_directions(D, L, seed=2)
    r = _signal(T, D, "bf16", 1)
    kinds = ["honest", "scale", "noise"]
    claims = [si.make_claim(k, r, "bf16", seed=i) for i, k in enumerate(kinds)]
    import torch
    sw = ver.sliced_wasserstein(torch.stack([dev(c, "bf16") for c in claims]), dev(r, "bf16"), dev(u, "bf16"), 1.0)
    _check(host(sw), claims, [r], u)
    ver.close()


def test_sw_many_submissions_span_several_groups():
    sv, ver = _ver(256)
    T, D, L = 256, 64, 128                                # 32 submissions per group with a shared reference, 16 with own ones
    u = si.make_directions(D, L, seed=3)
    refs = [_signal(T, D, "bf16", 100 + i) for i in range(45)]
    claims = [si.make_claim(KINDS[i % len(KINDS)], refs[i], "bf16", seed=i) for i in range(45)]
    import torch
    cl = torch.stack([dev(c, "bf16") for c in claims])
    sw = ver.sliced_wasserstein(cl, torch.stack([dev(r, "bf16") for r in refs]), dev(u, "bf16"), 1.0)
    _check(host(sw), claims, refs, u)
    sw = ver.sliced_wasserstein(cl, dev(refs[0], "bf16"), dev(u, "bf16"), 1.0)
    _check(host(sw), claims, refs[:1], u)
    ver.close()


def test_sw_non_finite_submission_is_flagged_and_limits():
    sv, ver = _ver(256)
    T, D, L = 200, 64, 32
    u = dev(si.make_directions(D, L, seed=4), "bf16")
    r = _signal(T, D, "bf16", 0)
    bad = r.copy(); bad[17, 5] = np.nan
    import torch
    cl = torch.stack([dev(r, "bf16"), dev(bad, "bf16")])
    clean = torch.stack([dev(r, "bf16"), dev(r, "bf16")])
    res = ver.score_and_flag(clean, dev(r, "bf16"), tau={"rel_l2": 1e9})["result"]        # both un-flagged so far
    sw = host(ver.sliced_wasserstein(cl, dev(r, "bf16"), u, 1e9, results=res))
    out = ver.read_results(res)
    assert sw[0] == 0.0 and not np.isfinite(sw[1])
    assert out["flag"][1] == 1
    # limits are refused, not mis-computed
    with pytest.raises(sv.SVError):
        ver.sliced_wasserstein(cl, dev(r, "bf16"), dev(si.make_directions(D, 48, 0), "bf16"), 1.0)
    with pytest.raises(sv.SVError):
        ver.sliced_wasserstein(cl[:, :, :32].contiguous(), dev(r[:, :32], "bf16"), dev(si.make_directions(32, 32, 0), "bf16"), 1.0)
    big = torch.zeros((1, 300, D), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(sv.SVError):
        ver.sliced_wasserstein(big, big[0], u, 1.0)                               # T above the context's max_tokens
    ver.close()
    plain = sv.Verifier(si.TINY.desc, 256, 64)
    with pytest.raises(sv.SVError):
        plain.sliced_wasserstein(cl, dev(r, "bf16"), u, 1.0)                      # context without the scratch
    plain.close()


def test_sw_against_projection_and_projection_ema():
    """The statistic against a reference known only through its projections equals the statistic against the reference,
    and the projections of the EMA follow from those of the submissions (linearity of the projection)."""
    import torch
    sv, ver = _ver(1024)
    T, D, L, beta = 700, 256, 64, 0.8
    u = si.make_directions(D, L, seed=5)
    g = np.random.default_rng(5)
    m = (0.7 * g.standard_normal((T, D))).astype(np.float32)
    claims = [si.make_claim(k, m, "bf16", seed=i) for i, k in enumerate(KINDS)]
    Tpad = sv.lib.sv_sw_row_len(T)
    assert Tpad == 1024
    uq = np.asarray(si.to_stage_dtype(u, "bf16"), np.float64)
    pm = np.zeros((L, Tpad), np.float32)
    pm[:, :T] = (m.astype(np.float64) @ uq.T).T
    pm[:, T:] = -123.0                                  # padding of the caller's array is ignored
    pm_dev = dev(pm, "f32")
    cl = torch.stack([dev(c, "bf16") for c in claims])
    sw, proj = ver.sw_against_projection(cl, pm_dev, dev(u, "bf16"), 1.0)
    _check(host(sw), claims, [m], u)
    direct = ver.sliced_wasserstein(cl, dev(m, "f32"), dev(u, "bf16"), 1.0)
    np.testing.assert_allclose(host(sw), host(direct), rtol=1e-4, atol=1e-6)
    want_p = np.stack([(np.asarray(c, np.float64) @ uq.T).T for c in claims])
    np.testing.assert_allclose(host(proj)[:, :, :T], want_p, rtol=1e-5, atol=1e-5)
    # EMA over the submissions 0, 2, 3 (1, 4, 5 skipped): projections of the new EMA
    skip = [0, 1, 0, 0, 1, 1]
    ver.sw_projection_ema(pm_dev, proj, T, skip, beta)
    m_new = beta * m.astype(np.float64) + (1 - beta) * np.mean([np.asarray(c, np.float64) for c, k in zip(claims, skip) if not k], axis=0)
    np.testing.assert_allclose(host(pm_dev)[:, :T], (m_new @ uq.T).T, rtol=1e-5, atol=1e-5)
    # nobody left: unchanged
    before = host(pm_dev).copy()
    ver.sw_projection_ema(pm_dev, proj, T, [1] * 6, beta)
    assert np.array_equal(host(pm_dev), before)
    ver.close()


def test_sw_against_projection_limits():
    """256 submissions x 128 directions in one call (32768 rows in one sort launch); 257 submissions and rows beyond one
    LDS chunk are refused."""
    import torch
    sv, ver = _ver(20000)
    T, D, L, n = 128, 64, 128, 256
    u = si.make_directions(D, L, seed=6)
    uq = np.asarray(si.to_stage_dtype(u, "bf16"), np.float64)
    g = np.random.default_rng(6)
    m = g.standard_normal((T, D)).astype(np.float32)
    claims = [si.to_stage_dtype(m + np.float32(0.01 * (i % 7)) * g.standard_normal((T, D)).astype(np.float32), "bf16") for i in range(n)]
    pm = dev((m.astype(np.float64) @ uq.T).T.astype(np.float32), "f32")
    cl = torch.stack([dev(c, "bf16") for c in claims])
    sw, proj = ver.sw_against_projection(cl, pm, dev(u, "bf16"), 1.0)
    _check(host(sw)[::37], claims[::37], [m], u)
    with pytest.raises(sv.SVError):
        ver.sw_against_projection(torch.cat([cl, cl[:1]]), pm, dev(u, "bf16"), 1.0)
    big = torch.zeros((1, 20000, D), dtype=torch.bfloat16, device="cuda")            # row length 32768 > 16384
    with pytest.raises(sv.SVError):
        ver.sw_against_projection(big, torch.zeros((L, 32768), dtype=torch.float32, device="cuda"), dev(u, "bf16"), 1.0)
    ver.close()
