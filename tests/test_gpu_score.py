"""GPU parity: sv_score_and_flag and sv_ema_update against the CPU oracle, element by element."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import stage_inputs as si
from oracle import stage_oracle as so
from gpu_util import dev, host

TAU = {"rel_l2": 2e-2, "l1": 0.05, "zl2": 0.01, "sfr": 0.02}


def _verifier():
    import paper_2603_03592_amd as sv
    return sv, sv.Verifier(si.TINY.desc, 128, 64)


def _claims(ref, dtype, seed):
    kinds = ["honest", "scale", "sign", "zero", "noise", "tok_scale", "tok_zero"]
    out = [si.make_claim(k, ref, dtype, seed + i) for i, k in enumerate(kinds)]
    # an honest worker with a different rounding order: tiny relative jitter
    g = np.random.default_rng(seed)
    out.append(si.to_stage_dtype(ref * (1 + 1e-3 * g.standard_normal(ref.shape).astype(np.float32)), dtype))
    return kinds + ["jitter"], out


def _compare(res, tok, claims, refs, reduce, metrics):
    tau = {m: TAU[m] for m in metrics}
    for i, c in enumerate(claims):
        r = refs[i] if len(refs) > 1 else refs[0]
        want = so.scores(c, r, reduce)
        got = dict(zip(so.METRICS, res["score"][i]))
        for m in so.METRICS:
            if m not in metrics:
                assert got[m] == 0.0        # sums of metrics outside the mask are not formed
                continue
            # zl2 is formed from moments, so a true zero comes out as rounding noise of the variances
            tol = dict(rel=1e-4, abs=5e-6) if m == "zl2" else dict(rel=3e-5, abs=2e-7)
            assert got[m] == pytest.approx(want[m], **tol), (i, m, got, want)
        wf = so.flag(want, tau)
        margin = min(abs(want[m] / tau[m] - 1.0) for m in tau)
        if margin > 0.05:
            assert bool(res["flag"][i]) == wf, (i, got, want)
        wt = so.token_rel_l2(c, r)
        np.testing.assert_allclose(tok[i], wt, rtol=3e-5, atol=1e-7)
        assert res["max_token_rell2"][i] == pytest.approx(wt.max(), rel=3e-5)
        assert wt[res["argmax_token"][i]] == pytest.approx(wt.max(), rel=1e-4)


@pytest.mark.parametrize("cd,rd", [("f32", "f32"), ("bf16", "bf16"), ("bf16", "f32"), ("f32", "bf16")])
@pytest.mark.parametrize("shared", [True, False])
@pytest.mark.parametrize("reduce", ["max_token", "global"])
def test_scores_and_flags_match_oracle_ragged(cd, rd, shared, reduce):
    sv, ver = _verifier()
    T, D = 50, 72                                  # T not a multiple of the 16-token tile, D of 512
    g = np.random.default_rng(1)
    base = si.to_stage_dtype((1.3 * g.standard_normal((T, D)) + 0.1).astype(np.float32), rd)
    kinds, claims = _claims(base, cd, seed=3)
    n = len(claims)
    if shared:
        refs = [base]
        ref_dev = dev(base, rd)
    else:
        refs = [si.to_stage_dtype(base * np.float32(1 + 0.01 * i), rd) for i in range(n)]
        ref_dev = dev(np.stack(refs), rd)
    metrics = ("rel_l2", "l1", "zl2", "sfr")
    out = ver.score_and_flag(dev(np.stack(claims), cd), ref_dev, metrics=metrics, tau=TAU, reduce=reduce, want_token_scores=True)
    res = ver.read_results(out["result"])
    _compare(res, host(out["token_scores"]), claims, refs, reduce, metrics)
    assert list(res["metric_mask"]) == [15] * n
    ver.close()


def test_scores_many_tiles_bf16_and_single_metric_mask():
    sv, ver = _verifier()
    T, D = 3000, 1024
    g = np.random.default_rng(2)
    base = si.to_stage_dtype(g.standard_normal((T, D)).astype(np.float32), "bf16")
    kinds, claims = _claims(base, "bf16", seed=5)
    out = ver.score_and_flag(dev(np.stack(claims), "bf16"), dev(base, "bf16"), metrics=("rel_l2",), tau=TAU, want_token_scores=True)
    res = ver.read_results(out["result"])
    _compare(res, host(out["token_scores"]), claims, [base], "max_token", ("rel_l2",))
    flags = dict(zip(kinds, res["flag"]))
    assert flags == {"honest": 0, "scale": 1, "sign": 1, "zero": 1, "noise": 1, "tok_scale": 1, "tok_zero": 1, "jitter": 0}
    # with only the sign-flip metric enabled a positive scaling goes unnoticed
    out = ver.score_and_flag(dev(np.stack(claims), "bf16"), dev(base, "bf16"), metrics=("sfr",), tau=TAU)
    flags = dict(zip(kinds, ver.read_results(out["result"])["flag"]))
    assert flags["scale"] == 0 and flags["zero"] == 1 and flags["sign"] == 1
    ver.close()


def test_threshold_is_strict_and_nonfinite_is_flagged():
    sv, ver = _verifier()
    ref = np.ones((16, 8), np.float32)
    claim = ref.copy()
    claim[:, :] = 1.5                                # every score is exactly 0.5 / 0.5 / -, representable
    out = ver.score_and_flag(dev(claim[None], "f32"), dev(ref, "f32"), metrics=("rel_l2", "l1"), tau={"rel_l2": 0.5, "l1": 0.5})
    res = ver.read_results(out["result"])
    assert res["score"][0][0] == 0.5 and res["score"][0][1] == 0.5 and res["flag"][0] == 0     # equal is not above
    out = ver.score_and_flag(dev(claim[None], "f32"), dev(ref, "f32"), metrics=("rel_l2",), tau={"rel_l2": np.nextafter(np.float32(0.5), np.float32(0))})
    assert ver.read_results(out["result"])["flag"][0] == 1
    bad = claim.copy()
    bad[3, 2] = np.nan
    out = ver.score_and_flag(dev(bad[None], "f32"), dev(ref, "f32"), metrics=("rel_l2",), tau={"rel_l2": 10.0})
    assert ver.read_results(out["result"])["flag"][0] == 1
    assert so.flag(so.scores(bad, ref), {"rel_l2": 10.0})
    ver.close()


def test_empty_inputs_are_no_ops():
    import torch
    sv, ver = _verifier()
    e = torch.empty((0, 16, 8), dtype=torch.float32, device="cuda")
    r = torch.zeros((16, 8), dtype=torch.float32, device="cuda")
    st = sv.lib.sv_score_and_flag(ver._ctx, e.data_ptr(), 128, 0, r.data_ptr(), 0, 0, 0, 16, 8, 1, None, 1, None, None, None)
    assert st == 0
    st = sv.lib.sv_ema_update(ver._ctx, r.data_ptr(), e.data_ptr(), 128, 0, 0, None, 16, 8, 0.9, None)
    assert st == 0
    st = sv.lib.sv_score_and_flag(ver._ctx, r.data_ptr(), 120, 1, r.data_ptr(), 0, 0, 0, 20, 6, 1, None, 1, None, r.data_ptr(), None)
    assert st != 0                                    # D not a multiple of 8 (and tau NULL) is an error, not a crash
    ver.close()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_ema_update_matches_oracle(dtype):
    import torch
    sv, ver = _verifier()
    T, D, n, beta = 77, 40, 6, 0.9
    g = np.random.default_rng(4)
    m0 = g.standard_normal((T, D)).astype(np.float32)
    claims = [si.to_stage_dtype(g.standard_normal((T, D)).astype(np.float32), dtype) for _ in range(n)]
    cd = dev(np.stack(claims), dtype)
    for flags in ([0, 1, 0, 0, 1, 0], [0] * n, [1] * n, None):
        m = dev(m0, "f32")
        fd = None if flags is None else torch.tensor(flags, dtype=torch.uint8, device="cuda")
        ver.ema_update(m, cd, fd, beta)
        want = so.ema_update(m0, claims, flags if flags is not None else [0] * n, beta)
        np.testing.assert_allclose(host(m), want, rtol=2e-6, atol=2e-7)
        if flags == [1] * n:
            assert np.array_equal(host(m), m0.astype(np.float64))     # nothing clean: bit-identical
    # closed form: constant input from m = 0 gives (1 - beta^t) c
    c = claims[0]
    m = torch.zeros((T, D), dtype=torch.float32, device="cuda")
    one = dev(c[None], dtype)
    for t in range(1, 6):
        ver.ema_update(m, one, None, beta)
        np.testing.assert_allclose(host(m), (1 - beta ** t) * c.astype(np.float64), rtol=1e-5, atol=1e-7)
    ver.close()


def test_score_then_ema_excludes_flagged_claims():
    """Flag bytes produced by the score kernel drive the clean set of the EMA update."""
    import torch
    sv, ver = _verifier()
    T, D = 64, 128
    g = np.random.default_rng(6)
    m0 = si.to_stage_dtype(g.standard_normal((T, D)).astype(np.float32), "bf16")
    kinds = ["honest", "scale", "jit", "zero"]
    claims = [si.to_stage_dtype(m0 * np.float32(1 + 0.002 * i), "bf16") if k in ("honest", "jit") else si.make_claim(k, m0, "bf16", i)
              for i, k in enumerate(kinds)]
    cd = dev(np.stack(claims), "bf16")
    m = dev(m0, "f32")
    out = ver.score_and_flag(cd, m, metrics=("rel_l2", "sfr"), tau={"rel_l2": 0.02, "sfr": 0.1}, reduce="global")
    res = ver.read_results(out["result"])
    assert list(res["flag"]) == [0, 1, 0, 1]
    flags = out["result"].view(torch.int32)[:, 4].to(torch.uint8).contiguous()
    ver.ema_update(m, cd, flags, 0.8)
    want = so.ema_update(m0, claims, [0, 1, 0, 1], 0.8)
    np.testing.assert_allclose(host(m), want, rtol=2e-6, atol=2e-7)
    ver.close()


# The kernel that holds the shared reference's token row in registers serves submissions whose rows are 2, 4 or 8 KB;
# groups of up to 16 submissions share a workgroup, one lane of each wave keeping a submission's running sums.
@pytest.mark.parametrize("cd,rd,D", [("bf16", "bf16", 1024), ("bf16", "f32", 2048), ("bf16", "f32", 4096), ("bf16", "bf16", 4096),
                                     ("f32", "f32", 512), ("f32", "bf16", 1024), ("f32", "f32", 2048),
                                     ("bf16", "f32", 3072), ("f32", "f32", 3584), ("bf16", "bf16", 8192)])   # rows taken in parts
@pytest.mark.parametrize("n,metrics,reduce", [(2, ("rel_l2", "l1", "zl2", "sfr"), "global"), (9, ("rel_l2",), "max_token"),
                                              (37, ("rel_l2", "l1", "zl2", "sfr"), "max_token")])
def test_shared_reference_row_in_registers(cd, rd, D, n, metrics, reduce):
    sv, ver = _verifier()
    T = 45                                         # three 16-token tiles, the last one ragged
    g = np.random.default_rng(D + n)
    base = si.to_stage_dtype((1.3 * g.standard_normal((T, D)) + 0.1).astype(np.float32), rd)
    kinds = ["honest", "scale", "sign", "zero", "noise", "tok_scale", "tok_zero"]
    claims = [si.make_claim(kinds[i % len(kinds)], base.astype(np.float32), cd, seed=7 * i + 1) for i in range(n)]
    out = ver.score_and_flag(dev(np.stack(claims), cd), dev(base, rd), metrics=metrics, tau=TAU, reduce=reduce, want_token_scores=True)
    res = ver.read_results(out["result"])
    _compare(res, host(out["token_scores"]), claims, [base], reduce, metrics)
    ver.close()


@pytest.mark.parametrize("dtype,D", [("f32", 512), ("bf16", 1024)])
def test_sign_flip_ratio_special_values_in_register_kernel(dtype, D):
    """sign(0) = sign(-0) = sign(NaN) = 0 and denormals keep their sign: every pairing of the classes, counted exactly."""
    sv, ver = _verifier()
    tiny = 1e-40                                   # denormal in both float32 and bfloat16
    vals = np.array([0.0, -0.0, tiny, -tiny, 1.0, -2.5, np.inf, -np.inf, np.nan], np.float32)
    T = 18
    g = np.random.default_rng(0)
    ref = vals[g.integers(0, len(vals) - 1, size=(T, D))]          # no NaN in the reference: the other sums stay defined
    claims = np.stack([vals[g.integers(0, len(vals), size=(T, D))] for _ in range(3)] + [ref.copy()])
    ref, claims = si.to_stage_dtype(ref, dtype), si.to_stage_dtype(claims, dtype)
    out = ver.score_and_flag(dev(claims, dtype), dev(ref, dtype), metrics=("sfr",), tau={"sfr": 0.5}, reduce="global")
    res = ver.read_results(out["result"])
    for i in range(4):
        c, r = np.asarray(claims[i], np.float64), np.asarray(ref, np.float64)
        want = np.count_nonzero(so._sgn(c) != so._sgn(r))
        assert round(float(res["score"][i][3]) * T * D) == want, (i, res["score"][i][3] * T * D, want)
    assert res["score"][3][3] == 0.0
    ver.close()


# sv_score_and_sum: the scores of sv_score_and_flag plus the sum over the un-skipped submissions, and
# sv_ema_from_sum, which turns that sum into the EMA update.  Rows are taken in parts of 2 or 4 KB.
@pytest.mark.parametrize("cd,rd,D", [("bf16", "f32", 4096), ("bf16", "bf16", 3072), ("bf16", "f32", 1024), ("f32", "f32", 1024),
                                     ("f32", "bf16", 512), ("f32", "f32", 3584)])
@pytest.mark.parametrize("n,skip", [(1, None), (5, [0, 1, 0, 0, 1]), (16, [0] * 16), (32, [i % 3 == 0 for i in range(32)]), (3, [1, 1, 1])])
def test_score_and_sum_matches_oracle(cd, rd, D, n, skip):
    sv, ver = _verifier()
    T, beta = 37, 0.9
    g = np.random.default_rng(D + n)
    base = si.to_stage_dtype((1.3 * g.standard_normal((T, D)) + 0.1).astype(np.float32), rd)
    kinds = ["honest", "scale", "sign", "zero", "noise", "tok_scale", "tok_zero"]
    claims = [si.make_claim(kinds[i % len(kinds)], base.astype(np.float32), cd, seed=5 * i + 2) for i in range(n)]
    metrics = ("rel_l2", "l1", "zl2", "sfr") if n != 5 else ("rel_l2",)
    out = ver.score_and_sum(dev(np.stack(claims), cd), dev(base, rd), skip=skip, metrics=metrics, tau=TAU, reduce="global",
                            want_token_scores=True)
    res = ver.read_results(out["result"])
    _compare(res, host(out["token_scores"]), claims, [base], "global", metrics)
    keep = [c for i, c in enumerate(claims) if skip is None or not skip[i]]
    want = np.sum([np.asarray(c, np.float64) for c in keep], axis=0) if keep else np.zeros((T, D))
    mag = np.sum([np.abs(np.asarray(c, np.float64)) for c in keep], axis=0) if keep else np.zeros((T, D))
    assert np.all(np.abs(host(out["sum"]) - want) <= 2e-7 * mag * max(len(keep), 1) + 1e-30)
    # the EMA update from the sum against the definition over the same clean set
    m0 = g.standard_normal((T, D)).astype(np.float32)
    m = dev(m0, "f32")
    ver.ema_from_sum(m, out["sum"], len(keep), beta)
    flags = [0] * n if skip is None else [int(bool(x)) for x in skip]
    np.testing.assert_allclose(host(m), so.ema_update(m0, claims, flags, beta), rtol=2e-6, atol=2e-6)
    if not keep:
        assert np.array_equal(host(m), m0.astype(np.float64))
    ver.close()


def test_score_and_sum_limits():
    import torch
    sv, ver = _verifier()
    T, D = 16, 1024
    c = torch.zeros((33, T, D), dtype=torch.bfloat16, device="cuda")
    r = torch.zeros((T, D), dtype=torch.float32, device="cuda")
    with pytest.raises(sv.SVError):                              # more than 32 submissions
        ver.score_and_sum(c, r)
    with pytest.raises(sv.SVError):                              # a row of 1.5 KB
        ver.score_and_sum(torch.zeros((2, T, 768), dtype=torch.bfloat16, device="cuda"), torch.zeros((T, 768), dtype=torch.float32, device="cuda"))
    ver.score_and_sum(c[:32], r)                                 # the limit itself
    ver.close()
