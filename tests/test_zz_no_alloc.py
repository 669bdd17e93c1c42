"""sv_score_and_flag_noalloc -- the statistic for callers that cannot allocate -- against sv_score_and_flag on the same
inputs: same kernels, so the results (scores, flags, arg-max tokens, per-token scores) must be identical bit for bit.
Two calls in a row share the one static scratch of the GPU; the second is smaller, so records of the first stay behind
it and must not leak into its result.  Also checked against the CPU oracle, and the size limit."""
import ctypes

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import stage_inputs as si
from oracle import stage_oracle as so
from gpu_util import dev

TAU = {"rel_l2": 2e-2, "l1": 0.05, "zl2": 0.01, "sfr": 0.02}
KINDS = ["honest", "scale", "sign", "zero", "noise", "tok_scale", "tok_zero", "honest", "tok_neg"]


def _case(n, T, D, dtype, seed, shared):
    g = np.random.default_rng(seed)
    refs = [si.to_stage_dtype((1.2 * g.standard_normal((T, D)) + 0.05).astype(np.float32), dtype) for _ in range(1 if shared else n)]
    claims = [si.make_claim(KINDS[i % len(KINDS)], refs[0 if shared else i], dtype, seed + i) for i in range(n)]
    return claims, refs


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("shared", [True, False], ids=["shared_ref", "own_refs"])
def test_noalloc_entry_point_equals_the_context_one_on_two_calls_in_a_row(dtype, shared):
    import torch
    import paper_2603_03592_amd as sv
    ver = sv.Verifier(si.TINY.desc, 128, 64)
    metrics = ("rel_l2", "l1", "zl2", "sfr")
    # first call: 9 submissions of 1000 tokens x 1024 features (rows of 2 / 4 KB: the shared-reference kernel);
    # second call: smaller in both directions, ragged token count, 3 submissions
    for n, T, D in ((9, 1000, 1024), (3, 77, 1024)):
        claims, refs = _case(n, T, D, dtype, seed=5 + n, shared=shared)
        cl = dev(np.stack(claims), dtype)
        rf = dev(refs[0] if shared else np.stack(refs), dtype)
        want = ver.score_and_flag(cl, rf, metrics=metrics, tau=TAU, want_token_scores=True)
        res = torch.full((n, 32), 0xAB, dtype=torch.uint8, device="cuda")
        tok = torch.full((n, T), -7.0, dtype=torch.float32, device="cuda")
        got = sv.score_and_flag_noalloc(cl, rf, res, metrics=metrics, tau=TAU, token_scores=tok)
        torch.cuda.synchronize()
        assert torch.equal(got, want["result"]), (n, T)                       # every byte of every sv_result
        assert torch.equal(tok, want["token_scores"]), (n, T)
        # ... and both are right: against the oracle, outside the +-5 % band around a threshold
        r = ver.read_results(got)
        for i in range(n):
            w = so.scores(claims[i], refs[0 if shared else i])
            for j, m in enumerate(so.METRICS):
                tol = dict(rel=1e-4, abs=5e-6) if m == "zl2" else dict(rel=3e-5, abs=2e-7)
                assert float(r["score"][i][j]) == pytest.approx(w[m], **tol), (i, m)
            if min(abs(w[m] / TAU[m] - 1.0) for m in TAU) > 0.05:
                assert bool(r["flag"][i]) == so.flag(w, TAU), i
    ver.close()


def test_noalloc_entry_point_rejects_sizes_beyond_its_scratch():
    import torch
    import paper_2603_03592_amd as sv
    x = torch.zeros((8, 64), dtype=torch.float32, device="cuda")
    res = torch.zeros((1, 32), dtype=torch.uint8, device="cuda")
    tau = (ctypes.c_float * 4)(1, 1, 1, 1)
    # 65 537 submissions of one tile each: one record too many.  The host check fires before any pointer is used.
    st = sv.lib.sv_score_and_flag_noalloc(x.data_ptr(), 0, 65537, x.data_ptr(), 0, 0, 0, 8, 64, 1, tau, 1, None, res.data_ptr(), None)
    assert st == 2 and b"65536" in sv.lib.sv_last_error(None)
    st = sv.lib.sv_score_and_flag_noalloc(x.data_ptr(), 0, 1, x.data_ptr(), 0, 0, 0, 16 * 65536 + 1, 64, 1, tau, 1, None, res.data_ptr(), None)
    assert st == 2
    assert sv.lib.sv_score_and_flag_noalloc(x.data_ptr(), 0, 1, x.data_ptr(), 0, 0, 0, 8, 60, 1, tau, 1, None, res.data_ptr(), None) == 2   # D % 8
    assert sv.lib.sv_score_and_flag_noalloc(None, 0, 1, x.data_ptr(), 0, 0, 0, 8, 64, 1, tau, 1, None, res.data_ptr(), None) == 1
    assert sv.lib.sv_score_and_flag_noalloc(x.data_ptr(), 0, 0, x.data_ptr(), 0, 0, 0, 8, 64, 1, tau, 1, None, res.data_ptr(), None) == 0  # nothing to do
    # a call at exactly the limit of one dimension runs: 1 submission of 16 tokens -> 1 record
    y = torch.randn((16, 64), dtype=torch.float32, device="cuda")
    sv.score_and_flag_noalloc(y[None], y, res, tau={"rel_l2": 1e-3})
    torch.cuda.synchronize()
    assert int(sv.Verifier.read_results(res)["flag"][0]) == 0
