"""GPU parity: the library's verifier loop (sv_sentinel_*) against the oracle's SentinelStream on the same
synthetic stream -- 3 stages x 6 workers, warm-up, an activation attack that would cascade, a gradient attack,
a severe deviation.  Decisions (who is tainted where, counters, bans) must agree exactly; the statistics, the
EMAs and the fences agree to float32 accuracy; replaced gradients equal the EMA of before the call."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import stage_inputs as si
from oracle import sentinel_oracle as sn
from gpu_util import dev, host
from test_oracle_sentinel import D, DW, P, POLICY, T, WARM, _signals

METRICS = ("rel_l2", "l1", "zl2", "sfr", "sw")


def _pair(dtype, Dv=D):
    import torch
    import paper_2603_03592_amd as sv
    u = si.make_directions(Dv, 32, 0)
    ver = sv.Verifier(si.TINY.desc, T, 64, sliced_w=True)
    lib = sv.Sentinel(ver, P, DW, T, Dv, METRICS, dev(u, "bf16"), 0.9, 0.8, POLICY, POLICY)
    ref = sn.SentinelStream(P, DW, (T, Dv), METRICS, u, 0.9, 0.8, POLICY, POLICY)
    return torch, ver, lib, ref


def _sig(kind, s, t, attack, Dv):
    """_signals of the oracle's own test at another feature width."""
    if Dv == D:
        return _signals(kind, s, t, attack)
    out = [si.stream_signal(kind, s, r, t, T, Dv, "f32") for r in range(DW)]
    if attack is not None:
        a_s, a_r, a_kind = attack
        if s == a_s:
            out[a_r] = si.make_claim(a_kind, out[a_r], "f32", seed=t)
        elif kind == "h" and s > a_s:
            out[a_r] = si.make_claim("noise", out[a_r] * 1.2, "f32", seed=t)
    return out


def _gamma_close(got, want):
    # columns: rel_l2, l1, zl2, sfr, sw; fp32 sums on the device, EMAs kept in fp32
    np.testing.assert_allclose(got, want, rtol=2e-4, atol=1e-7)


def _iteration(torch, lib, ref, t, warm, dtype, attack_h=None, attack_g=None, Dv=D):
    lib.begin_iteration(warm); ref.begin_iteration(warm)
    for s in range(P):
        sig = [si.to_stage_dtype(x, dtype) for x in _sig("h", s, t, attack_h, Dv)]
        want, wg = ref.forward(s, sig)
        got, gg = lib.forward(s, torch.stack([dev(x, dtype) for x in sig]))
        assert got == want, (t, "h", s, got, want)
        _gamma_close(gg, wg)
    for s in reversed(range(P)):
        sig = [si.to_stage_dtype(x, dtype) for x in _sig("g", s, t, attack_g, Dv)]
        m_before = lib.ema(s, "g")
        want, wg, wout = ref.backward(s, sig)
        g_dev = torch.stack([dev(x, dtype) for x in sig])
        got, gg = lib.backward(s, g_dev)
        assert got == want, (t, "g", s, got, want)
        _gamma_close(gg, wg)
        out = host(g_dev)
        for r in range(DW):
            if wout[r] is sig[r]:
                assert np.array_equal(out[r], np.float64(sig[r])), (t, s, r)             # untouched
            else:
                assert np.array_equal(out[r], np.float64(si.to_stage_dtype(m_before, dtype))), (t, s, r)
                np.testing.assert_allclose(out[r], wout[r], rtol=1e-2 if dtype == "bf16" else 1e-5, atol=1e-6)


def _state_close(lib, ref):
    for kind in "hg":
        for s in range(P):
            st, pol = lib.state(s, kind), ref.pol[kind][s]
            assert list(st["violations"]) == pol.v and list(st["banned"]) == pol.banned, (kind, s)
            np.testing.assert_allclose(st["lower"], pol.lower, rtol=1e-3)
            np.testing.assert_allclose(st["upper"], pol.upper, rtol=1e-3)
            m = lib.ema(s, kind).astype(np.float64)
            assert np.linalg.norm(m - ref.m[kind][s]) <= 2e-6 * np.linalg.norm(ref.m[kind][s]), (kind, s)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_verifier_loop_matches_oracle(dtype):
    torch, ver, lib, ref = _pair(dtype)
    for t in range(WARM):
        _iteration(torch, lib, ref, t, True, dtype)
    _state_close(lib, ref)
    t = WARM
    for _ in range(2):                                   # honest iterations
        _iteration(torch, lib, ref, t, False, dtype); t += 1
    for _ in range(6):                                   # activation sign attack at stage 1, pipe 2: caught, banned after 5
        _iteration(torch, lib, ref, t, False, dtype, attack_h=(1, 2, "sign")); t += 1
    assert ref.pol["h"][1].banned[2] and lib.state(1, "h")["banned"][2]
    _iteration(torch, lib, ref, t, False, dtype, attack_g=(1, 4, "scale")); t += 1
    _iteration(torch, lib, ref, t, False, dtype, attack_g=(2, 0, "zero")); t += 1
    _iteration(torch, lib, ref, t, False, dtype, attack_h=(0, 5, "zero"), attack_g=(0, 1, "sign")); t += 1
    _state_close(lib, ref)
    assert sum(ref.pol["g"][1].v) > 0 and sum(ref.pol["h"][0].v) > 0
    lib.close(); ver.close()


@pytest.mark.parametrize("dtype,Dv", [("bf16", 1024), ("f32", 512)])
def test_verifier_loop_with_the_sum_from_the_score_pass(dtype, Dv):
    """Rows of 2 KB: the loop takes the statistics and the sum over the signals in one pass (sv_score_and_sum) and
    finishes the EMA from that sum whenever the verdicts exclude nobody beyond the workers known beforehand; an
    iteration with a new flag falls back to the update that reads the signals.  Same stream, same decisions, same EMAs."""
    torch, ver, lib, ref = _pair(dtype, Dv)
    import paper_2603_03592_amd as sv
    x = torch.zeros((DW, T, Dv), dtype=torch.bfloat16 if dtype == "bf16" else torch.float32, device="cuda")
    ver.score_and_sum(x, torch.zeros((T, Dv), dtype=torch.float32, device="cuda"))       # the shape is one the summing pass takes
    for t in range(WARM):
        _iteration(torch, lib, ref, t, True, dtype, Dv=Dv)
    _state_close(lib, ref)
    t = WARM
    for _ in range(2):                                   # honest: the sum covers everybody
        _iteration(torch, lib, ref, t, False, dtype, Dv=Dv); t += 1
    for _ in range(6):                                   # new flags (fallback), then a banned worker skipped beforehand
        _iteration(torch, lib, ref, t, False, dtype, attack_h=(1, 2, "sign"), Dv=Dv); t += 1
    assert ref.pol["h"][1].banned[2] and lib.state(1, "h")["banned"][2]
    for _ in range(2):                                   # the ban stands: sums without that worker
        _iteration(torch, lib, ref, t, False, dtype, Dv=Dv); t += 1
    _iteration(torch, lib, ref, t, False, dtype, attack_g=(1, 4, "scale"), Dv=Dv); t += 1
    _iteration(torch, lib, ref, t, False, dtype, attack_h=(0, 5, "zero"), attack_g=(0, 1, "sign"), Dv=Dv); t += 1
    _state_close(lib, ref)
    c = lib.counters()                                    # both ways of updating the EMA were taken, every SW check carried
    assert c["calls"] == 2 * P * t and c["ema_from_sum"] + c["ema_from_signals"] == c["calls"]
    assert c["ema_from_signals"] >= 7 and c["ema_from_sum"] > c["calls"] // 2 and c["sw_carried"] == c["calls"]
    lib.close(); ver.close()


def test_verifier_loop_value_replacing_and_delay_attacks():
    """The paper's remaining attack variants through both implementations: constant, random value, element-wise random
    sign and invisible noise are caught where they happen; a delayed honest signal passes."""
    dtype = "bf16"
    torch, ver, lib, ref = _pair(dtype)
    for t in range(WARM):
        _iteration(torch, lib, ref, t, True, dtype)
    t = WARM
    for w, kind in enumerate(("const_neg1", "random", "sign_p", "invisible")):
        _iteration(torch, lib, ref, t, False, dtype, attack_h=(0, w, kind), attack_g=(2, w + 1, kind)); t += 1
        assert ref.pol["h"][0].v[w] >= 1 and ref.pol["g"][2].v[w + 1] >= 1, kind
    # delay attack, k = 20: worker 5 of stage 1 re-sends what it sent 20 iterations ago
    lib.begin_iteration(False); ref.begin_iteration(False)
    for s in range(P):
        sig = [si.to_stage_dtype(x, dtype) for x in _signals("h", s, t)]
        if s == 1:
            sig[5] = si.to_stage_dtype(si.stream_signal("h", 1, 5, t - 20, T, D, "f32"), dtype)
        want, wg = ref.forward(s, sig)
        got, gg = lib.forward(s, torch.stack([dev(x, dtype) for x in sig]))
        assert got == want == [], (s, got, want)
        _gamma_close(gg, wg)
    _state_close(lib, ref)
    lib.close(); ver.close()


def test_replace_with_ema_entry_point():
    import torch
    import paper_2603_03592_amd as sv
    ver = sv.Verifier(si.TINY.desc, 128, 64)
    g = np.random.default_rng(0)
    for dtype in ("bf16", "f32"):
        sig = [si.to_stage_dtype(g.standard_normal((50, 72)).astype(np.float32), dtype) for _ in range(5)]
        m = g.standard_normal((50, 72)).astype(np.float32)
        x = torch.stack([dev(s_, dtype) for s_ in sig])
        mask = torch.tensor([0, 1, 0, 0, 1], dtype=torch.uint8, device="cuda")
        ver.replace_with_ema(x, mask, torch.from_numpy(m).cuda())
        out = host(x)
        for i in range(5):
            want = si.to_stage_dtype(m, dtype) if i in (1, 4) else sig[i]
            assert np.array_equal(out[i], np.float64(want)), (dtype, i)
    ver.close()
