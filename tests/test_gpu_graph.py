"""The check entry points enqueue kernels only (no allocation, no host wait, no memset), so a caller can capture them
into a HIP graph once and replay the graph for every micro-batch of the same shape; that takes the launch latency
out of small, launch-bound checks.  Each test captures after an eager warm-up (kernel attributes are set on a
kernel's first launch), replays several times with eager work and synchronisations in between, and compares every
replay bit for bit with the eager result on the same inputs."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import stage_inputs as si
from gpu_util import dev, dev_weights

CASES = {
    "tiny_f32": (si.TINY.desc, 2, 64, False),
    "mfma_bf16_bwd": (si.StageDesc(2, 256, 4, 2, 384), 2, 160, True),
    "moe_bf16_bwd": (si.StageDesc(1, 256, 4, 2, 256, n_experts=8, top_k=2, n_shared=1, router_norm=True), 2, 200, True),
}


@pytest.mark.parametrize("name", list(CASES))
def test_captured_check_replays_bit_exactly(name):
    import torch
    import paper_2603_03592_amd as sv
    desc, B, S, backward = CASES[name]
    w = si.make_weights(desc, 4)
    ver = sv.Verifier(desc, B * S, S, backward=backward, sliced_w=True)
    wc = ver.pack_weights(wd := dev_weights(w, desc.dtype))
    h = dev(si.make_activations(desc, B, S, 4), desc.dtype)
    g = dev(si.make_output_grad(desc, B, S, 4, std=1.0), desc.dtype)
    dirs = dev(si.make_directions(desc.d_model, 32, seed=1), "bf16")

    def check(hh, gg):
        if backward:
            first = ver.verify_backward(wc, hh, gg, want_g_hat=True, want_h_hat=True)
            sig = first["g_hat"]
        else:
            first = ver.verify_forward(wc, hh, want_h_hat=True)
            sig = first["h_hat"]
        # score the recomputation against a shifted copy of itself with every statistic, then update an EMA from it
        claim = (sig.float() * 1.25).to(sig.dtype)
        r = ver.score_and_flag(claim.reshape(1, B * S, -1), sig.reshape(B * S, -1), metrics=("rel_l2", "l1", "zl2", "sfr"),
                               tau=(0.1, 1e9, 1e9, 1e9), reduce="global")
        sw = ver.sliced_wasserstein(claim.reshape(1, B * S, -1), sig.reshape(B * S, -1), dirs, tau=1e9, results=r["result"])
        return sig, r["result"], sw

    eager = [t.clone() for t in check(h, g)]              # warm-up: also sets the kernels' attributes
    torch.cuda.synchronize()
    hs, gs = h.clone(), g.clone()                          # static inputs of the graph
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    with torch.cuda.graph(graph, stream=side):
        outs = check(hs, gs)
    torch.cuda.synchronize()
    for rep in range(4):
        if rep == 2:                                       # other inputs through the same graph, then back
            hs.copy_(h.flip(0)); gs.copy_(g.flip(0))
            graph.replay()
            torch.cuda.synchronize()
            other = [t.clone() for t in check(h.flip(0).contiguous(), g.flip(0).contiguous())]
            for a, b in zip(outs, other):
                assert torch.equal(a, b)
            hs.copy_(h); gs.copy_(g)
        graph.replay()
        torch.cuda.synchronize()
        for a, b in zip(outs, eager):
            assert torch.equal(a, b), (name, rep)
        _ = (h.float() @ h.float().transpose(-1, -2)).sum().item()   # unrelated eager work between replays
    res = ver.read_results(outs[1])
    assert int(res["flag"][0]) == 1 and abs(float(res["score"][0][0]) - 0.25) < 2e-2
    del graph
    ver.close()
