#!/usr/bin/env python3
"""Benchmark of the stage-verifier hot path on one MI355X.

One step = one stage check of one micro-batch through the C ABI: recompute the stage on the
worker's input (all blocks), then score the claimed output (and, for fwd+bwd workloads, the
claimed input gradient) and flag it.  Inputs, weights and claims are synthetic, generated on
the device before the timed region (shapes of the benchmark configs; claims are the device
recomputation with 1 % of tokens corrupted, so the flag path does real work).

Prints ONE JSON line with the verified tokens/s, the MFMA roofline of the dominant kernel (the
gate/up projection GEMM, timed with HIP events on the launch stream during the timed steps)
and the CPU oracle timed on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA peak
PEAK_HBM_GBS = 8000.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="large", help="tiny|small|medium|large|moe_top1|moe_top6|sweep_s<S>_b<B>")
    ap.add_argument("--graph", action="store_true", help="also time the step replayed from a captured HIP graph")
    ap.add_argument("--mode", default=None, choices=[None, "fwd", "fwdbwd"], help="default: the workload's own")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--plain", action="store_true", help="run the plain (non-MFMA) kernels")
    ap.add_argument("--fuse-norm", default="auto", choices=["auto", "on", "off"],
                    help="run the two RMSNorms of a block inside the neighbouring products (SV_FLAG_FUSE_NORM); auto: where it "
                         "measured faster (paper_2603_03592_amd.fuse_norm_pays)")
    ap.add_argument("--score-bench", action="store_true",
                    help="instead of the stage check, time the stand-alone scoring pass (128 submissions against one shared "
                         "reference) and the EMA update, and report them against the HBM roofline")
    ap.add_argument("--loop-bench", action="store_true",
                    help="instead of the recompute check, time the paper's own verifier loop (statistics against the EMA, policy, "
                         "gradient replacement, EMA update) for 4 stages x 16 workers of the large stage's signal shape")
    ap.add_argument("--gemm-bench", action="store_true",
                    help="instead of the stage check, time the plain bf16 product on the large stage's four GEMM shapes: this "
                         "library's kernel (sv_gemm_bf16) and, as a diagnostic yardstick only, the vendor BLAS behind torch.matmul")
    ap.add_argument("--sweep", action="store_true",
                    help="run the throughput sweep (single block, d_model 4096, seq x micro-batch grid, fwd+bwd) and print one "
                         "JSON line per point")
    ap.add_argument("--no-extra", action="store_true",
                    help="default run only: skip the further legs (forward + backward on the medium stage and on the large shape, "
                         "the 128-submission score pass against the HBM roofline)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run three 1 GiB device copies (a kernel of known traffic, to scale rocprofv3's FETCH_SIZE / WRITE_SIZE)")
    return ap.parse_args()


def get_workload(name):
    import stage_inputs as si
    if name in si.WORKLOADS:
        return si.WORKLOADS[name]
    if name.startswith("sweep_s"):
        s, b = name[len("sweep_s"):].split("_b")
        return si.sweep_point(int(s), int(b))
    raise SystemExit(f"unknown workload {name}")


def device_weights(desc, torch):
    """Random-init weights of the stage's shapes, generated on the device (N(0, 0.02^2) matrices)."""
    dt = torch.bfloat16 if desc.dtype == "bf16" else torch.float32
    g = torch.Generator(device="cuda").manual_seed(0)
    D, hd = desc.d_model, desc.head_dim
    Hq, Hkv, F = desc.n_heads * hd, desc.n_kv_heads * hd, desc.ffn_hidden

    def mat(o, i):
        return (0.02 * torch.randn((o, i), generator=g, device="cuda", dtype=torch.float32)).to(dt)

    def vec(mean, std):
        return (mean + std * torch.randn(D, generator=g, device="cuda", dtype=torch.float32)).to(dt)

    blocks = []
    E, Fs = desc.n_experts, desc.n_shared * F
    for _ in range(desc.n_blocks):
        w = dict(wq=mat(Hq, D), wk=mat(Hkv, D), wv=mat(Hkv, D), wo=mat(D, Hq), norm1_g=vec(1.0, 0.1), norm2_g=vec(1.0, 0.1),
                 norm1_b=vec(0.0, 0.02) if desc.norm == "ln" else None, norm2_b=vec(0.0, 0.02) if desc.norm == "ln" else None)
        if E > 0:      # routed experts one after the other, shared experts side by side
            w.update(w_gate=mat(E * F, D).view(E, F, D), w_up=mat(E * F, D).view(E, F, D), w_down=mat(E * D, F).view(E, D, F),
                     w_router=mat(E, D))
            if Fs:
                w.update(ws_gate=mat(Fs, D), ws_up=mat(Fs, D), ws_down=mat(D, Fs))
        else:
            w.update(w_up=mat(F, D), w_down=mat(D, F), w_gate=mat(F, D) if desc.mlp == "swiglu" else None)
        blocks.append(w)
    return blocks


def corrupt_tokens(x, torch, frac=0.01):
    """Claim manufactured on the device: the recomputation with `frac` of the tokens scaled by 1.5."""
    c = x.clone()
    flat = c.view(-1, c.shape[-1])
    n = max(1, int(frac * flat.shape[0]))
    idx = torch.randperm(flat.shape[0], device=x.device, generator=torch.Generator(device="cuda").manual_seed(1))[:n]
    flat[idx] = (flat[idx].float() * 1.5).to(c.dtype)
    return c


def cpu_baseline(wl, wdev, h_in, g_out, backward):
    """The oracle as it stands, on one sequence of the micro-batch (stage work is independent per sequence)."""
    import numpy as np
    from oracle import stage_oracle as so
    w = [{k: (None if v is None else v.float().cpu().numpy()) for k, v in b.items()} for b in wdev]
    h = h_in[:1].float().cpu().numpy()
    t0 = time.perf_counter()
    if backward:
        so.stage_backward(h, g_out[:1].float().cpu().numpy(), w, wl.desc)
    else:
        so.stage_forward(h, w, wl.desc)
    dt = time.perf_counter() - t0
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [os.cpu_count()])
    except Exception:
        cores = os.cpu_count()
    return {"value": wl.seq / dt, "unit": "verified tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"1 of {wl.batch} sequences ({wl.seq} tokens) through all {wl.desc.n_blocks} blocks, "
                      f"{'fwd+bwd' if backward else 'fwd'}, numpy float64, {dt:.1f} s"}


def measured_traffic(workload, kernel):
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3 --pmc summary (FETCH_SIZE and
    WRITE_SIZE runs scaled by a copy of known size), or None when no summary covers this workload/kernel.
    `workload` carries the suffix _fwdbwd when a forward-only configuration is run forward + backward."""
    path = os.path.join(ROOT, "profiles", f"{workload}_{kernel}_hbm_traffic.txt")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":")[1])
    except OSError:
        pass
    return None


def score_traffic():
    """HBM bytes per launch of the score pass in the 128-submission bench, from the committed rocprofv3 --pmc summary."""
    try:
        for line in open(os.path.join(ROOT, "profiles", "score_bench_hbm_traffic.txt")):
            if line.startswith("score_traffic_bytes_per_launch:"):
                return float(line.split(":")[1])
    except OSError:
        pass
    return None


def score_bench(a):
    """HBM-bound half of the verifier: Gamma = Omega(h, reference) for 128 concurrent submissions of the large
    stage's signal shape [8192, 4096] bf16 against one shared reference (the paper's EMA mode, or one
    recomputation shared by many workers), then the EMA update over the un-flagged ones."""
    import torch
    import paper_2603_03592_amd as sv
    import stage_inputs as si
    T, D, n = 8192, 4096, 128
    torch.cuda.set_device(0)
    ver = sv.Verifier(si.TINY.desc, T, 64, sliced_w=True)
    g = torch.Generator(device="cuda").manual_seed(0)
    ref = torch.randn((T, D), generator=g, device="cuda", dtype=torch.float32)
    claims = torch.empty((n, T, D), dtype=torch.bfloat16, device="cuda")
    for i in range(n):
        claims[i] = (ref * (1.5 if i % 8 == 3 else 1.0)).to(torch.bfloat16)
    m = ref.clone()
    refb = ref.to(torch.bfloat16)
    tau = {"rel_l2": 2e-2, "l1": 0.05, "zl2": 0.01, "sfr": 0.02}

    def timed(fn, steps):
        for _ in range(2):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(steps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / steps

    out = {}
    ms = timed(lambda: out.update(r=ver.score_and_flag(claims, refb, metrics=("rel_l2", "l1", "zl2", "sfr"), tau=tau)), a.steps)
    flags = ver.read_results(out["r"]["result"])["flag"]
    assert [int(f) for f in flags] == [int(i % 8 == 3) for i in range(n)]
    score_bytes = n * T * D * 2 + T * D * 2 + n * T * 4            # claims + the shared reference once (+ nothing else of size)
    ms_lite = timed(lambda: ver.score_and_flag(claims, refb, metrics=("rel_l2",), tau=tau), a.steps)
    fl = out["r"]["result"].view(torch.int32)[:, 4].to(torch.uint8).contiguous()
    ms_ema = timed(lambda: ver.ema_update(m, claims, fl, 0.9), a.steps)
    n_clean = int((fl == 0).sum())
    ema_bytes = n_clean * T * D * 2 + 2 * T * D * 4
    # sliced Wasserstein statistic: 64 directions, the same 128 submissions against the shared reference
    n_dirs = 64
    dirs = torch.from_numpy(si.make_directions(D, n_dirs, 0)).cuda().to(torch.bfloat16)
    sw_out = {}
    ms_sw = timed(lambda: sw_out.update(v=ver.sliced_wasserstein(claims, refb, dirs, 1e-2)), max(2, a.steps // 4))
    swv = sw_out["v"].float().cpu().numpy()
    assert all((swv[i] > 1e-2) == (i % 8 == 3) for i in range(n)), swv[:8]
    ver.profile_enable(True)
    ver.sliced_wasserstein(claims, refb, dirs, 1e-2)
    prof = ver.profile_read()
    ver.profile_enable(False)
    sw_bytes = (n + 1) * T * D * 2
    res = {
        "metric": "scored tokens/sec (stand-alone statistic, 128 submissions, shared reference)", "value": n * T / (ms * 1e-3),
        "unit": "tokens/s", "n_gpus": 1, "steps": a.steps, "warmup": 2, "ms_per_step": ms, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "score_128x8192x4096", "claims": n, "tokens": T, "d_model": D, "metrics": "rel_l2,l1,zl2,sfr"},
        "roofline": {"bound": "hbm", "kernel": "score_parts_kernel", "achieved": score_bytes / (ms * 1e-3) / 1e9, "peak": PEAK_HBM_GBS,
                     "unit": "GB/s", "frac": score_bytes / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS, "traffic": score_traffic()},
        "rel_l2_only": {"ms": ms_lite, "achieved_GBs": score_bytes / (ms_lite * 1e-3) / 1e9,
                        "frac": score_bytes / (ms_lite * 1e-3) / 1e9 / PEAK_HBM_GBS},
        "sliced_wasserstein": {"ms": ms_sw, "directions": n_dirs, "achieved_GBs": sw_bytes / (ms_sw * 1e-3) / 1e9,
                               "frac": sw_bytes / (ms_sw * 1e-3) / 1e9 / PEAK_HBM_GBS,
                               "project_ms": prof["sw_project"]["ms"], "sort_ms": prof["sw_sort"]["ms"],
                               "project_GBs": sw_bytes / (prof["sw_project"]["ms"] * 1e-3) / 1e9},
        "ema": {"ms": ms_ema, "clean": n_clean, "achieved_GBs": ema_bytes / (ms_ema * 1e-3) / 1e9,
                "frac": ema_bytes / (ms_ema * 1e-3) / 1e9 / PEAK_HBM_GBS},
    }
    ver.close()
    print(json.dumps(res))


def gemm_bench(a):
    """C = A B^T in bf16 (fp32 accumulation) on the four product shapes of the large stage, 8192 tokens: this library's
    256 x 256 direct-to-LDS kernel without any fused epilogue, and beside it the vendor BLAS that torch.matmul calls.
    The vendor figure is a diagnostic of what the chip sustains on these shapes under its power management (it is given
    the same operands right after ours); no product path of the library calls it."""
    import torch
    import paper_2603_03592_amd as sv
    torch.cuda.set_device(0)
    shapes = [("qkv", 8192, 6144, 4096), ("out", 8192, 4096, 4096), ("gate_or_up", 8192, 14336, 4096), ("down", 8192, 4096, 14336)]
    g = torch.Generator(device="cuda").manual_seed(0)
    rows = []
    for name, M, N, K in shapes:
        x = torch.randn((M, K), generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
        w = (0.02 * torch.randn((N, K), generator=g, device="cuda", dtype=torch.float32)).to(torch.bfloat16)
        out = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
        wt = w.t()

        def timed(fn):
            for _ in range(a.warmup):
                fn()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(a.steps):
                fn()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / a.steps

        ms_own = timed(lambda: sv.sv_gemm_bf16(x, w, tile=1, out=out))
        ref = torch.matmul(x, wt)
        err = float((out.float() - ref.float()).norm() / ref.float().norm())
        assert err < 1e-2, err
        ms_lib = timed(lambda: torch.matmul(x, wt, out=ref))
        fl = 2.0 * M * N * K
        rows.append({"product": name, "M": M, "N": N, "K": K, "own_ms": ms_own, "own_tflops": fl / ms_own / 1e9,
                     "own_frac": fl / ms_own / 1e9 / PEAK_BF16_TFLOPS, "vendor_ms": ms_lib, "vendor_tflops": fl / ms_lib / 1e9,
                     "vendor_frac": fl / ms_lib / 1e9 / PEAK_BF16_TFLOPS, "rel_diff": err})
    tot = sum(2.0 * r["M"] * r["N"] * r["K"] for r in rows)
    own = sum(r["own_ms"] for r in rows)
    print(json.dumps({
        "metric": "bf16 GEMM TFLOP/s on the large stage's product shapes (plain product, no fused epilogue)", "value": tot / own / 1e9,
        "unit": "TFLOP/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": own, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic", "config": {"workload": "gemm_large_shapes"},
        "roofline": {"bound": "mfma", "kernel": "gemm_mfma_dma_kernel", "achieved": tot / own / 1e9, "peak": PEAK_BF16_TFLOPS,
                     "unit": "TFLOP/s", "frac": tot / own / 1e9 / PEAK_BF16_TFLOPS, "traffic": None},
        "products": rows}))


def loop_bench(a):
    """The paper's verifier loop (EMA reference instead of recomputation): 4 stages x 16 workers, signals [8192, 4096] bf16,
    all five statistics (64 directions for the sliced Wasserstein distance).  A step is one iteration: forward over the
    stages, then backward; the signals are resident in HBM (one set per stage and kind, reused every iteration)."""
    import torch
    import paper_2603_03592_amd as sv
    import stage_inputs as si
    P_, d, T, D = 4, 16, 8192, 4096
    torch.cuda.set_device(0)
    ver = sv.Verifier(si.TINY.desc, T, 64, sliced_w=True)
    dirs = torch.from_numpy(si.make_directions(D, 64, 0)).cuda().to(torch.bfloat16)
    pol = dict(c=5, t_forgive=100, window=100, k0=1.5, alpha=0.01, grow=1.1, shrink=0.9, n_max=10, min_dist_mult=0.35, eps=1e-4)
    loop = sv.Sentinel(ver, P_, d, T, D, ("rel_l2", "l1", "zl2", "sfr", "sw"), dirs, 0.9, 0.8, pol, pol)
    g = torch.Generator(device="cuda").manual_seed(0)
    sig = {}
    for kind, scale in (("h", 1.0), ("g", 1e-3)):
        for s_ in range(P_):
            base = torch.randn((T, D), generator=g, device="cuda", dtype=torch.float32)
            x = torch.empty((d, T, D), dtype=torch.bfloat16, device="cuda")
            for r in range(d):
                x[r] = (scale * (base + 0.5 * torch.randn((T, D), generator=g, device="cuda", dtype=torch.float32))).to(torch.bfloat16)
            sig[kind, s_] = x

    def iteration(warm):
        loop.begin_iteration(warm)
        flagged = 0
        for s_ in range(P_):
            flagged += len(loop.forward(s_, sig["h", s_])[0])
        for s_ in reversed(range(P_)):
            flagged += len(loop.backward(s_, sig["g", s_])[0])
        return flagged

    for _ in range(max(a.warmup, 12)):
        iteration(True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    flagged = 0
    for _ in range(a.steps):
        flagged += iteration(False)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / a.steps
    signals = 2 * P_ * d
    # bytes one iteration moves by design: every signal is read by the score pass and by the projection; per stage call
    # the EMA is read by the score pass, the sum over the signals is written and read back, and the EMA is read and written
    alg = signals * T * D * 2 * 2 + 2 * P_ * T * D * 4 * 5
    print(json.dumps({
        "metric": "verified tokens/sec (EMA-reference verifier loop, 4 stages x 16 workers, fwd+bwd signals)",
        "value": signals * T / (ms * 1e-3), "unit": "tokens/s", "n_gpus": 1, "steps": a.steps, "warmup": max(a.warmup, 12),
        "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "loop_4x16x8192x4096", "stages": P_, "workers": d, "tokens": T, "d_model": D,
                   "metrics": "rel_l2,l1,zl2,sfr,sw(64)", "flagged_in_timed_steps": flagged},
        "roofline": {"bound": "hbm", "kernel": "whole iteration (score+sum, projection/sort, EMA from the sum)", "achieved": alg / (ms * 1e-3) / 1e9,
                     "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": alg / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS, "traffic": None}}))
    loop.close(); ver.close()


def main():
    a = parse()
    if a.gpus != 1:
        raise SystemExit("bench.py measures one GPU: this build has no multi-GPU path (every stage check is "
                         "independent per micro-batch, so submissions would be dealt round-robin to GPUs that each hold the stage weights). Use --gpus 1.")
    if a.score_bench:
        return score_bench(a)
    if a.loop_bench:
        return loop_bench(a)
    if a.gemm_bench:
        return gemm_bench(a)
    if a.sweep:
        import subprocess
        for s_ in (512, 2048, 4096):
            for b_ in (1, 4, 16):
                r = subprocess.run([sys.executable, os.path.abspath(__file__), "--workload", f"sweep_s{s_}_b{b_}", "--steps", str(a.steps),
                                    "--warmup", str(a.warmup), "--no-cpu-baseline"], capture_output=True, text=True)
                print(r.stdout.strip() if r.returncode == 0 else json.dumps({"workload": f"sweep_s{s_}_b{b_}", "error": r.stderr[-300:]}), flush=True)
        return
    import torch
    import paper_2603_03592_amd as sv
    wl = get_workload(a.workload)
    backward = wl.backward if a.mode is None else (a.mode == "fwdbwd")
    desc, B, S = wl.desc, wl.batch, wl.seq
    T = B * S
    torch.cuda.set_device(0)
    dt = torch.bfloat16 if desc.dtype == "bf16" else torch.float32
    wdev = device_weights(desc, torch)
    g = torch.Generator(device="cuda").manual_seed(2)
    h_in = torch.randn((B, S, desc.d_model), generator=g, device="cuda", dtype=torch.float32).to(dt)
    g_out = (1e-3 * torch.randn((B, S, desc.d_model), generator=g, device="cuda", dtype=torch.float32)).to(dt)

    fuse_norm = a.fuse_norm == "on" or (a.fuse_norm == "auto" and sv.fuse_norm_pays(desc))
    ver = sv.Verifier(desc, T, S, backward=backward, plain_kernels=a.plain, fuse_norm=fuse_norm)
    wc = ver.pack_weights(wdev)
    prepare_ms = None
    if backward or fuse_norm:
        # the stage parameters stay fixed while the micro-batches of an iteration are checked: the context's copies of
        # them (transposed for the backward products, with the norm gains folded in for the products that follow a
        # norm) are made once, outside the timed steps, and the cost is reported
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        ver.prepare_weights(wc)
        e1.record()
        torch.cuda.synchronize()
        prepare_ms = e0.elapsed_time(e1)
    tau = {"rel_l2": wl.tau}
    if backward:
        first = ver.verify_backward(wc, h_in, g_out, want_g_hat=True, want_h_hat=True)
        claim_h, claim_g = corrupt_tokens(first["h_hat"], torch), corrupt_tokens(first["g_hat"], torch)
    else:
        first = ver.verify_forward(wc, h_in, want_h_hat=True)
        claim_h, claim_g = corrupt_tokens(first["h_hat"], torch), None
    res = torch.empty((2, 32), dtype=torch.uint8, device="cuda")
    h_hat = torch.empty_like(h_in) if backward else None
    dcode = 1 if desc.dtype == "bf16" else 0
    tau_c = (sv.binding.C.c_float * 4)(wl.tau, 0, 0, 0)
    stream = torch.cuda.current_stream().cuda_stream
    L = sv.lib

    def step():
        if backward:
            # one pass recomputes forward and backward; the gradient claim is scored inside the call,
            # the activation claim against the recomputed stage output it hands back
            st = L.sv_verify_backward(ver._ctx, wc, h_in.data_ptr(), g_out.data_ptr(), B, S, claim_g.data_ptr(), 1, tau_c, 1,
                                      None, h_hat.data_ptr(), None, res[1:].data_ptr(), stream)
            assert st == 0, L.sv_last_error(ver._ctx)
            st = L.sv_score_and_flag(ver._ctx, claim_h.data_ptr(), 0, 1, h_hat.data_ptr(), 0, dcode, dcode, T, desc.d_model, 1,
                                     tau_c, 1, None, res.data_ptr(), stream)
            assert st == 0, L.sv_last_error(ver._ctx)
        else:
            st = L.sv_verify_forward(ver._ctx, wc, h_in.data_ptr(), B, S, claim_h.data_ptr(), 1, tau_c, 1, None, None,
                                     res.data_ptr(), stream)
            assert st == 0, L.sv_last_error(ver._ctx)

    if a.copy_calibration:
        src = torch.empty(1 << 29, dtype=torch.bfloat16, device="cuda").normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(a.warmup):
        step()
    torch.cuda.synchronize()
    # The per-operation table comes from an untimed pass with events around every launch (a check is up to a hundred
    # launches, and a pair of events around each costs a check of short launches 3-5 %); the timed steps bracket only the
    # dominant product, whose launch duration the roofline object needs from that same timed region.
    ver.profile_select(None)
    ver.profile_enable(True)
    for _ in range(min(a.steps, 5)):
        step()
    torch.cuda.synchronize()
    prof_all = ver.profile_read()
    ver.profile_enable(False)
    prof_steps = min(a.steps, 5)
    dom = max((k for k in prof_all if k.startswith(("gemm", "bwd_gemm"))), key=lambda k: prof_all[k]["flop"])
    ver.profile_select([dom])
    ver.profile_enable(True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(a.steps):
        step()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    prof_dom = ver.profile_read()
    ver.profile_enable(False)
    ver.profile_select(None)
    flags = ver.read_results(res)["flag"]
    assert flags[0] == 1 and (not backward or flags[1] == 1), "the corrupted claims must be flagged"
    graph_ms = None
    if a.graph:
        # the step enqueues kernels only, so it can be captured once and replayed per micro-batch: launch latency drops out
        res.zero_()
        torch.cuda.synchronize()
        graph, side = torch.cuda.CUDAGraph(), torch.cuda.Stream()
        with torch.cuda.graph(graph, stream=side):
            stream = torch.cuda.current_stream().cuda_stream
            step()
        stream = torch.cuda.current_stream().cuda_stream
        for _ in range(a.warmup):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(a.steps):
            graph.replay()
        torch.cuda.synchronize()
        graph_ms = 1e3 * (time.perf_counter() - t0) / a.steps
        flags = ver.read_results(res)["flag"]
        assert flags[0] == 1 and (not backward or flags[1] == 1), "the corrupted claims must be flagged (graph replay)"
        del graph

    ms_step = 1e3 * wall / a.steps
    prof = prof_all
    tot_flop = sum(p["flop"] for p in prof.values()) / prof_steps
    tot_ms = sum(p["ms"] for p in prof.values()) / prof_steps
    d = prof_dom[dom]                                       # the dominant product's launches of the TIMED steps
    achieved = d["flop"] / (d["ms"] * 1e-3) / 1e12 if d["ms"] > 0 else 0.0
    out = {
        "metric": "verified tokens/sec per stage check" + (" (fwd+bwd)" if backward else " (fwd)"),
        "value": T / (ms_step * 1e-3), "unit": "tokens/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": ms_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": desc.dtype, "data": "synthetic",
        "config": {"workload": wl.name, "n_blocks": desc.n_blocks, "d_model": desc.d_model, "n_heads": desc.n_heads,
                   "n_kv_heads": desc.n_kv_heads, "ffn_hidden": desc.ffn_hidden, "micro_batch": B, "seq_len": S,
                   "check": "fwd+bwd" if backward else "fwd", "claims_per_step": 1, "kernels": "plain" if a.plain else "mfma", "norms": "inside the products" if fuse_norm else "own passes",
                   "weight_prepare_ms_once": prepare_ms,
                   **({"n_experts": desc.n_experts, "top_k": desc.top_k, "n_shared": desc.n_shared, "router_score": desc.router_score,
                       "router_norm": desc.router_norm} if desc.n_experts else {})},
        "roofline": {"bound": "mfma", "kernel": dom, "achieved": achieved, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / PEAK_BF16_TFLOPS,
                     "traffic": measured_traffic(wl.name + ("_fwdbwd" if backward and not wl.backward else ""), dom),
                     "launch_ms": d["ms"] / max(d["launches"], 1), "flop_per_launch": d["flop"] / max(d["launches"], 1)},
        "recompute": {"flop_per_step": tot_flop, "tflops": tot_flop / (ms_step * 1e-3) / 1e12,
                      "frac_of_bf16_mfma_peak": tot_flop / (ms_step * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
                      "kernel_ms_per_step": tot_ms,
                      "per_op_source": f"untimed pass of {prof_steps} steps with events around every launch; the timed steps bracket {dom} only",
                      "per_op_ms": {k: round(v["ms"] / prof_steps, 4) for k, v in prof.items() if v["launches"]},
                      "per_op_tflops": {k: round(v["flop"] / (v["ms"] * 1e-3) / 1e12, 1) for k, v in prof.items() if v["flop"] and v["ms"] > 0}},
    }
    if graph_ms is not None:
        out["graph_replay"] = {"ms_per_step": graph_ms, "value": T / (graph_ms * 1e-3), "unit": "tokens/s"}
    if wl.name.startswith("sweep"):
        # many workers per stage: up to 128 concurrent submissions of the stage output scored in one call against the
        # recomputation they share (submissions made on the device from the recomputed output; capped at 16 GiB)
        n_sub = int(max(1, min(128, (16 << 30) // (T * desc.d_model * 2))))
        ref_out = first["h_hat"].reshape(T, desc.d_model)
        subs = torch.empty((n_sub, T, desc.d_model), dtype=ref_out.dtype, device="cuda")
        for i in range(n_sub):
            subs[i] = ref_out * (1.5 if i % 8 == 3 else 1.0)
        ver.score_and_flag(subs, ref_out, tau=tau)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(5):
            r = ver.score_and_flag(subs, ref_out, tau=tau)
        e1.record()
        torch.cuda.synchronize()
        ms_sc = e0.elapsed_time(e1) / 5
        fl = ver.read_results(r["result"])["flag"]
        assert [int(f) for f in fl] == [int(i % 8 == 3) for i in range(n_sub)]
        by = (n_sub + 1) * T * desc.d_model * 2
        out["concurrent_scoring"] = {"submissions": n_sub, "ms": ms_sc, "achieved_GBs": by / (ms_sc * 1e-3) / 1e9,
                                     "frac_of_hbm_peak": by / (ms_sc * 1e-3) / 1e9 / PEAK_HBM_GBS}
        del subs
    if not a.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, wdev, h_in, g_out, backward)
    ver.close()
    if wl.name == "large" and a.mode is None and not a.plain and not a.no_extra:
        # Further legs of the same measurement, each in a child process of its own (one context at a time on the GPU):
        #   fwd_bwd_check  the forward + backward form of the check on the configuration that defines it (medium stage);
        #   fwd_bwd_large  the same form on the LARGEST shape (the large stage's four blocks, 8192 tokens);
        #   score_roofline the HBM-bound half: 128 submissions of [8192, 4096] scored against one shared reference.
        import subprocess
        del wdev, h_in, first, claim_h, wc
        torch.cuda.empty_cache()

        def child(extra):
            r = subprocess.run([sys.executable, os.path.abspath(__file__), *extra, "--steps", str(a.steps), "--warmup", str(a.warmup),
                                "--no-cpu-baseline"], capture_output=True, text=True)
            if r.returncode != 0:
                return None, r.stderr[-300:]
            return json.loads(r.stdout.strip().splitlines()[-1]), None

        for key, extra in (("fwd_bwd_check", ["--workload", "medium"]), ("fwd_bwd_large", ["--workload", "large", "--mode", "fwdbwd"])):
            m, err = child(extra)
            out[key] = {"error": err} if m is None else {
                "metric": m["metric"], "value": m["value"], "unit": m["unit"], "ms_per_step": m["ms_per_step"], "config": m["config"],
                "roofline": m["roofline"], "recompute_tflops": m["recompute"]["tflops"],
                "frac_of_bf16_mfma_peak": m["recompute"]["frac_of_bf16_mfma_peak"], "per_op_ms": m["recompute"]["per_op_ms"],
                "per_op_tflops": m["recompute"]["per_op_tflops"]}
        m, err = child(["--score-bench"])
        out["score_roofline"] = {"error": err} if m is None else {
            "metric": m["metric"], "value": m["value"], "unit": m["unit"], "ms_per_step": m["ms_per_step"], "config": m["config"],
            "roofline": m["roofline"], "rel_l2_only": m["rel_l2_only"], "ema": m["ema"]}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
