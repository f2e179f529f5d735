#!/usr/bin/env python3
"""Benchmark of the draft-then-verify step on one MI355X.

Workload (BASELINE config 2): 7B-shape bf16 target (32 layers, d 4096, 32 heads,
FFN 11008, vocab 32000) with the 68M-shape draft (2 layers, d 768), batch 1,
prompt of 512 uniform tokens, gamma = 5, T = 1, random N(0, 0.02) weights.
A "step" is one pass of the whole hot path: sd_draft (gamma candidates) followed
by sd_verify (gamma+1 rows, accept/resample, commit).  Inputs (weights, prompt,
uniforms, KV cache of the prefilled prompt) are resident in HBM before the timed
region starts.

Secondary objects on the same line: the verify pass alone and the whole routed step (four drafts of
different shapes) at batch 32, plain autoregressive decoding through the same library, and the CPU oracle.

Prints ONE JSON line.  `value` is verified candidate tokens per second over the
whole step, B*gamma*K / t.  `roofline` is for the dominant kernel (the SwiGLU
gate/up weight-streaming GEMM), timed live with HIP events on the launch stream in
a separate pass; `cpu_baseline` times the CPU oracle on one step of the same shape.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
GATEUP_TRAFFIC_BYTES = 181.3e6  # FETCH_SIZE + WRITE_SIZE per launch (181.1 + 0.2 MB), rocprofv3 --pmc: profiles/config2_b1_7b_hbm_traffic.md


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=40)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--layers", type=int, default=0, help="debug: reduce target depth (invalidates the number)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-batch32", action="store_true", help="skip the secondary batch-32 verify measurement")
    ap.add_argument("--no-long-context", action="store_true", help="skip the verify passes of configs 4 and 5")
    ap.add_argument("--batch32-only", action="store_true",
                    help="only the batch-32 verify pass (config 3 shape), a few repetitions: the command the "
                         "batch-32 rocprofv3 summaries under profiles/ are taken from (own JSON line)")
    ap.add_argument("--stream-probe", action="store_true",
                    help="only a plain streaming read of 33.6 / 100.7 / 180.4 / 262.1 MB / 1 GiB buffers (the sizes of "
                         "the 7B shape's weight matrices): the practical HBM read ceiling (own JSON line)")
    ap.add_argument("--temperature", type=float, default=1.0)
    ap.add_argument("--prompt", type=int, default=512)
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run a plain 1 GiB device copy three times (known traffic, to scale HBM counters)")
    ap.add_argument("--prefill-bench", action="store_true",
                    help="side measurement: prompt prefill of the 7B-shape target at 512 / 2048 / 8192 tokens (own JSON line)")
    ap.add_argument("--long-context", action="store_true",
                    help="side measurement: the verify pass of configs 4 (13B shape, batch 32, context 2048) and 5 "
                         "(7B shape, batch 64, contexts 1024..8192) with prefilled caches (own JSON line; minutes)")
    ap.add_argument("--multi-lora", action="store_true",
                    help="side measurement: draft phase of 32 routed sequences as four group calls vs one batch of the "
                         "shared base with per-sequence adapters (own JSON line)")
    ap.add_argument("--classifier", action="store_true",
                    help="side measurement: route 400 synthetic prompts with the prompt classifier (own JSON line)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU only: this build has no multi-GPU path (sequences are independent, so a "
              "batch would shard by sequence with no communication inside a step). Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2505_08600_amd import api
    from paper_2505_08600_amd import datagen as dg

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    if args.copy_calibration:
        n = 1 << 30
        src = torch.ones(n, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes_read": n, "copy_bytes_written": n, "launches": 3}))
        return
    api.lib()
    if args.classifier:
        classifier_bench(api, dg, torch, np, args)
        return
    if args.stream_probe:
        stream_probe(api, torch, np)
        return
    if args.batch32_only:
        st = dg.SHAPES["t7b"] if not args.layers else dg.with_layers(dg.SHAPES["t7b"], args.layers)
        gt = api.Model(st, dg.make_weights(st, 2025, threads=16), max_rows=192, max_pos=1200)
        res = batch32_verify(api, dg, torch, np, gt, st, 2025, 32, (128, 1024), 5, reps=max(3, args.steps if args.steps != 40 else 5))
        print(json.dumps({"metric": "batch32_verify_candidates_per_s", "value": res["candidates_per_s"],
                          "unit": "candidate tokens/s", "n_gpus": 1, "dtype": "bf16", "data": "synthetic",
                          "higher_is_better": True, "vs_baseline": None, "config": {"workload": res["workload"]},
                          "batch32_verify": res}))
        return
    if args.prefill_bench:
        prefill_bench(api, dg, torch, np, args)
        return
    if args.multi_lora:
        multi_lora_bench(api, dg, torch, np, args)
        return
    if args.long_context:
        long_context_bench(api, dg, torch, np, args)
        return
    seed, gamma, T, B = 2025, 5, float(args.temperature), 1
    st = dg.SHAPES["t7b"] if not args.layers else dg.with_layers(dg.SHAPES["t7b"], args.layers)
    sd_ = dg.SHAPES["draft_a"]
    V = st.vocab
    K, W = args.steps, args.warmup
    DIST_STEPS = max(50, K)   # steps timed one by one for the median / p10 / p90 (whatever --steps says)
    n_total = K + W + 8 + DIST_STEPS
    AR_STEPS = 16  # plain autoregressive decoding with the same library (gamma = 0), timed after the main loop
    cap = args.prompt + n_total * (gamma + 1) + 16 + AR_STEPS

    t0 = time.time()
    wt = dg.make_weights(st, seed, threads=16)
    wd = dg.make_weights(sd_, seed + 1, threads=16)
    log(f"[bench] weights generated on host in {time.time() - t0:.1f}s")
    t0 = time.time()
    B32, LEN32 = 32, (128, 1024)  # secondary measurement: the verify pass of config 3's batch (32 prompts, gamma 5)
    gt = api.Model(st, wt, max_rows=max(16, B32 * (gamma + 1)), max_pos=max(cap, LEN32[1] + 64) + 64)
    gd = api.Model(sd_, wd, max_rows=16, max_pos=cap + 64)
    torch.cuda.synchronize()
    log(f"[bench] uploaded in {time.time() - t0:.1f}s")

    prompt = [int(t) for t in dg.make_prompt(seed, 0, args.prompt, V)]
    ctx = api.Context([cap])
    ctx.attach(gt)
    ctx.attach(gd)
    ctx.set_tokens([prompt])
    t0 = time.time()
    api.sd_prefill(gt, ctx, None, 1, len(prompt) - 1)
    api.sd_prefill(gd, ctx, None, 1, len(prompt) - 1)
    torch.cuda.synchronize()
    log(f"[bench] prefill of {len(prompt)} tokens: {time.time() - t0:.2f}s")

    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    ud = [dev(dg.make_uniforms(seed, dg.DRAFT_STREAM, 0, k, gamma)[None]) for k in range(n_total)]
    uv = [dev(dg.make_uniforms(seed, dg.VERIFY_STREAM, 0, k, gamma + 1)[None]) for k in range(n_total)]
    cand = torch.zeros((B, gamma), dtype=torch.int32, device="cuda")
    q = torch.zeros((B, gamma, V), dtype=torch.float32, device="cuda")
    na = torch.zeros(B, dtype=torch.int32, device="cuda")
    nx = torch.zeros(B, dtype=torch.int32, device="cuda")
    na_log = torch.zeros((n_total, B), dtype=torch.int32, device="cuda")

    def step(k):
        api.sd_draft(gd, ctx, None, B, gamma, T, ud[k] if T > 0 else None, cand, q if T > 0 else None)
        api.sd_verify(gt, ctx, None, B, gamma, T, cand, q if T > 0 else None, uv[k] if T > 0 else None, na, nx, True)
        na_log[k].copy_(na)

    for k in range(W):
        step(k)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(W, W + K):
        step(k)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / K * 1e3
    n_acc = na_log[W:W + K, 0].cpu().numpy()
    ctx.sync()  # raises if a kernel flagged an inconsistency

    # ---- the same step timed one at a time (events on the launch stream around each step): spread of the step time
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(DIST_STEPS)]
    for i, k in enumerate(range(W + K + 8, W + K + 8 + DIST_STEPS)):
        evs[i][0].record()
        step(k)
        evs[i][1].record()
    torch.cuda.synchronize()
    step_ms = np.array([a.elapsed_time(b) for a, b in evs])
    ctx.sync()

    # ---- phase split: draft-only and verify-only timings (same state machine, separate loops)
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    reps = min(K, 20)
    t_draft = t_verify = 0.0
    for k in range(W + K, W + K + 4):
        ev0.record()
        api.sd_draft(gd, ctx, None, B, gamma, T, ud[k] if T > 0 else None, cand, q if T > 0 else None)
        ev1.record()
        torch.cuda.synchronize()
        t_draft += ev0.elapsed_time(ev1)
        ev0.record()
        api.sd_verify(gt, ctx, None, B, gamma, T, cand, q if T > 0 else None, uv[k] if T > 0 else None, na, nx, True)
        ev1.record()
        torch.cuda.synchronize()
        t_verify += ev0.elapsed_time(ev1)
    t_draft /= 4
    t_verify /= 4

    # ---- per-kernel pass with HIP events on the launch stream (library option "profile")
    api.set_option("profile", 1)
    for k in range(W + K + 4, W + K + 8):
        step(k)
    torch.cuda.synchronize()
    api.set_option("profile", 0)
    prof = api.profile_read()
    ctx.sync()
    # dominant kernel: SwiGLU gate/up GEMM of the target.  Algorithmic bytes per launch: both weight
    # matrices once (2*F*d bf16) + the M input rows (M*d bf16) + the M output rows (M*F bf16).
    M = B * (gamma + 1)
    gu_bytes = 2 * st.d_ffn * st.d_model * 2 + M * st.d_model * 2 + M * st.d_ffn * 2
    # gate/up launches of the profile pass: 4 verify forwards (target) + 4*gamma draft forwards; split by
    # model via launch counts (the draft has 2 layers, the target n_layers)
    cnt, tot_ms = prof["gemm_gateup"]
    # weight the classes by bytes: draft launches are ~50x smaller; report the target's kernel only by
    # timing it in isolation below
    api.set_option("profile", 1)
    for k in range(3):
        api.sd_verify(gt, ctx, None, B, gamma, T, cand, q if T > 0 else None, uv[k] if T > 0 else None, na, nx, False)
        torch.cuda.synchronize()
        ctx.truncate(gt, 0, int(ctx.sync()[0][0]) - 1)
    api.set_option("profile", 0)
    vprof = api.profile_read()
    gcnt, gms = vprof["gemm_gateup"]
    gu_ms = gms / max(gcnt, 1)
    # the draft alone, same way: launches and time per class of one sd_draft call (the draft is bound by the
    # number of dependent launches; its one bandwidth-shaped kernel is the LM head)
    n_tok0, kv0 = ctx.sync(gd)
    api.set_option("profile", 1)
    for k in range(3):
        api.sd_draft(gd, ctx, None, B, gamma, T, ud[k] if T > 0 else None, cand, q if T > 0 else None)
        torch.cuda.synchronize()
        ctx.truncate(gd, 0, int(kv0[0]))
    api.set_option("profile", 0)
    dprof = api.profile_read()
    d_launches = sum(v[0] for v in dprof.values())
    lm_cnt, lm_ms = dprof.get("gemm_lmhead", (0, 0.0))
    lm_us = lm_ms / max(lm_cnt, 1) * 1e3
    draft_obj = {"us_per_token": t_draft / gamma * 1e3, "launches_per_token": d_launches / (3.0 * gamma),
                 "lm_head_us_per_launch": lm_us, "lm_head_mb": sd_.vocab * sd_.d_model * 2 / 1e6,
                 "lm_head_gb_per_s": sd_.vocab * sd_.d_model * 2 / max(lm_us, 1e-9) / 1e3,
                 "kernel_us_per_token": {k: v[1] * 1e3 / (3.0 * gamma) for k, v in dprof.items() if v[0]}}
    achieved = gu_bytes / (gu_ms * 1e-3) / 1e9
    # whole verify call against its own algorithmic traffic
    n_ctx = int(ctx.sync()[0][0])
    verify_bytes = st.n_streamed_params() * 2 + st.kv_bytes_per_token() * n_ctx
    verify_frac = verify_bytes / (t_verify * 1e-3) / 1e9 / HBM_PEAK_GBS

    tau = float(np.mean(n_acc + 1))
    alpha_hat = api.alpha_hat(n_acc.reshape(-1).tolist(), gamma)
    c_ratio = (t_draft / gamma) / t_verify
    eq1 = api.eq1_speedup(alpha_hat, gamma, c_ratio)
    best_gamma, best_eq1 = api.choose_gamma(alpha_hat, c_ratio, 15)   # Equation 1's optimum for this pair

    out = {
        "metric": "verified candidate tokens/s + accepted tokens/s, 7B-shape target, gamma=5, batch 1",
        "value": B * gamma * K / dt,
        "unit": "candidate tokens/s",
        "n_gpus": 1, "steps": K, "warmup": W, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "config 2: 7B-shape target + 68M-shape draft, batch 1, prompt %d, gamma 5, T=%g"
                               % (args.prompt, T),
                   "target_layers": st.n_layers, "batch": B, "gamma": gamma, "temperature": T},
        "emitted_tokens_per_s": float((n_acc + 1).sum() / dt),
        "accepted_tokens_per_s": float(n_acc.sum() / dt),
        "verify_only_candidates_per_s": B * gamma / (t_verify * 1e-3),
        "step_ms_distribution": {"n": int(DIST_STEPS), "median": float(np.median(step_ms)),
                                 "p10": float(np.percentile(step_ms, 10)), "p90": float(np.percentile(step_ms, 90))},
        "ms_draft": t_draft, "ms_verify": t_verify,
        "acceptance_rate_eq2": float(n_acc.sum() / (K * gamma)), "tau": tau, "alpha_hat": alpha_hat,
        "c_draft_over_target": c_ratio, "eq1_speedup_model": eq1,
        "eq1_best_gamma": best_gamma, "eq1_best_speedup": best_eq1,
        "verify_hbm_frac": verify_frac,
        "roofline": {"bound": "hbm", "kernel": "gemm_ksplit_kernel<2,true,1,2,1> (gate/up + SiLU*mul) M=%d N=%d K=%d" % (M, st.d_ffn, st.d_model),
                     "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     # FETCH_SIZE + WRITE_SIZE per launch of this kernel at this shape, scaled by a plain copy
                     # (profiles/config2_b1_7b_hbm_traffic.md); only meaningful for the default workload
                     "traffic": GATEUP_TRAFFIC_BYTES if (not args.layers and args.prompt == 512) else None,
                     "us_per_launch": gu_ms * 1e3, "algorithmic_bytes": gu_bytes},
        "kernel_ms_per_verify": {k: v[1] / 3.0 for k, v in vprof.items() if v[0]},
        "draft": draft_obj,
    }

    # ---- Equation 1 against a measurement: plain autoregressive decoding of the same target through the
    # same library (verify with gamma = 0: one row, one token per call).  Last use of this context: the
    # draft's cache is left behind.
    u_ar = uv[0][:, :1].contiguous()
    for r in range(AR_STEPS + 2):
        if r == 2:
            torch.cuda.synchronize()
            t0 = time.perf_counter()
        api.sd_verify(gt, ctx, None, B, 0, T, None, None, u_ar if T > 0 else None, na, nx, True)
    torch.cuda.synchronize()
    ms_ar = (time.perf_counter() - t0) / AR_STEPS * 1e3
    ctx.sync()
    emitted_per_s = float((n_acc + 1).sum() / dt)
    out["ar_baseline"] = {"ms_per_token": ms_ar, "tokens_per_s": B / (ms_ar * 1e-3),
                          "measured_speedup": emitted_per_s / (B / (ms_ar * 1e-3)),
                          "eq1_with_measured_alpha_c": eq1}

    # ---- the step at the candidate count Equation 1 picks for the measured (alpha, c): same loop, other gamma
    if best_gamma >= 1 and best_gamma != gamma:
        g2, n2 = best_gamma, 24
        ud2 = [dev(dg.make_uniforms(seed + 1, dg.DRAFT_STREAM, 0, k, g2)[None]) for k in range(n2)]
        uv2 = [dev(dg.make_uniforms(seed + 1, dg.VERIFY_STREAM, 0, k, g2 + 1)[None]) for k in range(n2)]
        cand2 = torch.zeros((B, g2), dtype=torch.int32, device="cuda")
        q2 = torch.zeros((B, g2, V), dtype=torch.float32, device="cuda")
        ctx2 = api.Context([args.prompt + n2 * (g2 + 1) + 16])
        ctx2.attach(gt)
        ctx2.attach(gd)
        ctx2.set_tokens([prompt])
        api.sd_prefill(gt, ctx2, None, 1, len(prompt) - 1)
        api.sd_prefill(gd, ctx2, None, 1, len(prompt) - 1)
        na2 = torch.zeros((n2, B), dtype=torch.int32, device="cuda")
        for k in range(n2):
            if k == 4:
                torch.cuda.synchronize()
                t0 = time.perf_counter()
            api.sd_draft(gd, ctx2, None, B, g2, T, ud2[k] if T > 0 else None, cand2, q2 if T > 0 else None)
            api.sd_verify(gt, ctx2, None, B, g2, T, cand2, q2 if T > 0 else None, uv2[k] if T > 0 else None, na, nx, True)
            na2[k].copy_(na)
        torch.cuda.synchronize()
        dt2 = time.perf_counter() - t0
        ctx2.sync()
        ctx2.close()
        acc2 = na2[4:, 0].cpu().numpy()
        out["step_at_eq1_gamma"] = {"gamma": g2, "steps": n2 - 4, "ms_per_step": dt2 / (n2 - 4) * 1e3,
                                    "emitted_tokens_per_s": float((acc2 + 1).sum() / dt2),
                                    "emitted_tokens_per_s_at_gamma_5": emitted_per_s}
    if not args.no_batch32:
        out["batch32_verify"] = batch32_verify(api, dg, torch, np, gt, st, seed, B32, LEN32, gamma)
        out["batch32_step"] = batch32_step(api, dg, torch, np, gt, st, seed, B32, LEN32, gamma)
    ctx.close()
    gd.close()
    gt.close()
    del gt, gd
    torch.cuda.empty_cache()
    if not args.no_long_context and not args.layers:
        out["long_context"], out["prefill_8192"] = long_context_cases(api, dg, torch, np, args)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(st, sd_, wt, wd, args.prompt, gamma, T, seed)
    print(json.dumps(out))


def batch32_verify(api, dg, torch, np, gt, st, seed, B, len_range, gamma, T=0.7, reps=10):
    """Verify pass alone at config 3's batch: B prompts with lengths uniform in len_range, gamma + 1 rows each
    (M = B * (gamma + 1) rows through every GEMM).  Reports the matrix-core rate: every weight is multiplied
    with the hi and the lo plane of each row, so 4 * M flops per streamed parameter are executed."""
    V = st.vocab
    lens = dg.make_prompt_lengths(seed + 7, B, len_range[0], len_range[1])
    prompts = [[int(t) for t in dg.make_prompt(seed + 7, b, int(lens[b]), V)] for b in range(B)]
    ctx = api.Context([int(l) + 4 * (gamma + 1) for l in lens])
    ctx.attach(gt)
    ctx.set_tokens(prompts)
    api.sd_prefill(gt, ctx, None, B, int(lens.max()) - 1)
    torch.cuda.synchronize()
    g = torch.Generator(device="cuda").manual_seed(seed)
    cand = torch.randint(0, V, (B, gamma), dtype=torch.int32, device="cuda", generator=g)
    q = torch.softmax(torch.randn((B, gamma, V), device="cuda", generator=g), dim=-1).contiguous()
    u = torch.rand((B, gamma + 1), device="cuda", generator=g)
    na = torch.zeros(B, dtype=torch.int32, device="cuda")
    nx = torch.zeros(B, dtype=torch.int32, device="cuda")
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ts = []
    for r in range(reps + 2):  # commit=False, then roll the cache lengths back: every repetition verifies the same state
        ev0.record()
        api.sd_verify(gt, ctx, None, B, gamma, T, cand, q, u, na, nx, False)
        ev1.record()
        torch.cuda.synchronize()
        if r >= 2:
            ts.append(ev0.elapsed_time(ev1))
        for b in range(B):
            ctx.truncate(gt, b, int(lens[b]) - 1)
    ms = float(np.mean(ts))
    # per-kernel-class times of one more call (HIP events around every launch; adds ~2 us per launch)
    api.set_option("profile", 1)
    api.sd_verify(gt, ctx, None, B, gamma, T, cand, q, u, na, nx, False)
    torch.cuda.synchronize()
    api.set_option("profile", 0)
    prof = api.profile_read()
    ctx.sync()
    ctx.close()
    M = B * (gamma + 1)
    # the method's own work: 2 flops per streamed parameter and row.  The kernels issue twice that, because every
    # activation row enters the matrix cores as two bf16 terms (hi + lo).
    useful = 2.0 * M * st.n_streamed_params()
    d, F, V_ = st.d_model, st.d_ffn, st.vocab
    per_class = {}
    for name, params in (("gemm_qkv", 3 * d * d), ("gemm_o", d * d), ("gemm_gateup", 2 * F * d), ("gemm_down", F * d),
                         ("gemm_lmhead", V_ * d)):
        cnt, tot = prof.get(name, (0, 0.0))
        if cnt:
            us = tot / cnt * 1e3
            per_class[name] = {"us_per_launch": us, "mfma_frac_useful": 2.0 * M * params / (us * 1e-6) / 2.5e15,
                               "mfma_frac_issued": 4.0 * M * params / (us * 1e-6) / 2.5e15,
                               "weight_gb_per_s": params * 2 / (us * 1e-6) / 1e9}
    for name in ("attention", "rmsnorm", "verify_tail"):
        cnt, tot = prof.get(name, (0, 0.0))
        if cnt:
            per_class[name] = {"us_per_launch": tot / cnt * 1e3, "launches": cnt}
    kv_bytes = float(lens.sum()) * st.kv_bytes_per_token()
    return {"workload": "config 3 shape: %d prompts, lengths U[%d,%d], gamma %d, T=%g, verify pass only" %
                        (B, len_range[0], len_range[1], gamma, T),
            "rows": M, "ms_verify": ms, "ms_verify_median": float(np.median(ts)), "reps": len(ts),
            "candidates_per_s": B * gamma / (ms * 1e-3),
            "mfma_peak_tflops": 2500.0,
            "mfma_frac_useful": useful / (ms * 1e-3) / 2.5e15,      # headline: 2*M flops per parameter
            "mfma_frac_issued": 2.0 * useful / (ms * 1e-3) / 2.5e15,  # hi and lo plane: 4*M flops per parameter
            "hbm_frac": (st.n_streamed_params() * 2 + kv_bytes) / (ms * 1e-3) / 8e12,
            "kv_gb": kv_bytes / 1e9, "kernels": per_class}


def batch32_step(api, dg, torch, np, gt, st, seed, B, len_range, gamma, T=0.7, steps=10, warmup=2):
    """The whole step at config 3's batch: B prompts routed by the linear classifier to four drafts of different
    shapes (68M shape; 4 and 6 layers of width 1024; 2 layers of width 2048), sequences ordered by draft so that
    every group is a contiguous slice of the batch; a step = one sd_draft per group (each group on a stream of
    its own) + one sd_verify (commit fused) over all B sequences.  Same candidate-token accounting as the headline value."""
    V = st.vocab
    shapes = [dg.SHAPES[n] for n in ("draft_a", "draft_b", "draft_c", "draft_d")]
    Wr, br = dg.make_router(seed + 8)
    emb = dg.make_prompt_embeddings(seed + 8, B)
    ids = torch.zeros(B, dtype=torch.int32, device="cuda")
    api.sd_route(torch.from_numpy(Wr).cuda(), torch.from_numpy(br).cuda(), torch.from_numpy(emb).cuda(), ids)
    route = np.sort(ids.cpu().numpy(), kind="stable")     # batch order = by routed draft
    bounds = [(int(np.searchsorted(route, g, "left")), int(np.searchsorted(route, g, "right"))) for g in range(4)]
    lens = dg.make_prompt_lengths(seed + 8, B, len_range[0], len_range[1])
    prompts = [[int(t) for t in dg.make_prompt(seed + 8, b, int(lens[b]), V)] for b in range(B)]
    n_total = steps + warmup
    gds = [api.Model(sh, dg.make_weights(sh, seed + 20 + i, threads=16), max_rows=2 * B,
                     max_pos=len_range[1] + n_total * (gamma + 1) + 64) for i, sh in enumerate(shapes)]
    ctx = api.Context([int(l) + n_total * (gamma + 1) + 16 for l in lens])
    ctx.attach(gt)
    for gd in gds:
        ctx.attach(gd)
    ctx.set_tokens(prompts)
    api.sd_prefill(gt, ctx, None, B, int(lens.max()) - 1)
    gid = [torch.arange(a, b, dtype=torch.int32, device="cuda") for a, b in bounds]
    for g, (a, b) in enumerate(bounds):
        if b > a:
            api.sd_prefill(gds[g], ctx, gid[g], b - a, int(lens[a:b].max()) - 1)
    torch.cuda.synchronize()
    gen = torch.Generator(device="cuda").manual_seed(seed + 8)
    ud = torch.rand((n_total, B, gamma), device="cuda", generator=gen)
    uv = torch.rand((n_total, B, gamma + 1), device="cuda", generator=gen)
    cand = torch.zeros((B, gamma), dtype=torch.int32, device="cuda")
    q = torch.zeros((B, gamma, V), dtype=torch.float32, device="cuda")
    na = torch.zeros(B, dtype=torch.int32, device="cuda")
    nx = torch.zeros(B, dtype=torch.int32, device="cuda")
    na_log = torch.zeros((n_total, B), dtype=torch.int32, device="cuda")
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(n_total)]

    # the groups' drafts are independent models: one stream each (default priority), joined before the verify
    main = torch.cuda.current_stream()
    streams = [torch.cuda.Stream() for _ in range(4)]

    def step(k):
        ev[k][0].record()
        for g, (a, b) in enumerate(bounds):
            if b > a:
                streams[g].wait_stream(main)
                with torch.cuda.stream(streams[g]):
                    api.sd_draft(gds[g], ctx, gid[g], b - a, gamma, T, ud[k, a:b], cand[a:b], q[a:b])
        for g, (a, b) in enumerate(bounds):
            if b > a:
                main.wait_stream(streams[g])
        ev[k][1].record()
        api.sd_verify(gt, ctx, None, B, gamma, T, cand, q, uv[k], na, nx, True)
        na_log[k].copy_(na)
        ev[k][2].record()

    for k in range(warmup):
        step(k)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(warmup, n_total):
        step(k)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ctx.sync()
    acc = int(na_log[warmup:].sum().item())
    ms_d = sum(ev[k][0].elapsed_time(ev[k][1]) for k in range(warmup, n_total)) / steps
    ms_v = sum(ev[k][1].elapsed_time(ev[k][2]) for k in range(warmup, n_total)) / steps
    out = {"workload": "config 3: %d prompts, lengths U[%d,%d], four routed drafts (groups of %s), gamma %d, T=%g" %
                       (B, len_range[0], len_range[1], "/".join(str(b - a) for a, b in bounds), gamma, T),
           "steps": steps, "ms_per_step": dt / steps * 1e3, "ms_draft_phase": ms_d, "ms_verify": ms_v,
           "candidates_per_s": B * gamma * steps / dt, "accepted_tokens_per_s": acc / dt,
           "emitted_tokens_per_s": (acc + B * steps) / dt, "acceptance_rate_eq2": acc / (B * gamma * steps)}
    ctx.close()
    for gd in gds:
        gd.close()
    return out


def prefill_bench(api, dg, torch, np, args):
    """The step before the hot path: sd_prefill of one prompt into the 7B-shape target, for four workspace sizes
    (max_rows decides how many 16-row groups one forward carries; the GEMMs' blocks fill the chip in whole rounds
    at 1024 and 2048 rows and in one and a half at 576).  Issued MFMA work counts the hi and the lo
    plane of every row (4 flops per parameter and token); attention is not counted."""
    st = dg.SHAPES["t7b"] if not args.layers else dg.with_layers(dg.SHAPES["t7b"], args.layers)
    wt = dg.make_weights(st, 2025, threads=16)
    res = []
    for max_rows in (192, 576, 1024, 2048):
        gt = api.Model(st, wt, max_rows, 8300)
        for n in (512, 2048, 8192):
            prompt = [[int(t) for t in dg.make_prompt(2025, 0, n, st.vocab)]]
            ctx = api.Context([n + 64])
            ctx.attach(gt)
            for rep in range(2):      # the second pass is the measured one
                ctx.set_tokens(prompt)
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                api.sd_prefill(gt, ctx, None, 1, n - 1)
                torch.cuda.synchronize()
                dt = time.perf_counter() - t0
            ctx.sync()
            res.append({"max_rows": max_rows, "prompt": n, "ms": dt * 1e3, "tokens_per_s": (n - 1) / dt,
                        "mfma_tflops": 4.0 * (n - 1) * st.n_streamed_params() / dt / 1e12})
            ctx.close()
        gt.close()
    best = max(r["tokens_per_s"] for r in res)
    print(json.dumps({"metric": "prefill_tokens_per_s", "value": best, "unit": "tokens/s", "n_gpus": 1, "dtype": "bf16",
                      "data": "synthetic", "higher_is_better": True, "vs_baseline": None,
                      "config": {"workload": "prefill of one prompt, 7B-shape target, batch 1"}, "cases": res}))


def long_context_bench(api, dg, torch, np, args):
    res, prefill = long_context_cases(api, dg, torch, np, args)
    print(json.dumps({"metric": "long_context_verify_candidates_per_s", "value": res[-1]["candidates_per_s"],
                      "unit": "candidate tokens/s", "n_gpus": 1, "dtype": "bf16", "data": "synthetic",
                      "higher_is_better": True, "vs_baseline": None,
                      "config": {"workload": "verify pass of configs 4 and 5 (value: config 5)"}, "cases": res,
                      "prefill_8192": prefill}))


def long_context_cases(api, dg, torch, np, args):
    """The verify pass of the two long-context configurations, caches filled by real prefills: config 4 (13B-shape
    target, 32 sequences at context 2048, gamma 3 / 5 / 8) and config 5 (7B-shape target, 64 sequences with
    contexts uniform in [1024, 8192], gamma 8).  Bytes = streamed weights + live KV of the call."""
    res, prefill = [], None
    for name, shape, B, lens, gammas in (("config 4", "t13b", 32, np.full(32, 2048, np.int32), (3, 5, 8)),
                                         ("config 5", "t7b", 64, dg.make_prompt_lengths(5055, 64, 1024, 8192), (8,))):
        st = dg.SHAPES[shape] if not args.layers else dg.with_layers(dg.SHAPES[shape], args.layers)
        V, T = st.vocab, 1.0
        t0 = time.time()
        wt = dg.make_weights(st, 2025, threads=16)
        max_pos = (max(int(lens.max()), 8192) if shape == "t7b" else int(lens.max())) + 64
        gt = api.Model(st, wt, max(16 * B, B * (max(gammas) + 1)), max_pos)   # 16 prompt rows per sequence and forward
        del wt
        prompts = [[int(t) for t in dg.make_prompt(2025, b, int(lens[b]), V)] for b in range(B)]
        ctx = api.Context([int(l) + 64 for l in lens])
        ctx.attach(gt)
        ctx.set_tokens(prompts)
        api.sd_prefill(gt, ctx, None, B, int(lens.max()) - 1)
        torch.cuda.synchronize()
        log(f"[bench] {name}: weights, upload and prefill of {int(lens.sum())} tokens in {time.time() - t0:.1f}s")
        g = torch.Generator(device="cuda").manual_seed(2025)
        for gamma in gammas:
            cand = torch.randint(0, V, (B, gamma), dtype=torch.int32, device="cuda", generator=g)
            q = torch.softmax(torch.randn((B, gamma, V), device="cuda", generator=g), dim=-1).contiguous()
            u = torch.rand((B, gamma + 1), device="cuda", generator=g)
            na = torch.zeros(B, dtype=torch.int32, device="cuda")
            nx = torch.zeros(B, dtype=torch.int32, device="cuda")
            ms, reps = 0.0, 5
            for r in range(reps + 2):   # commit = False, then the cache lengths are rolled back
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                api.sd_verify(gt, ctx, None, B, gamma, T, cand, q, u, na, nx, False)
                e1.record()
                torch.cuda.synchronize()
                if r >= 2:
                    ms += e0.elapsed_time(e1) / reps
                for b in range(B):
                    ctx.truncate(gt, b, int(lens[b]) - 1)
            M = B * (gamma + 1)
            nbytes = st.n_streamed_params() * 2 + float(lens.sum()) * st.kv_bytes_per_token()
            res.append({"config": name, "rows": M, "gamma": gamma, "ms_verify": ms, "bytes_gb": nbytes / 1e9,
                        "tb_per_s": nbytes / ms / 1e9, "hbm_frac": nbytes / ms / 1e9 / 8.0,
                        "mfma_frac_useful": 2.0 * M * st.n_streamed_params() / (ms * 1e-3) / 2.5e15,
                        "mfma_frac_issued": 4.0 * M * st.n_streamed_params() / (ms * 1e-3) / 2.5e15,
                        "candidates_per_s": B * gamma / ms * 1e3})
        ctx.sync()
        ctx.close()
        if shape == "t7b":   # the same model (1024-row workspace) prefilling one 8192-token prompt: the step before the hot path
            n = 8192
            prompt = [[int(t) for t in dg.make_prompt(2025, 0, n, V)]]
            c1 = api.Context([n + 64])
            c1.attach(gt)
            for rep in range(2):      # the second pass is the measured one
                c1.set_tokens(prompt)
                torch.cuda.synchronize()
                t1 = time.perf_counter()
                api.sd_prefill(gt, c1, None, 1, n - 1)
                torch.cuda.synchronize()
                dt = time.perf_counter() - t1
            c1.sync()
            c1.close()
            prefill = {"workload": "prefill of one 8192-token prompt, 7B-shape target, batch 1", "workspace_rows": 16 * B,
                       "ms": dt * 1e3, "tokens_per_s": (n - 1) / dt,
                       "mfma_frac_issued": 4.0 * (n - 1) * st.n_streamed_params() / dt / 2.5e15}
        gt.close()
        del gt
        torch.cuda.empty_cache()
    return res, prefill


def multi_lora_bench(api, dg, torch, np, args):
    """Draft phase of config 3's batch (32 prompts of 128..1024 tokens, gamma 5, T = 0.7) with the 68M-shape base
    draft: one batch without adapters, four calls on the routed groups (what separate per-task drafts of this
    shape cost), and one batch with four rank-8 adapters chosen per sequence (Section 2.3)."""
    B, gamma, T, seed = 32, 5, 0.7, 2025
    sh = dg.SHAPES["draft_a"]
    V = sh.vocab
    gd = api.Model(sh, dg.make_weights(sh, seed, threads=16), max_rows=2 * B, max_pos=1200)
    lora = dg.make_lora(sh, seed + 1, n_adapters=4, rank=8)
    Wr, br = dg.make_router(seed)
    ids = torch.zeros(B, dtype=torch.int32, device="cuda")
    api.sd_route(torch.from_numpy(Wr).cuda(), torch.from_numpy(br).cuda(),
                 torch.from_numpy(dg.make_prompt_embeddings(seed, B)).cuda(), ids)
    route = np.sort(ids.cpu().numpy(), kind="stable")
    bounds = [(int(np.searchsorted(route, g, "left")), int(np.searchsorted(route, g, "right"))) for g in range(4)]
    lens = dg.make_prompt_lengths(seed, B, 128, 1024)
    prompts = [[int(t) for t in dg.make_prompt(seed, b, int(lens[b]), V)] for b in range(B)]
    ctx = api.Context([int(l) + 64 for l in lens])
    ctx.attach(gd)
    ctx.set_tokens(prompts)
    api.sd_prefill(gd, ctx, None, B, int(lens.max()) - 1)
    torch.cuda.synchronize()
    gen = torch.Generator(device="cuda").manual_seed(seed)
    ud = torch.rand((B, gamma), device="cuda", generator=gen)
    cand = torch.zeros((B, gamma), dtype=torch.int32, device="cuda")
    q = torch.zeros((B, gamma, V), device="cuda")
    gid = [torch.arange(a, b, dtype=torch.int32, device="cuda") for a, b in bounds]

    def timed(fn):
        ts = []
        for rep in range(args.warmup + args.steps):
            torch.cuda.synchronize()
            for b in range(B):            # every repetition drafts from the same cache state
                ctx.truncate(gd, b, int(lens[b]) - 1)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            fn()
            e1.record()
            torch.cuda.synchronize()
            ts.append(e0.elapsed_time(e1))
        return float(np.median(ts[args.warmup:]))

    def groups():
        for g, (a, b) in enumerate(bounds):
            if b > a:
                api.sd_draft(gd, ctx, gid[g], b - a, gamma, T, ud[a:b], cand[a:b], q[a:b])

    ms_base = timed(lambda: api.sd_draft(gd, ctx, None, B, gamma, T, ud, cand, q))
    ms_groups = timed(groups)
    gd.set_lora(lora, 2.0)
    ctx.set_adapters(gd, route.tolist())
    ms_lora = timed(lambda: api.sd_draft(gd, ctx, None, B, gamma, T, ud, cand, q))
    ctx.sync()
    print(json.dumps({"metric": "multi_lora_draft_candidates_per_s", "value": B * gamma / ms_lora * 1e3,
                      "unit": "candidate tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
                      "ms_per_step": ms_lora, "higher_is_better": True, "dtype": "bf16", "data": "synthetic",
                      "vs_baseline": None,
                      "config": {"workload": "draft phase, 32 sequences (groups of %s), 68M-shape base, gamma 5, T=0.7, "
                                             "four rank-8 adapters on q,k,v,o" % "/".join(str(b - a) for a, b in bounds)},
                      "ms_one_batch_no_adapters": ms_base, "ms_four_group_calls": ms_groups,
                      "ms_one_batch_with_adapters": ms_lora}))
    ctx.close()
    gd.close()


def classifier_bench(api, dg, torch, np, args):
    """Routing by the prompt classifier (Sections 2.4, 3.3.3): 400 prompts, the size of the paper's
    classifier test set (Table 2), of log-normal length around 24 tokens after stop-word removal,
    default classifier shape, random weights.  One launch routes the whole batch."""
    shape, n, max_len, seed = dg.ClassifierShape(), 400, 128, 2025
    w = dg.make_classifier(shape, seed)
    tokens, lens = dg.make_classifier_prompts(seed, n, shape.vocab, max_len)
    cls = api.Classifier(shape, w)
    t, l = torch.from_numpy(tokens).cuda(), torch.from_numpy(lens).cuda()
    ids = torch.zeros(n, dtype=torch.int32, device="cuda")
    for _ in range(args.warmup):
        cls.route(t, l, ids)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(args.steps):
        cls.route(t, l, ids)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / args.steps
    out = {"metric": "classifier_prompts_per_s", "value": n / ms * 1e3, "unit": "prompts/s", "n_gpus": 1,
           "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True, "dtype": "f32",
           "data": "synthetic", "vs_baseline": None,
           "config": {"workload": f"{n} prompts, {int(lens.sum())} tokens, longest {int(lens.max())}, "
                                  f"d_model {shape.d_model}, d_inner {shape.d_inner}, d_state {shape.d_state}"},
           "tokens_per_s": float(lens.sum()) / ms * 1e3}
    if not args.no_cpu_baseline:
        from oracle import mamba
        sample = 100
        t0 = time.time()
        ref = [mamba.classify(w, tokens[i, :lens[i]])[1] for i in range(sample)]
        dt = time.time() - t0
        got = ids.cpu().numpy()[:sample]
        out["cpu_baseline"] = {"value": sample / dt, "unit": "prompts/s", "cores": 1, "kind": "oracle",
                               "sample": f"the first {sample} prompts", "labels_equal": int((got == np.array(ref)).sum())}
    cls.close()
    print(json.dumps(out))


def stream_probe(api, torch, np):
    """A kernel that only reads: buffers of the 7B shape's weight-matrix sizes (a fresh region of a 4 GiB pool every
    launch, so nothing is cache resident) and one 1 GiB read, in two patterns: every block reading one contiguous
    range with the nontemporal hint (what the weight-streaming kernels use) and a grid-strided read with ordinary loads."""
    pool = torch.ones(1 << 32, dtype=torch.uint8, device="cuda")
    word = torch.zeros(1, dtype=torch.int32, device="cuda")
    res = []
    for nt in (1, 0):
        api.set_option("stream_read_nt", nt)
        for mb in (33.6, 100.7, 180.4, 262.1, 1073.7):
            nbytes = int(mb * 1e6) // 4096 * 4096
            n_regions = max(1, (1 << 32) // nbytes)
            reps = min(n_regions, 12)
            views = [pool[i * nbytes:(i + 1) * nbytes] for i in range(n_regions)]
            api.stream_read(views[-1], word)
            torch.cuda.synchronize()
            evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
            for i in range(reps):
                evs[i][0].record()
                api.stream_read(views[i % n_regions], word)
                evs[i][1].record()
            torch.cuda.synchronize()
            us = float(np.median([a.elapsed_time(b) for a, b in evs])) * 1e3
            res.append({"pattern": "contiguous ranges, nontemporal" if nt else "grid-strided, ordinary loads", "mb": nbytes / 1e6,
                        "us": us, "gb_per_s": nbytes / us / 1e3, "frac_of_8_tb_s": nbytes / us / 1e3 / 8000.0})
    api.set_option("stream_read_nt", 1)
    print(json.dumps({"metric": "stream_read_gb_per_s", "value": res[4]["gb_per_s"], "unit": "GB/s", "n_gpus": 1,
                      "dtype": "u8", "data": "synthetic", "higher_is_better": True, "vs_baseline": None,
                      "config": {"workload": "plain streaming read, one launch per buffer (value: 1 GiB, contiguous ranges with the nontemporal hint)"},
                      "cases": res}))


def _cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def _omp_set_threads(n):
    """Thread count of the oracle's OpenMP loops for the calls that follow (the oracle itself is left as it is)."""
    import ctypes
    try:
        ctypes.CDLL("libgomp.so.1").omp_set_num_threads(int(n))
        return True
    except OSError:
        return False


def cpu_baseline(st, sd_, wt, wd, n_ctx, gamma, T, seed, reps=3):
    """Time the CPU oracle (as it stands) on ONE draft+verify step of the same shapes, with the
    caches holding synthetic rows for the n_ctx-token context (filling them by the oracle's own
    prefill would take minutes)."""
    import numpy as np

    import oracle
    from paper_2505_08600_amd import datagen as dg

    threads = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    ot, od = oracle.OracleModel(st, wt), oracle.OracleModel(sd_, wd)
    tseq, dseq = ot.new_seq(n_ctx + 16), od.new_seq(n_ctx + 16)
    for m, seq, shp in ((ot, tseq, st), (od, dseq, sd_)):
        for l in range(shp.n_layers):
            k, v = dg.make_kv_rows(seed, l, 0, n_ctx - 1, shp.n_heads, shp.head_dim, shp.dtype)
            seq.set_kv(l, k, v)
    ctx_t = [int(t) for t in dg.make_prompt(seed, 0, n_ctx, st.vocab)]
    ud = dg.make_uniforms(seed, dg.DRAFT_STREAM, 0, 0, gamma)
    uv = dg.make_uniforms(seed, dg.VERIFY_STREAM, 0, 0, gamma + 1)
    _omp_set_threads(threads)
    td, tv = [], []
    for r in range(reps):   # the same step every time: both caches are rolled back to the context
        t0 = time.perf_counter()
        cand, q, _ = dseq.draft(ctx_t, gamma, T, ud)
        t1 = time.perf_counter()
        tseq.verify(ctx_t, gamma, T, cand, q, uv)
        t2 = time.perf_counter()
        td.append(t1 - t0)
        tv.append(t2 - t1)
        dseq.truncate(n_ctx - 1)
        tseq.truncate(n_ctx - 1)
    step_s = float(np.median(np.array(td) + np.array(tv)))
    out = {"value": gamma / step_s, "unit": "candidate tokens/s", "cores": threads, "kind": "oracle",
           "cpu_model": _cpu_model(), "repetitions": reps,
           "sample": "one draft+verify step (gamma=%d, batch 1) at context %d with synthetic cache rows, %d target "
                     "layers, median of %d repetitions; draft %.2fs, verify %.2fs" %
                     (gamma, n_ctx, st.n_layers, reps, float(np.median(td)), float(np.median(tv)))}
    # one thread: the same step with a 2-layer target of the same widths (all layers would take minutes), beside
    # the same 2-layer step on all threads - the ratio is the oracle's thread scaling
    st2 = dg.with_layers(st, 2)
    w2 = dict(wt)
    for k_ in ("wq", "wk", "wv", "wo", "wgate", "wup", "wdown", "norm_attn", "norm_ffn"):
        w2[k_] = wt[k_][:2]
    o2 = oracle.OracleModel(st2, w2)
    s2 = o2.new_seq(n_ctx + 16)
    for l in range(2):
        k, v = dg.make_kv_rows(seed, l, 0, n_ctx - 1, st.n_heads, st.head_dim, st.dtype)
        s2.set_kv(l, k, v)
    t_l2 = {}
    for nthr in (threads, 1):
        if not _omp_set_threads(nthr):
            break
        t0 = time.perf_counter()
        s2.verify(ctx_t, gamma, T, cand, q, uv)
        t_l2[nthr] = time.perf_counter() - t0
        s2.truncate(n_ctx - 1)
    _omp_set_threads(threads)
    if 1 in t_l2:
        out["one_thread"] = {"sample": "the verify call alone with a 2-layer target of the same widths (LM head included)",
                             "seconds_1_thread": t_l2[1], "seconds_%d_threads" % threads: t_l2[threads],
                             "candidates_per_s_1_thread": gamma / t_l2[1]}
    return out


if __name__ == "__main__":
    main()
