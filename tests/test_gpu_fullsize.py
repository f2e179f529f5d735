"""Full-size parity (BASELINE config 2 shapes) in the launch configuration bench.py times:
7B-shape bf16 target, all 32 layers, context 512, gamma = 5, batch 1, with the 68M-shape draft.

The oracle cannot prefill 511 tokens through 32 layers in reasonable time, so the target's
cache is loaded on both sides with the same synthetic rows (K, V ~ N(0,1), seeded); the
draft's cache comes from a real prefill on both sides.  Needs an MI355X and ~1-2 minutes."""
import time

import numpy as np
import pytest
import torch

import oracle
from paper_2505_08600_amd import api
from paper_2505_08600_amd import datagen as dg

import sdharness as H

pytestmark = pytest.mark.gpu


@pytest.mark.timeout(1500)
def test_config2_full_size_draft_and_verify():
    seed, gamma, n_ctx = 2025, 5, 512
    st_, sd_ = dg.SHAPES["t7b"], dg.SHAPES["draft_a"]
    t0 = time.time()
    wt = dg.make_weights(st_, seed, threads=16)
    wd = dg.make_weights(sd_, seed + 1, threads=16)
    print(f"full-size: weights in {time.time() - t0:.1f}s", flush=True)
    pair = H.Pair(st_, sd_, seed, target_weights=wt, draft_weights=wd, max_rows=16, max_pos=640)
    prompt = [int(t) for t in dg.make_prompt(seed, 0, n_ctx, st_.vocab)]
    tseq, dseq = pair.ot.new_seq(600), pair.od.new_seq(600)
    ctx = api.Context([600])
    ctx.attach(pair.gt)
    ctx.attach(pair.gd)
    ctx.set_tokens([prompt])
    for l in range(st_.n_layers):
        k, v = dg.make_kv_rows(seed, l, 0, n_ctx - 1, st_.n_heads, st_.head_dim, st_.dtype)
        tseq.set_kv(l, k, v)
        ctx.set_kv(pair.gt, l, 0, k, v)
    t0 = time.time()
    oracle.prefill(dseq, prompt)
    api.sd_prefill(pair.gd, ctx, None, 1, n_ctx - 1)
    torch.cuda.synchronize()
    print(f"full-size: caches ready in {time.time() - t0:.1f}s", flush=True)
    t0 = time.time()
    steps, toks = H.oracle_steps(tseq, dseq, prompt, gamma, 1.0, 2, seed)
    print(f"full-size: oracle 2 sampled steps in {time.time() - t0:.1f}s, n_acc={[s.n_acc for s in steps]}", flush=True)
    st = H.lockstep(pair, ctx, steps, gamma, 1.0)
    print(f"full-size T=1: flagged={st.flagged} logit_rel={st.max_logit_rel:.2e} "
          f"q_abs={st.max_q_abs:.2e}", flush=True)
    assert st.max_logit_rel < 2e-2
    steps0, toks = H.oracle_steps(tseq, dseq, toks, gamma, 0.0, 1, seed + 7)
    st0 = H.lockstep(pair, ctx, steps0, gamma, 0.0)
    print(f"full-size T=0: flagged={st0.flagged} logit_rel={st0.max_logit_rel:.2e}", flush=True)
    assert st0.max_logit_rel < 2e-2
    nt, kv = ctx.sync(pair.gt)
    assert nt[0] == len(toks) and kv[0] == len(toks) - 1
    assert list(ctx.get_tokens(0)) == toks
    ctx.close()
    pair.close()


def _batched_case(name, target_shape, draft_shapes, B, lens, gamma, T, seed, check_ids, n_steps=1):
    """A full-size batched step: every sequence runs on the GPU; the oracle recomputes the sequences in
    check_ids one by one (sequences are independent).  The target's cache holds seeded synthetic rows
    (sequence b uses the first len_b - 1 rows of one shared draw); draft caches come from real prefills.
    Unchecked sequences are verified with the GPU drafts' own candidates; checked ones with the oracle's."""
    V = target_shape.vocab
    t0 = time.time()
    wt = dg.make_weights(target_shape, seed, threads=16)
    wds = [dg.make_weights(sh, seed + 1 + i, threads=16) for i, sh in enumerate(draft_shapes)]
    print(f"{name}: weights in {time.time() - t0:.1f}s", flush=True)
    max_len = int(max(lens))
    gt = api.Model(target_shape, wt, max_rows=B * (gamma + 1), max_pos=max_len + 64)
    gds = [api.Model(sh, w, max_rows=16 * B, max_pos=max_len + 64)
           for sh, w in zip(draft_shapes, wds)]
    ot = oracle.OracleModel(target_shape, wt)
    ods = [oracle.OracleModel(sh, w) for sh, w in zip(draft_shapes, wds)]
    nd = len(draft_shapes)
    if nd > 1:
        Wr, br = dg.make_router(seed, nd)
        emb = dg.make_prompt_embeddings(seed, B)
        ids_g = torch.zeros(B, dtype=torch.int32, device="cuda")
        api.sd_route(H.dev(Wr), H.dev(br), H.dev(emb), ids_g)
        route = oracle.route(Wr, br, emb)
        assert np.array_equal(ids_g.cpu().numpy(), route)
    else:
        route = np.zeros(B, np.int32)
    groups = [[b for b in range(B) if route[b] == g] for g in range(nd)]
    prompts = [[int(t) for t in dg.make_prompt(seed, b, int(lens[b]), V)] for b in range(B)]
    ctx = api.Context([int(l) + (n_steps + 1) * (gamma + 1) + 8 for l in lens])
    ctx.attach(gt)
    for gd in gds:
        ctx.attach(gd)
    ctx.set_tokens(prompts)
    t0 = time.time()
    tseqs = {b: ot.new_seq(int(lens[b]) + (n_steps + 1) * (gamma + 1) + 8) for b in check_ids}
    for l in range(target_shape.n_layers):
        k, v = dg.make_kv_rows(seed, l, 0, max_len - 1, target_shape.n_heads, target_shape.head_dim, target_shape.dtype)
        kd, vd = H.dev(k.view(np.int16)), H.dev(v.view(np.int16))  # one upload per layer; rows are bf16 bit patterns
        for b in range(B):
            ctx.set_kv(gt, l, b, kd[:lens[b] - 1], vd[:lens[b] - 1])
        for b in check_ids:
            tseqs[b].set_kv(l, k[:lens[b] - 1], v[:lens[b] - 1])
    print(f"{name}: target caches loaded in {time.time() - t0:.1f}s", flush=True)
    gid = [H.dev(np.array(g, np.int32)) if g else None for g in groups]
    for g in range(nd):
        if groups[g]:
            api.sd_prefill(gds[g], ctx, gid[g], len(groups[g]), max(int(lens[b]) for b in groups[g]) - 1)
    torch.cuda.synchronize()
    t0 = time.time()
    recs = {}
    for b in check_ids:
        dseq = ods[route[b]].new_seq(int(lens[b]) + (n_steps + 1) * (gamma + 1) + 8)
        oracle.prefill(dseq, prompts[b])
        recs[b], _ = H.oracle_steps(tseqs[b], dseq, prompts[b], gamma, T, n_steps, seed, seq=b)
    print(f"{name}: oracle on sequences {list(check_ids)} in {time.time() - t0:.1f}s, "
          f"n_acc={[[s.n_acc for s in recs[b]] for b in check_ids]}", flush=True)
    cand_all = torch.zeros((B, gamma), dtype=torch.int32, device="cuda")
    q_all = torch.zeros((B, gamma, V), dtype=torch.float32, device="cuda") if T > 0 else None
    na = torch.zeros(B, dtype=torch.int32, device="cuda")
    nx = torch.zeros(B, dtype=torch.int32, device="cuda")
    flagged, max_rel = 0, 0.0
    for k in range(n_steps):
        ud_all = np.stack([dg.make_uniforms(seed, dg.DRAFT_STREAM, b, k, gamma) for b in range(B)])
        uv_all = np.stack([dg.make_uniforms(seed, dg.VERIFY_STREAM, b, k, gamma + 1) for b in range(B)])
        for g in range(nd):
            if not groups[g]:
                continue
            ng = len(groups[g])
            cand = torch.zeros((ng, gamma), dtype=torch.int32, device="cuda")
            q = torch.zeros((ng, gamma, V), dtype=torch.float32, device="cuda") if T > 0 else None
            api.sd_draft(gds[g], ctx, gid[g], ng, gamma, T, H.dev(ud_all[groups[g]]) if T > 0 else None, cand, q)
            idx = gid[g].long()
            cand_all[idx] = cand
            if T > 0:
                q_all[idx] = q
            cg = cand.cpu().numpy()
            for j, b in enumerate(groups[g]):
                if b in recs:
                    qg = q[j].cpu().numpy() if T > 0 else None
                    f, first_bad, _ = H.check_draft_step(recs[b][k], cg[j], qg, T, dg.BF16, V)
                    flagged += int(f)
        for b in check_ids:  # checked sequences are verified on the oracle's candidates and q
            cand_all[b] = H.dev(recs[b][k].cand.astype(np.int32))
            if T > 0:
                q_all[b] = H.dev(recs[b][k].q)
        api.sd_verify(gt, ctx, None, B, gamma, T, cand_all, q_all, H.dev(uv_all) if T > 0 else None, na, nx, commit=False)
        torch.cuda.synchronize()
        lg = gt.last_logits().reshape(B, gamma + 1, V)
        assert bool(torch.isfinite(lg).all())
        na_h, nx_h = na.cpu().numpy().copy(), nx.cpu().numpy().copy()
        assert ((na_h >= 0) & (na_h <= gamma) & (nx_h >= 0) & (nx_h < V)).all()
        for b in check_ids:
            f, rel = H.check_verify_step(recs[b][k], int(na_h[b]), int(nx_h[b]), lg[b].cpu().numpy(), T, dg.BF16, V)
            flagged += int(f)
            max_rel = max(max_rel, rel)
            na_h[b], nx_h[b] = recs[b][k].n_acc, recs[b][k].next_token
        api.sd_commit(ctx, None, B, gamma, cand_all, H.dev(na_h), H.dev(nx_h))
        # every sequence advanced by its own n_acc + 1 and rolled its caches back (ragged rollback)
        nt, kv = ctx.sync(gt)
        assert np.array_equal(kv, nt - 1)
    print(f"{name}: flagged={flagged} logit_rel={max_rel:.2e} n_acc(all)={na_h.tolist()}", flush=True)
    assert max_rel < 2e-2
    ctx.close()
    gt.close()
    for gd in gds:
        gd.close()


@pytest.mark.timeout(1500)
def test_config3_full_size_routed_batch32():
    """BASELINE config 3: 7B-shape target, four heterogeneous drafts routed per prompt, 32 prompts with
    lengths uniform in [128, 1024], gamma = 5, T = 0.7; oracle on two sequences."""
    seed, B = 3033, 32
    lens = dg.make_prompt_lengths(seed, B, 128, 1024)
    drafts = [dg.SHAPES[n] for n in ("draft_a", "draft_b", "draft_c", "draft_d")]
    check = [int(np.argmin(lens)), int(np.argsort(lens)[B // 2])]
    _batched_case("config3", dg.SHAPES["t7b"], drafts, B, lens, 5, 0.7, seed, check)


@pytest.mark.timeout(1500)
def test_config4_13b_batch32_context2048():
    """BASELINE config 4: 13B-shape target with the 68M-shape draft, batch 32, context 2048, gamma = 8
    (M = 288 rows), T = 1; oracle on one sequence."""
    seed, B = 4044, 32
    lens = np.full(B, 2048, np.int32)
    _batched_case("config4", dg.SHAPES["t13b"], [dg.SHAPES["draft_a"]], B, lens, 8, 1.0, seed, [5])


@pytest.mark.timeout(1500)
def test_config5_batch64_long_ragged_contexts():
    """BASELINE config 5 shapes: 7B-shape target, batch 64, per-sequence contexts uniform in
    [1024, 8192], gamma = 8 (M = 576 rows), T = 1: long ragged KV (about 150 GB of cache), split
    attention and per-sequence rollback.  Proposals come from the 68M-shape draft here (the synthetic
    rho-mixed q of this config is exercised at full vocabulary in test_gpu_parity); oracle on the
    shortest sequence and on one at the lower eighth of the lengths (the oracle's draft prefill
    grows quadratically with the context; these two keep the test near a minute of CPU work)."""
    seed, B = 5055, 64
    lens = dg.make_prompt_lengths(seed, B, 1024, 8192)
    order = np.argsort(lens)
    _batched_case("config5", dg.SHAPES["t7b"], [dg.SHAPES["draft_a"]], B, lens, 8, 1.0, seed,
                  [int(order[0]), int(order[B // 8])])
