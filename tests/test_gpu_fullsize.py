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


class _Rig:
    """The models of one full-size configuration, on both sides (built once, reused over a sweep)."""

    def __init__(self, name, target_shape, draft_shapes, seed, max_rows_t, max_rows_d, max_pos):
        t0 = time.time()
        self.wt = dg.make_weights(target_shape, seed, threads=16)
        self.wds = [dg.make_weights(sh, seed + 1 + i, threads=16) for i, sh in enumerate(draft_shapes)]
        print(f"{name}: weights in {time.time() - t0:.1f}s", flush=True)
        self.gt = api.Model(target_shape, self.wt, max_rows=max_rows_t, max_pos=max_pos)
        self.gds = [api.Model(sh, w, max_rows=max_rows_d, max_pos=max_pos) for sh, w in zip(draft_shapes, self.wds)]
        self.ot = oracle.OracleModel(target_shape, self.wt)
        self.ods = [oracle.OracleModel(sh, w) for sh, w in zip(draft_shapes, self.wds)]

    def close(self):
        self.gt.close()
        for gd in self.gds:
            gd.close()


def _batched_case(name, target_shape, draft_shapes, B, lens, gamma, T, seed, check_ids, n_steps=1, rig=None):
    """A full-size batched step: every sequence runs on the GPU; the oracle recomputes the sequences in
    check_ids one by one (sequences are independent).  The target's cache holds seeded synthetic rows
    (sequence b uses the first len_b - 1 rows of one shared draw); draft caches come from real prefills.
    Unchecked sequences are verified with the GPU drafts' own candidates; checked ones with the oracle's."""
    V = target_shape.vocab
    max_len = int(max(lens))
    own_rig = rig is None
    if own_rig:
        rig = _Rig(name, target_shape, draft_shapes, seed, B * (gamma + 1), 16 * B, max_len + 64)
    gt, gds, ot, ods = rig.gt, rig.gds, rig.ot, rig.ods
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
    assert max_rel < 2e-2 and flagged <= 1
    ctx.close()
    if own_rig:
        rig.close()


@pytest.mark.timeout(1500)
def test_config3_full_size_routed_batch32():
    """BASELINE config 3: 7B-shape target, four heterogeneous drafts routed per prompt, 32 prompts with
    lengths uniform in [128, 1024], gamma = 5, T = 0.7; oracle on two sequences."""
    seed, B = 3033, 32
    lens = dg.make_prompt_lengths(seed, B, 128, 1024)
    drafts = [dg.SHAPES[n] for n in ("draft_a", "draft_b", "draft_c", "draft_d")]
    check = [int(np.argmin(lens)), int(np.argsort(lens)[B // 2])]
    _batched_case("config3", dg.SHAPES["t7b"], drafts, B, lens, 5, 0.7, seed, check)


@pytest.mark.timeout(2400)
def test_config4_13b_batch32_context2048_gamma_sweep():
    """BASELINE config 4: 13B-shape target with the 68M-shape draft, batch 32, context 2048, T = 1, gamma swept over
    3, 5 and 8 (M = 128 rows: the 64-row GEMM blocks; 192; 288); the oracle recomputes one sequence per gamma (a
    different one each time)."""
    seed, B = 4044, 32
    lens = np.full(B, 2048, np.int32)
    shape, drafts = dg.SHAPES["t13b"], [dg.SHAPES["draft_a"]]
    rig = _Rig("config4", shape, drafts, seed, B * 9, 16 * B, 2048 + 64)
    try:
        for gamma, check in ((3, 11), (5, 20), (8, 5)):
            _batched_case(f"config4 gamma={gamma}", shape, drafts, B, lens, gamma, 1.0, seed, [check], rig=rig)
    finally:
        rig.close()


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


class _Config5Rig:
    """7B-shape target with 64 sequences of contexts U[1024, 8192] whose caches hold seeded synthetic rows, on the
    GPU (all sequences) and in the oracle (the longest sequence and a median one)."""

    def __init__(self):
        self.seed, self.B, self.gamma, self.T = 5055, 64, 8, 1.0
        seed, B, gamma = self.seed, self.B, self.gamma
        self.shape = shape = dg.SHAPES["t7b"]
        V = shape.vocab
        self.lens = lens = dg.make_prompt_lengths(seed, B, 1024, 8192)
        order = np.argsort(lens)
        self.check_ids = [int(order[-1]), int(order[B // 2])]
        t0 = time.time()
        wt = dg.make_weights(shape, seed, threads=16)
        self.gt = api.Model(shape, wt, max_rows=B * (gamma + 1), max_pos=int(lens.max()) + 64)
        self.ot = oracle.OracleModel(shape, wt)
        self.prompts = [[int(t) for t in dg.make_prompt(seed, b, int(lens[b]), V)] for b in range(B)]
        self.ctx = api.Context([int(l) + 2 * (gamma + 1) + 8 for l in lens])
        self.ctx.attach(self.gt)
        self.ctx.set_tokens(self.prompts)
        self.tseqs = {b: self.ot.new_seq(int(lens[b]) + 2 * (gamma + 1) + 8) for b in self.check_ids}
        max_len = int(lens.max())
        for l in range(shape.n_layers):
            k, v = dg.make_kv_rows(seed, l, 0, max_len - 1, shape.n_heads, shape.head_dim, shape.dtype)
            kd, vd = H.dev(k.view(np.int16)), H.dev(v.view(np.int16))
            for b in range(B):
                self.ctx.set_kv(self.gt, l, b, kd[:lens[b] - 1], vd[:lens[b] - 1])
            for b in self.check_ids:
                self.tseqs[b].set_kv(l, k[:lens[b] - 1], v[:lens[b] - 1])
        gen = torch.Generator(device="cuda").manual_seed(seed)
        self.q_all = torch.softmax(4.0 * torch.randn((B, gamma, V), device="cuda", generator=gen), dim=-1).contiguous()
        self.cand_all = torch.multinomial(self.q_all.reshape(B * gamma, V), 1, generator=gen).reshape(B, gamma) \
            .to(torch.int32).contiguous()
        self.n_acc_seen = {}
        print(f"config5 synthetic q: sequences {self.check_ids} (contexts {[int(lens[b]) for b in self.check_ids]}), "
              f"weights and caches in {time.time() - t0:.1f}s", flush=True)

    def close(self):
        self.ctx.close()
        self.gt.close()


@pytest.fixture(scope="module")
def config5_rig():
    rig = _Config5Rig()
    yield rig
    rig.close()


@pytest.mark.timeout(1500)
@pytest.mark.parametrize("rho", [0.0, 0.5, 0.9])
def test_config5_synthetic_q_long_contexts(config5_rig, rho):
    """BASELINE config 5 as stated: 7B-shape target, batch 64, contexts uniform in [1024, 8192], gamma = 8, T = 1, and
    NO draft model: the proposal distributions are synthetic, q_i = softmax(rho * target logits_i + (1 - rho) * 4 *
    N(0,1)), candidates drawn from q by inverse CDF.  The target cache holds seeded synthetic rows on both sides.
    For a median-length sequence (every rho) and the LONGEST one (rho = 0.5) the oracle builds q and the candidates
    position by position (one single-row target forward per position, then the cache is rolled back) and runs the
    verify; the GPU verifies all 64 sequences in one call (the other sequences carry rho = 0 proposals made on the
    device) and must reproduce the oracle's logits (2e-2) and decisions (flat 1e-3 rule) on the checked ones."""
    R = config5_rig
    seed, B, gamma, T, lens, V = R.seed, R.B, R.gamma, R.T, R.lens, R.shape.vocab
    tag = int(rho * 10)
    checked = R.check_ids if rho == 0.5 else R.check_ids[1:]
    recs = {}
    t0 = time.time()
    for b in checked:
        n0, seq = int(lens[b]), R.tseqs[b]
        ud = dg.make_uniforms(seed, dg.DRAFT_STREAM, b, tag, gamma)
        uv = dg.make_uniforms(seed, dg.VERIFY_STREAM, b, tag, gamma + 1)
        cand, q = [], np.zeros((gamma, V), np.float32)
        fed = [R.prompts[b][-1]]
        for i in range(gamma):   # position i: logits of the row fed last, given everything fed before
            lg_i = seq.forward([fed[-1]])[0]
            z = rho * lg_i + (1.0 - rho) * 4.0 * dg.make_logit_noise(seed, b, 100 * tag + i, V)
            q[i] = oracle.softmax_T(z.astype(np.float32), T)
            cand.append(oracle.sample_cdf(q[i].astype(np.float64), float(ud[i]))[0])
            fed.append(cand[-1])
        seq.truncate(n0 - 1)   # roll back: the verify feeds the same rows again in one pass
        r_na, r_nx, mg, lg = seq.verify(R.prompts[b], gamma, T, cand, q, uv, want_logits=True)
        seq.truncate(n0 - 1)
        recs[b] = oracle.StepRecord(n0, np.array(cand, np.int32), q, ud, uv, r_na, r_nx, np.zeros(gamma), mg, lg)
        R.cand_all[b] = H.dev(np.array(cand, np.int32))
        R.q_all[b] = H.dev(q)
    uv_all = np.stack([dg.make_uniforms(seed, dg.VERIFY_STREAM, b, tag, gamma + 1) for b in range(B)])
    print(f"config5 rho={rho}: oracle built q and verified {checked} in {time.time() - t0:.1f}s, "
          f"n_acc={[recs[b].n_acc for b in checked]}", flush=True)
    na = torch.zeros(B, dtype=torch.int32, device="cuda")
    nx = torch.zeros(B, dtype=torch.int32, device="cuda")
    api.sd_verify(R.gt, R.ctx, None, B, gamma, T, R.cand_all, R.q_all, H.dev(uv_all), na, nx, commit=False)
    torch.cuda.synchronize()
    lg_g = R.gt.last_logits().reshape(B, gamma + 1, V)
    assert bool(torch.isfinite(lg_g).all())
    na_h, nx_h = na.cpu().numpy(), nx.cpu().numpy()
    assert ((na_h >= 0) & (na_h <= gamma) & (nx_h >= 0) & (nx_h < V)).all()
    for b in range(B):   # nothing was committed: roll every cache length back for the next case
        R.ctx.truncate(R.gt, b, int(lens[b]) - 1)
    R.ctx.sync()
    flagged = 0
    for b in checked:
        f, rel = H.check_verify_step(recs[b], int(na_h[b]), int(nx_h[b]), lg_g[b].cpu().numpy(), T, dg.BF16, V)
        flagged += int(f)
        R.n_acc_seen[(b, rho)] = recs[b].n_acc
        print(f"  seq {b} (context {int(lens[b])}): gpu ({int(na_h[b])},{int(nx_h[b])}) oracle ({recs[b].n_acc},"
              f"{recs[b].next_token}) logit_rel={rel:.2e} flagged={f}", flush=True)
        assert rel < 2e-2
    assert flagged <= 1
    if rho == 0.9:   # sharing more of the target's logits must not lower the median sequence's acceptance
        med = R.check_ids[1]
        if (med, 0.0) in R.n_acc_seen:
            assert R.n_acc_seen[(med, 0.9)] >= R.n_acc_seen[(med, 0.0)]


@pytest.mark.timeout(900)
@pytest.mark.parametrize("max_rows,n_ctx", [(576, 600), (1024, 1300)])
def test_prefill_at_full_width_matches_oracle_and_the_split_kernels(max_rows, n_ctx):
    """The prefill path at the 7B shape's widths in two of the configurations bench.py --prefill-bench times (576-row
    workspace: 36 row groups of one prompt per forward, nine blocks of four groups per head, tile ranges split
    over blocks with the combine pass; 1024-row workspace: 64 groups, the GEMMs in 64-row blocks, a full forward
    followed by a partial one), cut to two layers so that the oracle can prefill the same prompt:
    the verify pass that follows must give the oracle's logits.  The same prefill through the decode path's
    split kernel per group (prefill_attn = 0) agrees to rounding level, and with the cache append one block per
    row (rope_group = 0) bit for bit."""
    seed, gamma = 2031, 5
    st_ = dg.with_layers(dg.SHAPES["t7b"], 2)
    wt = dg.make_weights(st_, seed, threads=16)
    om = oracle.OracleModel(st_, wt)
    gm = api.Model(st_, wt, max_rows=max_rows, max_pos=n_ctx + 64)
    V = st_.vocab
    prompt = [int(t) for t in dg.make_prompt(seed, 0, n_ctx, V)]
    cand = dg.make_prompt(seed + 1, 0, gamma, V).astype(np.int32)
    t0 = time.time()
    seq = om.new_seq(n_ctx + 16)
    oracle.prefill(seq, prompt)
    r_na, r_nx, mg, r_lg = seq.verify(prompt, gamma, 0.0, cand, None, np.zeros(gamma + 1, np.float32), want_logits=True)
    print(f"full-width prefill: oracle prefill + verify in {time.time() - t0:.1f}s", flush=True)
    outs = {}
    for name, opts in (("default", {}), ("split kernel per group", {"prefill_attn": 0}), ("append per row", {"rope_group": 0})):
        for k, v in opts.items():
            api.set_option(k, v)
        try:
            ctx = api.Context([n_ctx + 16])
            ctx.attach(gm)
            H.gpu_prefill(ctx, [gm], [prompt])
            na = torch.zeros(1, dtype=torch.int32, device="cuda")
            nx = torch.zeros(1, dtype=torch.int32, device="cuda")
            api.sd_verify(gm, ctx, None, 1, gamma, 0.0, H.dev(cand[None]), None, None, na, nx, commit=False)
            ctx.sync()
            outs[name] = gm.last_logits().cpu().numpy()
            ctx.close()
        finally:
            for k in opts:
                api.set_option(k, 1)
    rel = np.abs(outs["default"] - r_lg).max() / np.abs(r_lg).max()
    rel_split = np.abs(outs["default"] - outs["split kernel per group"]).max() / np.abs(r_lg).max()
    print(f"full-width prefill: logits vs oracle {rel:.2e}, vs split kernel per group {rel_split:.2e}", flush=True)
    assert rel < 2e-2 and rel_split < 5e-4
    assert np.array_equal(outs["default"], outs["append per row"])
    gm.close()
