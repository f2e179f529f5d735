"""Shared helpers of the GPU parity tests: run the oracle's trajectory first, then
teacher-force the HIP path along it step by step.

Parity bar: candidate ids, n_accepted and next tokens bit-exact; a step may be
*flagged* instead only when the ORACLE's own decision margin is below a fixed
threshold.  Logits: max |gpu - oracle| / max |oracle| per row below the dtype's
tolerance.  No expected value ever comes from the HIP path: after every step the
HIP context is committed with the ORACLE's result.

The flag rule is flat: nothing measured on the HIP side widens it.
  - accept test (T > 0):  flagged only if |u - p/q| < 1e-3 (bf16) or 1e-5 (fp32);
  - inverse-CDF draw:     the HIP token is valid only if u lies within that same
                          threshold (as a fraction of the total mass) of the token's
                          interval of the oracle's CDF - judged in CDF space because
                          with 32000 tokens almost every u is within 1e-3 of *some* edge;
  - greedy:               the argmax may differ only if the oracle's top-1/top-2 gap,
                          relative to the row's largest |logit|, is below the threshold;
  - draft q rows:         |q_gpu - q_oracle| <= the threshold, element-wise.
A decision that differs with a larger margin is a failure, whatever the logits did.
"""
from __future__ import annotations

import dataclasses
from typing import List, Optional

import numpy as np
import torch

import oracle
from paper_2505_08600_amd import api
from paper_2505_08600_amd import datagen as dg

LOGIT_TOL = {dg.FP32: 1e-4, dg.BF16: 2e-2}     # max relative error of a logits row
MARGIN_THR = {dg.FP32: 1e-5, dg.BF16: 1e-3}    # probability-space decision margins
# greedy draft candidates: the draft's logits are not read back, so the oracle's top-1/top-2 gap is judged in
# absolute logit units (the test models' logits are O(1..10))
GREEDY_GAP_THR = {dg.FP32: 1e-4, dg.BF16: 1e-2}


def flag_cap(steps: int) -> int:
    """How many steps of a run may be flagged (measured: 0-4 in 1453 steps of the random-shape sweep)."""
    return max(1, steps // 50)


@dataclasses.dataclass
class ParityStats:
    steps: int = 0
    flagged: int = 0
    max_logit_rel: float = 0.0
    max_q_abs: float = 0.0
    n_acc: List[int] = dataclasses.field(default_factory=list)

    def merge_logits(self, gpu: np.ndarray, ref: np.ndarray):
        rel = float(np.max(np.abs(gpu.astype(np.float64) - ref) / np.max(np.abs(ref), axis=-1, keepdims=True)))
        self.max_logit_rel = max(self.max_logit_rel, rel)
        return rel


def uf(seed, stream, seq=0):
    return lambda step, n: dg.make_uniforms(seed, stream, seq, step, n)


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.cuda()


class Pair:
    """Target + draft, the same weights loaded into the oracle and into libsd."""

    def __init__(self, shape_t, shape_d, seed, lm_scale=1.0, draft_weights=None, target_weights=None,
                 max_rows=32, max_pos=256):
        self.shape_t, self.shape_d = shape_t, shape_d
        self.wt = target_weights if target_weights is not None else dg.make_weights(shape_t, seed, lm_scale)
        self.wd = draft_weights if draft_weights is not None else dg.make_weights(shape_d, seed + 1, lm_scale)
        self.ot = oracle.OracleModel(shape_t, self.wt)
        self.od = oracle.OracleModel(shape_d, self.wd)
        self.gt = api.Model(shape_t, self.wt, max_rows=max_rows, max_pos=max_pos)
        self.gd = api.Model(shape_d, self.wd, max_rows=max_rows, max_pos=max_pos)

    def close(self):
        self.gt.close()
        self.gd.close()


def oracle_trajectory(pair: Pair, prompt, gamma, T, n_tokens, seed, seq=0, keep_logits=True):
    cap = len(prompt) + n_tokens + 2 * gamma + 4
    toks, steps = oracle.sd_generate(pair.ot.new_seq(cap), pair.od.new_seq(cap), prompt, gamma, T, n_tokens,
                                     uf(seed, dg.DRAFT_STREAM, seq), uf(seed, dg.VERIFY_STREAM, seq),
                                     keep_logits=keep_logits)
    return toks, steps, cap


def gpu_prefill(ctx: api.Context, models, prompts, seq_ids=None):
    ctx.set_tokens(prompts, seq_ids)
    n = len(prompts)
    ids = dev(np.asarray(seq_ids, np.int32)) if seq_ids is not None else None
    mx = max(len(p) for p in prompts) - 1
    for m in models:
        api.sd_prefill(m, ctx, ids, n, mx)
    torch.cuda.synchronize()


def teacher_forced_parity(pair: Pair, prompt, gamma, T, n_tokens, seed) -> ParityStats:
    """One sequence: HIP draft and verify are compared with the oracle at every step
    of the oracle's own trajectory."""
    dtype = pair.shape_t.dtype
    thr = MARGIN_THR[dtype]
    toks, steps, cap = oracle_trajectory(pair, prompt, gamma, T, n_tokens, seed, keep_logits=True)
    V = pair.shape_t.vocab
    ctx = api.Context([cap])
    ctx.attach(pair.gt)
    ctx.attach(pair.gd)
    gpu_prefill(ctx, [pair.gt, pair.gd], [list(prompt)])
    st = lockstep(pair, ctx, steps, gamma, T)
    nt, kv = ctx.sync(pair.gt)
    n_expected = len(prompt) + sum(s.n_acc + 1 for s in steps)
    assert nt[0] == n_expected and kv[0] == n_expected - 1
    got = ctx.get_tokens(0)
    ref_all = list(prompt)
    for s in steps:
        ref_all += [int(c) for c in s.cand[:s.n_acc]] + [s.next_token]
    assert list(got) == ref_all
    ctx.close()
    return st


def oracle_steps(tseq, dseq, ctx_tokens, gamma, T, n_steps, seed, seq=0):
    """n_steps draft/verify/commit steps of the oracle from the caches' current state.
    -> (records, tokens after the last step)"""
    ctx_t = [int(t) for t in ctx_tokens]
    out = []
    for k in range(n_steps):
        ud = dg.make_uniforms(seed, dg.DRAFT_STREAM, seq, k, gamma)
        uv = dg.make_uniforms(seed, dg.VERIFY_STREAM, seq, k, gamma + 1)
        cand, q, mgd = dseq.draft(ctx_t, gamma, T, ud)
        n0 = len(ctx_t)
        na, nx, mgv, lg = tseq.verify(ctx_t, gamma, T, cand, q, uv, want_logits=True)
        oracle.loop.commit(ctx_t, tseq, dseq, cand, na, nx)
        out.append(oracle.StepRecord(n0, cand, q, ud, uv, na, nx, mgd, mgv, lg))
    return out, ctx_t


def check_draft_step(s, cg, qg, T, dtype, V):
    """Compare one sequence's HIP draft output (cand cg [gamma], q qg [gamma][V] or None) with the
    oracle's step record.  -> (flagged, first differing candidate index or None, max |dq|)"""
    thr = MARGIN_THR[dtype]
    gamma = len(s.cand)
    first_bad = None
    for i in range(gamma):
        if cg[i] != s.cand[i]:
            first_bad = i
            break
    if first_bad is not None:
        if T > 0:  # valid iff u is within the threshold of the HIP token's interval of the oracle's CDF
            mg = oracle.cdf_distance(s.q[first_bad], s.u_draft[first_bad], int(cg[first_bad])) \
                if 0 <= cg[first_bad] < V else 1.0
            lim = thr
        else:
            mg, lim = s.draft_margins[first_bad], GREEDY_GAP_THR[dtype]
        assert mg < lim, f"draft candidate {first_bad} differs ({cg} vs {s.cand}), margin {mg} lim {lim}"
    dq = 0.0
    if T > 0:
        upto = gamma if first_bad is None else first_bad + 1
        dq = float(np.abs(qg[:upto] - s.q[:upto]).max())
        assert dq <= thr, f"draft q differs by {dq}"
    return first_bad is not None, first_bad, dq


def check_verify_step(s, na, nx, lg, T, dtype, V):
    """Compare one sequence's HIP verify output (n_acc, next token, logits [gamma+1][V]) with the
    oracle's step record.  -> (flagged, logits rel err)"""
    thr = MARGIN_THR[dtype]
    gamma = len(s.cand)
    ref = s.logits.astype(np.float64)
    rel = float(np.max(np.abs(lg.astype(np.float64) - ref) / np.max(np.abs(ref), axis=-1, keepdims=True)))
    assert rel <= LOGIT_TOL[dtype], f"logits rel err {rel}"
    if (na, nx) == (s.n_acc, s.next_token):
        return False, rel
    if na != s.n_acc:      # the accept test (or argmax match) at the first differing position
        i = min(s.n_acc, na)
        mg = float(s.verify_margins[i])
        lim = thr if T > 0 else thr * float(np.abs(ref[i]).max())
    elif T > 0:            # same prefix, other next token
        w = oracle.next_weights(s.logits, s.q, s.n_acc, T)
        mg = oracle.cdf_distance(w, s.u_verify[gamma], nx) if 0 <= nx < V else 1.0
        lim = thr
    else:
        mg, lim = float(s.verify_margins[gamma]), thr * float(np.abs(ref[s.n_acc]).max())
    assert mg < lim, (f"verify differs: gpu ({na},{nx}) oracle ({s.n_acc},{s.next_token}), "
                      f"margin {mg} lim {lim}")
    return True, rel


def lockstep(pair: Pair, ctx: api.Context, steps, gamma, T) -> ParityStats:
    """Run the HIP draft and verify of sequence 0 along the oracle's recorded steps and
    compare every output; commits the oracle's result after each step."""
    dtype = pair.shape_t.dtype
    V = pair.shape_t.vocab
    st = ParityStats()
    cand_g = torch.zeros((1, gamma), dtype=torch.int32, device="cuda")
    q_g = torch.zeros((1, gamma, V), dtype=torch.float32, device="cuda") if T > 0 else None
    nacc_g = torch.zeros(1, dtype=torch.int32, device="cuda")
    next_g = torch.zeros(1, dtype=torch.int32, device="cuda")
    for k, s in enumerate(steps):
        # ---- draft (Figure 1a)
        ud = dev(s.u_draft[None]) if T > 0 else None
        api.sd_draft(pair.gd, ctx, None, 1, gamma, T, ud, cand_g, q_g)
        cg = cand_g.cpu().numpy()[0]
        qg = q_g.cpu().numpy()[0] if T > 0 else None
        try:
            f1, first_bad, dq = check_draft_step(s, cg, qg, T, dtype, V)
        except AssertionError as e:
            raise AssertionError(f"step {k}: {e}") from None
        st.max_q_abs = max(st.max_q_abs, dq)
        # ---- verify (Figure 1b) on the ORACLE's candidates and q
        cand_in = dev(s.cand[None].astype(np.int32))
        q_in = dev(s.q[None]) if T > 0 else None
        uv = dev(s.u_verify[None]) if T > 0 else None
        api.sd_verify(pair.gt, ctx, None, 1, gamma, T, cand_in, q_in, uv, nacc_g, next_g, commit=False)
        na, nx = int(nacc_g.item()), int(next_g.item())
        lg = pair.gt.last_logits().cpu().numpy()
        try:
            f2, rel = check_verify_step(s, na, nx, lg, T, dtype, V)
        except AssertionError as e:
            raise AssertionError(f"step {k}: {e}") from None
        st.max_logit_rel = max(st.max_logit_rel, rel)
        # ---- commit the oracle's result (teacher forcing)
        api.sd_commit(ctx, None, 1, gamma, cand_in, dev(np.array([s.n_acc], np.int32)),
                      dev(np.array([s.next_token], np.int32)))
        if first_bad is not None:  # the draft cache holds rows of other candidates: roll back and re-feed
            torch.cuda.synchronize()
            ctx.truncate(pair.gd, 0, s.n_ctx - 1 + first_bad)
            api.sd_prefill(pair.gd, ctx, None, 1, gamma + 2)
        st.steps += 1
        st.flagged += int(f1 or f2)
        st.n_acc.append(s.n_acc)
    torch.cuda.synchronize()
    return st


def free_running(pair: Pair, prompt, gamma, T, n_tokens, seed):
    """The production loop: draft -> verify(commit) with no host reads in between.
    -> (gpu tokens, n_steps)"""
    cap = len(prompt) + n_tokens + 2 * gamma + 4
    V = pair.shape_t.vocab
    ctx = api.Context([cap])
    ctx.attach(pair.gt)
    ctx.attach(pair.gd)
    gpu_prefill(ctx, [pair.gt, pair.gd], [list(prompt)])
    cand_g = torch.zeros((1, gamma), dtype=torch.int32, device="cuda")
    q_g = torch.zeros((1, gamma, V), dtype=torch.float32, device="cuda") if T > 0 else None
    nacc_g = torch.zeros(1, dtype=torch.int32, device="cuda")
    next_g = torch.zeros(1, dtype=torch.int32, device="cuda")
    max_steps = n_tokens
    uds = [dev(dg.make_uniforms(seed, dg.DRAFT_STREAM, 0, k, gamma)[None]) for k in range(max_steps)]
    uvs = [dev(dg.make_uniforms(seed, dg.VERIFY_STREAM, 0, k, gamma + 1)[None]) for k in range(max_steps)]
    n_acc_log = []
    steps = 0
    while True:
        api.sd_draft(pair.gd, ctx, None, 1, gamma, T, uds[steps] if T > 0 else None, cand_g, q_g)
        api.sd_verify(pair.gt, ctx, None, 1, gamma, T, cand_g, q_g, uvs[steps] if T > 0 else None, nacc_g, next_g,
                      commit=True)
        steps += 1
        n_acc_log.append(nacc_g.clone())
        if steps % 8 == 0 or steps >= max_steps:
            nt, _ = ctx.sync()
            if nt[0] - len(prompt) >= n_tokens or steps >= max_steps:
                break
    toks = ctx.get_tokens(0)[len(prompt):len(prompt) + n_tokens]
    ctx.close()
    return [int(t) for t in toks], steps, [int(t.item()) for t in n_acc_log]


def batched_teacher_forced(gt, gd, ot, od, prompts, gamma, T, n_tok, seed, dtype, adapters=None):
    """A ragged batch through ONE draft model and the target: every sequence's oracle trajectory is
    computed on its own (with its adapter, if any); the HIP path drafts all sequences in one call and
    verifies them in one call, step by step along those trajectories.  -> (steps, flagged)"""
    B = len(prompts)
    V = gt.shape.vocab
    trajs = []
    for b in range(B):
        cap = len(prompts[b]) + n_tok + 2 * gamma + 4
        dseq = od.new_seq(cap, adapters[b]) if adapters is not None else od.new_seq(cap)
        _, steps = oracle.sd_generate(ot.new_seq(cap), dseq, prompts[b], gamma, T, n_tok,
                                      uf(seed, dg.DRAFT_STREAM, b), uf(seed, dg.VERIFY_STREAM, b), keep_logits=True)
        trajs.append(steps)
    n_steps = min(len(t) for t in trajs)
    ctx = api.Context([len(p) + (n_steps + 1) * (gamma + 1) + 8 for p in prompts])
    ctx.attach(gt)
    ctx.attach(gd)
    if adapters is not None:
        ctx.set_adapters(gd, adapters)
    gpu_prefill(ctx, [gt, gd], prompts)
    na = torch.zeros(B, dtype=torch.int32, device="cuda")
    nx = torch.zeros(B, dtype=torch.int32, device="cuda")
    cand = torch.zeros((B, gamma), dtype=torch.int32, device="cuda")
    q = torch.zeros((B, gamma, V), dtype=torch.float32, device="cuda") if T > 0 else None
    flagged = 0
    for k in range(n_steps):
        ud = dev(np.stack([trajs[b][k].u_draft for b in range(B)])) if T > 0 else None
        api.sd_draft(gd, ctx, None, B, gamma, T, ud, cand, q)
        cg = cand.cpu().numpy()
        qg = q.cpu().numpy() if T > 0 else None
        refeed = []
        for b in range(B):
            f, first_bad, _ = check_draft_step(trajs[b][k], cg[b], qg[b] if T > 0 else None, T, dtype, V)
            flagged += int(f)
            if first_bad is not None:
                refeed.append((b, trajs[b][k].n_ctx - 1 + first_bad))
        cand_all = dev(np.stack([trajs[b][k].cand for b in range(B)]).astype(np.int32))
        q_all = dev(np.stack([trajs[b][k].q for b in range(B)])) if T > 0 else None
        uv = dev(np.stack([trajs[b][k].u_verify for b in range(B)])) if T > 0 else None
        api.sd_verify(gt, ctx, None, B, gamma, T, cand_all, q_all, uv, na, nx, commit=False)
        lg = gt.last_logits().cpu().numpy().reshape(B, gamma + 1, V)
        na_h, nx_h = na.cpu().numpy(), nx.cpu().numpy()
        for b in range(B):
            f, _ = check_verify_step(trajs[b][k], int(na_h[b]), int(nx_h[b]), lg[b], T, dtype, V)
            flagged += int(f)
        api.sd_commit(ctx, None, B, gamma, cand_all, dev(np.array([trajs[b][k].n_acc for b in range(B)], np.int32)),
                      dev(np.array([trajs[b][k].next_token for b in range(B)], np.int32)))
        for b, keep in refeed:   # that draft cache holds rows of other candidates: roll back and re-feed
            torch.cuda.synchronize()
            ctx.truncate(gd, b, keep)
            api.sd_prefill(gd, ctx, dev(np.array([b], np.int32)), 1, gamma + 2)
    nt, kv = ctx.sync(gt)
    for b in range(B):
        assert nt[b] == len(prompts[b]) + sum(s.n_acc + 1 for s in trajs[b][:n_steps]) and kv[b] == nt[b] - 1
    ctx.close()
    return n_steps, flagged

