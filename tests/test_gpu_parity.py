"""GPU parity: the HIP draft/verify path against the CPU oracle (needs an MI355X)."""
import dataclasses

import numpy as np
import pytest
import torch

import oracle
from paper_2505_08600_amd import api
from paper_2505_08600_amd import datagen as dg

import sdharness as H

pytestmark = pytest.mark.gpu

TINY_T, TINY_D = dg.SHAPES["tiny_target"], dg.SHAPES["tiny_draft"]


def _say(msg):
    print(msg, flush=True)


@pytest.fixture(scope="module")
def tiny_pair():
    p = H.Pair(TINY_T, TINY_D, seed=11, lm_scale=20.0)
    yield p
    p.close()


@pytest.fixture(scope="module")
def tiny_pair_bf16():
    p = H.Pair(dg.SHAPES["tiny_target_bf16"], dg.SHAPES["tiny_draft_bf16"], seed=12, lm_scale=20.0)
    yield p
    p.close()


@pytest.mark.parametrize("T", [0.0, 1.0])
def test_config1_tiny_fp32_teacher_forced(tiny_pair, T):
    """BASELINE config 1: tiny fp32 pair, gamma=4, prompt 32, 64 tokens."""
    _say(f"config1 fp32 T={T}")
    prompt = dg.make_prompt(11, 0, 32, TINY_T.vocab)
    st = H.teacher_forced_parity(tiny_pair, prompt, gamma=4, T=T, n_tokens=64, seed=11)
    _say(f"  steps={st.steps} flagged={st.flagged} logit_rel={st.max_logit_rel:.2e} q_abs={st.max_q_abs:.2e}")
    assert st.flagged <= 1 and st.max_logit_rel < 1e-4


@pytest.mark.parametrize("T", [0.0, 1.0])
def test_config1_tiny_fp32_free_running(tiny_pair, T):
    """Production loop (commit inside verify, no host reads between calls): emitted
    tokens equal the oracle's up to the oracle's first low-margin decision."""
    _say(f"config1 free-running T={T}")
    prompt = dg.make_prompt(11, 1, 32, TINY_T.vocab)
    toks, steps, _ = H.oracle_trajectory(tiny_pair, prompt, 4, T, 64, seed=21, keep_logits=False)
    got, n_steps, n_acc = H.free_running(tiny_pair, prompt, 4, T, 64, seed=21)
    # fp32 inverse-CDF sums differ from the oracle's fp64 ones by ~1e-7 of the mass; a step whose
    # margin is above 2e-6 cannot legitimately differ
    thr = 2e-6 if T > 0 else H.GREEDY_GAP_THR[dg.FP32]
    safe = 0
    for s in steps:
        if min(s.draft_margins.min(), s.verify_margins.min()) < thr:
            break
        safe += s.n_acc + 1
    safe = min(safe, 64)
    assert safe >= 32, "trajectory hits a low-margin decision too early to be a useful check"
    assert got[:safe] == toks[:safe]
    assert n_acc[:3] == [s.n_acc for s in steps[:3]]


@pytest.mark.parametrize("T", [0.0, 1.0])
def test_perturbed_draft_exercises_partial_acceptance(T):
    """A draft that is a noisy copy of the target accepts 0 < n_acc < gamma often."""
    _say(f"perturbed draft T={T}")
    wt = dg.make_weights(TINY_T, 31, 20.0)
    wd = dg.perturbed_copy(wt, TINY_T, seed=32, rel=0.5)
    pair = H.Pair(TINY_T, TINY_T, 31, target_weights=wt, draft_weights=wd)
    prompt = dg.make_prompt(31, 0, 17, TINY_T.vocab)
    st = H.teacher_forced_parity(pair, prompt, gamma=5, T=T, n_tokens=48, seed=31)
    _say(f"  n_acc={st.n_acc} flagged={st.flagged}")
    assert len(set(st.n_acc)) >= 3 and st.flagged <= 1
    pair.close()


def test_target_as_its_own_draft_accepts_everything():
    """Exercises the two-row catch-up of the draft after fully accepted steps."""
    _say("draft == target")
    wt = dg.make_weights(TINY_T, 41, 20.0)
    pair = H.Pair(TINY_T, TINY_T, 41, target_weights=wt, draft_weights=wt)
    prompt = dg.make_prompt(41, 0, 9, TINY_T.vocab)
    for T in (0.0, 0.8):
        st = H.teacher_forced_parity(pair, prompt, gamma=3, T=T, n_tokens=24, seed=41)
        assert all(a == 3 for a in st.n_acc)
    got, _, n_acc = H.free_running(pair, prompt, 3, 0.0, 24, seed=41)
    ar, _ = oracle.ar_generate(pair.ot.new_seq(64), prompt, 0.0, 24, H.uf(41, dg.VERIFY_STREAM))
    assert got == ar and all(a == 3 for a in n_acc)
    pair.close()


@pytest.mark.parametrize("T", [0.0, 1.0])
def test_tiny_bf16_teacher_forced(tiny_pair_bf16, T):
    _say(f"tiny bf16 T={T}")
    prompt = dg.make_prompt(12, 0, 32, TINY_T.vocab)
    st = H.teacher_forced_parity(tiny_pair_bf16, prompt, gamma=4, T=T, n_tokens=64, seed=12)
    _say(f"  steps={st.steps} flagged={st.flagged} logit_rel={st.max_logit_rel:.2e} q_abs={st.max_q_abs:.2e}")
    assert st.flagged <= max(2, st.steps // 10) and st.max_logit_rel < 2e-2


def test_gamma_zero_is_autoregressive_decoding(tiny_pair):
    _say("gamma = 0")
    prompt = dg.make_prompt(11, 2, 12, TINY_T.vocab)
    ar, _ = oracle.ar_generate(tiny_pair.ot.new_seq(64), prompt, 0.0, 16, H.uf(1, dg.VERIFY_STREAM))
    ctx = api.Context([64])
    ctx.attach(tiny_pair.gt)
    H.gpu_prefill(ctx, [tiny_pair.gt], [list(prompt)])
    na = torch.zeros(1, dtype=torch.int32, device="cuda")
    nx = torch.zeros(1, dtype=torch.int32, device="cuda")
    for _ in range(16):
        api.sd_verify(tiny_pair.gt, ctx, None, 1, 0, 0.0, None, None, None, na, nx, commit=True)
    ctx.sync()
    assert list(ctx.get_tokens(0)[12:]) == ar
    ctx.close()


def test_batched_sequences_with_seq_ids(tiny_pair):
    """Three ragged sequences in one context; calls select subsets through seq_ids.
    Every sequence must behave exactly as it does alone."""
    _say("batched seq_ids")
    gamma, T = 3, 1.0
    prompts = [dg.make_prompt(51, i, n, TINY_T.vocab) for i, n in enumerate((5, 23, 14))]
    trajs = [H.oracle_trajectory(tiny_pair, p, gamma, T, 12, seed=51, seq=i, keep_logits=False)
             for i, p in enumerate(prompts)]
    ctx = api.Context([t[2] for t in trajs])
    ctx.attach(tiny_pair.gt)
    ctx.attach(tiny_pair.gd)
    H.gpu_prefill(ctx, [tiny_pair.gt, tiny_pair.gd], [list(p) for p in prompts])
    V = TINY_T.vocab
    order = [2, 0, 1]                 # rows of the call are a permutation of the context's sequences
    ids = H.dev(np.array(order, np.int32))
    cand = torch.zeros((3, gamma), dtype=torch.int32, device="cuda")
    q = torch.zeros((3, gamma, V), dtype=torch.float32, device="cuda")
    na = torch.zeros(3, dtype=torch.int32, device="cuda")
    nx = torch.zeros(3, dtype=torch.int32, device="cuda")
    n_steps = min(len(t[1]) for t in trajs)
    for k in range(n_steps):
        ud = H.dev(np.stack([trajs[b][1][k].u_draft for b in order]))
        uv = H.dev(np.stack([trajs[b][1][k].u_verify for b in order]))
        api.sd_draft(tiny_pair.gd, ctx, ids, 3, gamma, T, ud, cand, q)
        ref_c = np.stack([trajs[b][1][k].cand for b in order])
        ref_q = np.stack([trajs[b][1][k].q for b in order])
        assert np.array_equal(cand.cpu().numpy(), ref_c), k
        assert np.abs(q.cpu().numpy() - ref_q).max() < 1e-5
        api.sd_verify(tiny_pair.gt, ctx, ids, 3, gamma, T, H.dev(ref_c), H.dev(ref_q), uv, na, nx, commit=True)
        assert list(na.cpu().numpy()) == [trajs[b][1][k].n_acc for b in order], k
        assert list(nx.cpu().numpy()) == [trajs[b][1][k].next_token for b in order], k
    nt, _ = ctx.sync()
    for b in range(3):
        assert nt[b] == len(prompts[b]) + sum(s.n_acc + 1 for s in trajs[b][1][:n_steps])
    ctx.close()


def test_route_matches_oracle():
    W, b = dg.make_router(7)
    e = dg.make_prompt_embeddings(7, 32)
    out = torch.zeros(32, dtype=torch.int32, device="cuda")
    api.sd_route(H.dev(W), H.dev(b), H.dev(e), out)
    ref = oracle.route(W, b, e)
    assert np.array_equal(out.cpu().numpy(), ref) and len(set(ref)) == 4


def test_capacity_and_state_errors_are_reported_not_faulted(tiny_pair):
    _say("error paths")
    ctx = api.Context([16])
    ctx.attach(tiny_pair.gt)
    with pytest.raises(api.SdError) as ei:
        ctx.set_tokens([list(range(100))])
    assert ei.value.code == api.SD_ECAP
    H.gpu_prefill(ctx, [tiny_pair.gt], [list(range(10))])
    na = torch.zeros(1, dtype=torch.int32, device="cuda")
    nx = torch.zeros(1, dtype=torch.int32, device="cuda")
    with pytest.raises(api.SdError) as ei:
        api.sd_verify(tiny_pair.gt, ctx, None, 1, 16, 0.0, na, None, None, na, nx)
    assert ei.value.code == api.SD_ECAP
    with pytest.raises(api.SdError) as ei:
        api.sd_verify(tiny_pair.gd, ctx, None, 1, 2, 0.0, na, None, None, na, nx)  # draft was never attached
    assert ei.value.code == api.SD_EINVAL
    # run the sequence into its capacity: the kernels refuse the rows and raise the flag
    cand = torch.zeros((1, 4), dtype=torch.int32, device="cuda")
    for _ in range(70):
        api.sd_verify(tiny_pair.gt, ctx, None, 1, 4, 0.0, cand, None, None, na, nx, commit=True)
    with pytest.raises(api.SdError) as ei:
        ctx.sync()
    assert ei.value.code == api.SD_ESTATE and "capacity" in str(ei.value)
    nt, _ = ctx.sync()
    assert nt[0] <= 64
    ctx.close()
