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
    print(f"full-size T=1: flagged={st.flagged} beyond_base={st.beyond_base} logit_rel={st.max_logit_rel:.2e} "
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
