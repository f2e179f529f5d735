"""Speculative-decoding loop over the oracle's draft / verify calls (test infrastructure).

State convention (this build's reading; the paper does not discuss caches):
ctx holds tokens x_0..x_{n-1}; the target cache covers positions [0, n-1) and the
last token is pending; the draft cache covers [0, m), m <= n-1.  One step =
draft gamma candidates (Figure 1a), verify them in one target pass (Figure 1b),
emit the accepted prefix plus one token from the target, roll both caches back
to the committed length.
"""
from __future__ import annotations

import dataclasses
from typing import Callable, List, Optional, Sequence

import numpy as np

from .binding import OracleSeq

UniformFn = Callable[[int, int], np.ndarray]  # (step, count) -> fp32 uniforms in [0,1)


@dataclasses.dataclass
class StepRecord:
    n_ctx: int                 # sequence length before the step
    cand: np.ndarray           # [gamma]
    q: Optional[np.ndarray]    # [gamma][V], None when greedy
    u_draft: np.ndarray
    u_verify: np.ndarray
    n_acc: int
    next_token: int
    draft_margins: np.ndarray  # [gamma]
    verify_margins: np.ndarray  # [gamma+1]
    logits: Optional[np.ndarray] = None


def prefill(seq: OracleSeq, ctx: Sequence[int]) -> None:
    """Feed all but the last token (which stays pending)."""
    if len(ctx) > 1:
        seq.forward(list(ctx[:-1]), logits_from=len(ctx) - 1)


def commit(ctx: List[int], target: OracleSeq, draft: Optional[OracleSeq], cand, n_acc: int, nxt: int) -> None:
    """Emit accepted candidates and the target's token; dead cache rows are cut off."""
    ctx.extend(int(c) for c in cand[:n_acc])
    ctx.append(int(nxt))
    target.truncate(len(ctx) - 1)
    if draft is not None:
        draft.truncate(min(draft.len, len(ctx) - 1))


def sd_generate(target: OracleSeq, draft: OracleSeq, prompt: Sequence[int], gamma: int, T: float, n_tokens: int,
                u_draft: UniformFn, u_verify: UniformFn, keep_logits: bool = False):
    """Generate until at least n_tokens are emitted, truncate to n_tokens.
    -> (emitted tokens, [StepRecord])"""
    ctx = [int(t) for t in prompt]
    prefill(target, ctx)
    prefill(draft, ctx)
    steps: List[StepRecord] = []
    step = 0
    while len(ctx) - len(prompt) < n_tokens:
        ud, uv = u_draft(step, gamma), u_verify(step, gamma + 1)
        cand, q, mgd = draft.draft(ctx, gamma, T, ud)
        n0 = len(ctx)
        n_acc, nxt, mgv, lg = target.verify(ctx, gamma, T, cand, q, uv, want_logits=keep_logits)
        commit(ctx, target, draft, cand, n_acc, nxt)
        steps.append(StepRecord(n0, cand, q, ud, uv, n_acc, nxt, mgd, mgv, lg))
        step += 1
    return ctx[len(prompt):len(prompt) + n_tokens], steps


def ar_generate(target: OracleSeq, prompt: Sequence[int], T: float, n_tokens: int, u_verify: UniformFn):
    """Plain autoregressive decoding of the target (the paper's baseline): one
    token per target pass, which is a verify step with gamma = 0."""
    ctx = [int(t) for t in prompt]
    prefill(target, ctx)
    margins = []
    for step in range(n_tokens):
        _, nxt, mg, _ = target.verify(ctx, 0, T, [], None, u_verify(step, 1))
        commit(ctx, target, None, [], 0, nxt)
        margins.append(mg[0])
    return ctx[len(prompt):], margins
