"""Pins for the oracle's low-rank adapters (Section 2.3: drafts are LoRA fine-tunes of one base model):
against merged weights built with numpy, and against the base model (CPU only)."""
import copy

import numpy as np
import pytest

import oracle
from paper_2505_08600_amd import datagen as dg

TINY = dg.SHAPES["tiny_draft"]   # fp32


def _logits(model, prompt, adapter=-1):
    seq = model.new_seq(64, adapter)
    return seq.forward(prompt)


def test_adapter_equals_the_model_with_merged_weights():
    """y = W x + s B (A x) = (W + s B A) x: an fp32 model with adapter a must give the logits of the plain
    model whose q, k, v, o matrices were merged in float64 and rounded to fp32 (the rounding of the merged
    weights bounds the difference), for every adapter; and a different adapter must give different logits."""
    w = dg.make_weights(TINY, 11, lm_head_scale=20.0)
    lora = dg.make_lora(TINY, 12, n_adapters=3, rank=4, std_a=0.05, std_b=0.05)
    scale = 2.0
    m = oracle.OracleModel(TINY, w)
    m.set_lora(lora, scale)
    prompt = [int(t) for t in dg.make_prompt(13, 0, 9, TINY.vocab)]
    base = _logits(oracle.OracleModel(TINY, w), prompt)
    outs = []
    for a in range(3):
        wm = copy.copy(w)
        for pnm, key in (("q", "wq"), ("k", "wk"), ("v", "wv"), ("o", "wo")):
            wm[key] = [(w[key][l].astype(np.float64) + scale * lora["b_" + pnm][l][a].astype(np.float64)
                        @ lora["a_" + pnm][l][a].astype(np.float64)).astype(np.float32) for l in range(TINY.n_layers)]
        merged = _logits(oracle.OracleModel(TINY, wm), prompt)
        got = _logits(m, prompt, a)
        assert np.abs(got - merged).max() < 2e-5 * np.abs(merged).max()
        assert np.abs(got - base).max() > 1e-3 * np.abs(base).max()
        outs.append(got)
    assert np.abs(outs[0] - outs[1]).max() > 1e-3 * np.abs(outs[0]).max()


def test_no_adapter_and_zero_update_are_the_base_model():
    w = dg.make_weights(TINY, 11, lm_head_scale=20.0)
    prompt = [int(t) for t in dg.make_prompt(13, 1, 7, TINY.vocab)]
    base = _logits(oracle.OracleModel(TINY, w), prompt)
    lora = dg.make_lora(TINY, 12, n_adapters=2, rank=4)
    m = oracle.OracleModel(TINY, w)
    m.set_lora(lora, 1.0)
    assert np.array_equal(_logits(m, prompt, -1), base)          # sequence without an adapter
    zero = dict(lora)
    for pnm in dg.LORA_PROJ:
        zero["b_" + pnm] = [np.zeros_like(b) for b in lora["b_" + pnm]]
    m0 = oracle.OracleModel(TINY, w)
    m0.set_lora(zero, 1.0)
    assert np.array_equal(_logits(m0, prompt, 1), base)          # B = 0: the update vanishes
    m1 = oracle.OracleModel(TINY, w)
    m1.set_lora(lora, 0.0)
    assert np.array_equal(_logits(m1, prompt, 0), base)          # scale = 0
    with pytest.raises(ValueError):
        m.new_seq(16, 2)                                          # adapter id out of range


def test_only_the_listed_projections_are_adapted():
    """An adapter given for q alone changes the logits; the same factors handed to no projection do not."""
    w = dg.make_weights(TINY, 11, lm_head_scale=20.0)
    lora = dg.make_lora(TINY, 12, n_adapters=1, rank=2, std_a=0.1, std_b=0.1)
    prompt = [int(t) for t in dg.make_prompt(13, 2, 6, TINY.vocab)]
    base = _logits(oracle.OracleModel(TINY, w), prompt)
    only_q = {k: v for k, v in lora.items() if k in ("n_adapters", "rank", "a_q", "b_q")}
    mq = oracle.OracleModel(TINY, w)
    mq.set_lora(only_q, 1.0)
    assert np.abs(_logits(mq, prompt, 0) - base).max() > 1e-4 * np.abs(base).max()
    none = {"n_adapters": 1, "rank": 2}
    mn = oracle.OracleModel(TINY, w)
    mn.set_lora(none, 1.0)
    assert np.array_equal(_logits(mn, prompt, 0), base)
