"""Pins for the oracle's decoder forward (CPU only).

The oracle is checked against things that are not itself: a third-party
LLaMA implementation, a library bf16 rounding, invariants of causal decoding and
rotary embeddings, and closed forms of degenerate weight settings.
"""
import dataclasses

import numpy as np
import pytest
import torch

import oracle
from paper_2505_08600_amd import datagen as dg

SMALL = dg.ModelShape("pin_small", 2, 64, 4, 16, 96, 50, dg.FP32)
SMALL_BF16 = dataclasses.replace(SMALL, dtype=dg.BF16, name="pin_small_bf16")


def _hf_llama(shape, w):
    from transformers import LlamaConfig, LlamaForCausalLM

    cfg = LlamaConfig(vocab_size=shape.vocab, hidden_size=shape.d_model, intermediate_size=shape.d_ffn,
                      num_hidden_layers=shape.n_layers, num_attention_heads=shape.n_heads,
                      num_key_value_heads=shape.n_heads, head_dim=shape.head_dim, rms_norm_eps=shape.rms_eps,
                      rope_theta=shape.rope_base, tie_word_embeddings=False, attention_bias=False, mlp_bias=False,
                      max_position_embeddings=512, attn_implementation="eager")
    m = LlamaForCausalLM(cfg).double().eval()
    sd = {"model.embed_tokens.weight": w["embed"], "lm_head.weight": w["lm_head"], "model.norm.weight": w["final_norm"]}
    names = {"wq": "self_attn.q_proj", "wk": "self_attn.k_proj", "wv": "self_attn.v_proj", "wo": "self_attn.o_proj",
             "wgate": "mlp.gate_proj", "wup": "mlp.up_proj", "wdown": "mlp.down_proj",
             "norm_attn": "input_layernorm", "norm_ffn": "post_attention_layernorm"}
    for l in range(shape.n_layers):
        for k, hf in names.items():
            sd[f"model.layers.{l}.{hf}.weight"] = w[k][l]
    sd = {k: torch.from_numpy(np.asarray(v, dtype=np.float64)) for k, v in sd.items()}
    missing, unexpected = m.load_state_dict(sd, strict=False)
    assert not unexpected and all("rotary" in k or "inv_freq" in k for k in missing), (missing, unexpected)
    return m


def test_forward_matches_third_party_llama():
    """Full-model logits against an independent LLaMA implementation in fp64: pins
    block order, weight orientation, RoPE pairing and frequencies, the 1/sqrt(hd)
    scale, causal masking, SwiGLU, RMSNorm eps placement, untied LM head."""
    w = dg.make_weights(SMALL, seed=3, lm_head_scale=5.0)
    # make activations O(1) so that a dropped term cannot hide below the tolerance
    for k in ("wq", "wk", "wv", "wo", "wgate", "wup", "wdown"):
        w[k] = [a * np.float32(8.0) for a in w[k]]
    toks = dg.make_prompt(3, 0, 12, SMALL.vocab)
    hf = _hf_llama(SMALL, w)
    with torch.no_grad():
        ref = hf(torch.from_numpy(toks.astype(np.int64))[None]).logits[0].numpy()
    seq = oracle.OracleModel(SMALL, w).new_seq(32)
    got = np.concatenate([seq.forward(toks[:7]), seq.forward(toks[7:9]), seq.forward(toks[9:])])
    assert got.shape == ref.shape
    assert np.abs(ref).max() > 0.5
    assert np.abs(got - ref).max() < 2e-5 * np.abs(ref).max()


@pytest.mark.parametrize("shape", [SMALL, SMALL_BF16])
def test_multirow_equals_row_by_row(shape):
    """Feeding rows together or one at a time is the same computation (causal
    mask over the new rows, position indexing, cache append)."""
    w = dg.make_weights(shape, seed=5)
    toks = dg.make_prompt(5, 0, 9, shape.vocab)
    m = oracle.OracleModel(shape, w)
    a = m.new_seq(16).forward(toks)
    s = m.new_seq(16)
    b = np.concatenate([s.forward(toks[i:i + 1]) for i in range(len(toks))])
    np.testing.assert_array_equal(a, b)


def test_truncate_then_refeed_is_rollback():
    """KV rollback moves no data: truncating and feeding other tokens equals
    feeding the other tokens after the shorter prefix from scratch."""
    w = dg.make_weights(SMALL, seed=6)
    m = oracle.OracleModel(SMALL, w)
    s = m.new_seq(32)
    s.forward([1, 2, 3, 4, 5, 6])
    s.truncate(3)
    a = s.forward([9, 8])
    b_seq = m.new_seq(32)
    b_seq.forward([1, 2, 3])
    b = b_seq.forward([9, 8])
    np.testing.assert_array_equal(a, b)
    with pytest.raises(ValueError):
        s.truncate(99)


def test_rope_relative_position_and_norm():
    rng = np.random.default_rng(0)
    q, k = rng.standard_normal(64), rng.standard_normal(64)
    d0 = oracle.rope(q, 5, 10000.0) @ oracle.rope(k, 2, 10000.0)
    d1 = oracle.rope(q, 105, 10000.0) @ oracle.rope(k, 102, 10000.0)
    assert abs(d0 - d1) < 1e-9
    assert abs(np.linalg.norm(oracle.rope(q, 77, 10000.0)) - np.linalg.norm(q)) < 1e-12
    np.testing.assert_allclose(oracle.rope(q, 0, 10000.0), q)
    # pair (0, hd/2) rotates by exactly pos radians (frequency base^0 = 1)
    e = np.zeros(64)
    e[0] = 1.0
    r = oracle.rope(e, 1, 10000.0)
    assert abs(r[0] - np.cos(1.0)) < 1e-12 and abs(r[32] - np.sin(1.0)) < 1e-12
    # last pair rotates by pos * base^(-(hd-2)/hd)
    e = np.zeros(64)
    e[31] = 1.0
    r = oracle.rope(e, 3, 10000.0)
    th = 3 * 10000.0 ** (-62.0 / 64.0)
    assert abs(r[31] - np.cos(th)) < 1e-12 and abs(r[63] - np.sin(th)) < 1e-12


def test_rmsnorm_closed_forms():
    g = np.linspace(0.5, 1.5, 8).astype(np.float32)
    out = oracle.rmsnorm(np.full(8, 3.0), g, 1e-5)
    np.testing.assert_allclose(out, g.astype(np.float64) * 3.0 / np.sqrt(9.0 + 1e-5), rtol=1e-12)
    x = np.random.default_rng(1).standard_normal(32)
    out = oracle.rmsnorm(x, np.ones(32, np.float32), 0.0)
    assert abs(np.mean(out ** 2) - 1.0) < 1e-12
    ref = torch.nn.functional.rms_norm(torch.from_numpy(x), (32,), eps=1e-5).numpy()
    np.testing.assert_allclose(oracle.rmsnorm(x, np.ones(32, np.float32), 1e-5), ref, rtol=1e-12)


def test_bf16_rounding_matches_library():
    rng = np.random.default_rng(2)
    xs = np.concatenate([rng.standard_normal(2000).astype(np.float32) * 3,
                         np.array([1.00390625, 1.01171875, -1.00390625, 0.0, 65280.0, 1e-30, 3.3895314e38],
                                  dtype=np.float32)])
    ref = torch.from_numpy(xs).to(torch.bfloat16).to(torch.float32).numpy()
    got = np.array([oracle.round_bf16(float(x)) for x in xs], dtype=np.float32)
    np.testing.assert_array_equal(got, ref)


def test_zero_output_projections_closed_form():
    """With W_o = W_down = 0 the residual stream is the embedding, so the logits are
    lm_head . rmsnorm(embed[token]) computed here in numpy: pins the embedding
    gather, final norm and the [vocab][d_model] orientation of the LM head."""
    w = dg.make_weights(SMALL, seed=7, lm_head_scale=10.0)
    w["wo"] = [np.zeros_like(a) for a in w["wo"]]
    w["wdown"] = [np.zeros_like(a) for a in w["wdown"]]
    toks = [4, 17, 4]
    got = oracle.OracleModel(SMALL, w).new_seq(8).forward(toks)
    for r, t in enumerate(toks):
        e = w["embed"][t].astype(np.float64)
        a = e / np.sqrt(np.mean(e * e) + SMALL.rms_eps) * w["final_norm"]
        a = a.astype(np.float32).astype(np.float64)
        ref = w["lm_head"].astype(np.float64) @ a
        np.testing.assert_allclose(got[r], ref, rtol=1e-5, atol=1e-6)


def test_uniform_attention_is_permutation_invariant():
    """W_q = 0 makes every score 0, so attention is the plain mean of the value
    rows: in a one-layer model the last row's logits cannot depend on the order
    of the earlier tokens."""
    shape = dataclasses.replace(SMALL, n_layers=1)
    w = dg.make_weights(shape, seed=8, lm_head_scale=10.0)
    w["wq"] = [np.zeros_like(a) for a in w["wq"]]
    for k in ("wv", "wo"):
        w[k] = [a * np.float32(20.0) for a in w[k]]
    m = oracle.OracleModel(shape, w)
    a = m.new_seq(8).forward([1, 2, 3, 4, 5])[-1]
    b = m.new_seq(8).forward([4, 1, 3, 2, 5])[-1]
    c = m.new_seq(8).forward([4, 1, 3, 3, 5])[-1]
    np.testing.assert_allclose(a, b, rtol=1e-6, atol=1e-7)
    assert np.abs(a - c).max() > 1e-3  # and it does depend on which tokens they are


def test_bf16_mode_is_fp32_mode_within_rounding():
    """bf16 models differ from the same weights run without activation rounding only
    by accumulated 2^-9 relative roundings."""
    wb = dg.make_weights(SMALL_BF16, seed=9, lm_head_scale=10.0)
    wf = {k: ([dg.bf16_bits_to_f32(a) if a.dtype == np.uint16 else a for a in v] if isinstance(v, list)
              else (dg.bf16_bits_to_f32(v) if v.dtype == np.uint16 else v)) for k, v in wb.items()}
    toks = dg.make_prompt(9, 0, 10, SMALL.vocab)
    lb = oracle.OracleModel(SMALL_BF16, wb).new_seq(16).forward(toks)
    lf = oracle.OracleModel(SMALL, wf).new_seq(16).forward(toks)
    err = np.abs(lb - lf).max() / np.abs(lf).max()
    assert 0 < err < 2e-2


def test_forward_rejects_bad_input():
    m = oracle.OracleModel(SMALL, dg.make_weights(SMALL, seed=1))
    s = m.new_seq(4)
    with pytest.raises(ValueError):
        s.forward([SMALL.vocab])
    with pytest.raises(ValueError):
        s.forward([1, 2, 3, 4, 5])
