"""Pins for the oracle's bf16 numeric contract, its synthetic-cache loader and its adapters with bf16 factors
(CPU only).

The decoder block (Section 3.1: LLaMA target and draft) is written out here a second time, in numpy float64,
with a LIBRARY bf16 cast (torch) at every point where the contract rounds:
  normed hidden, rotated query, attention output, SwiGLU product, final norm  -> two bf16 terms hi + lo
  rotated key, value (the cache)                                              -> one bf16 value
Nothing else is rounded; logits leave as fp32.  The oracle must reproduce that to fp32 output rounding, so a
forgotten rounding site, a dropped lo term or a cache row stored too wide shows up here.
"""
import dataclasses

import numpy as np
import pytest
import torch

import oracle
from paper_2505_08600_amd import datagen as dg

ONE = dg.ModelShape("pin_bf16_1l", 1, 64, 4, 16, 96, 50, dg.BF16)
TWO = dataclasses.replace(ONE, n_layers=2, name="pin_bf16_2l")


def _bf(x):
    """fp32 -> bf16 -> fp32 by the library's cast."""
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(torch.bfloat16).to(torch.float32).numpy()


def _act(x, bf16=True):
    """Activation entering a contraction: hi + lo, hi = bf16(x), lo = bf16(x - hi) (x as fp32)."""
    f = np.asarray(x, dtype=np.float64).astype(np.float32)
    if not bf16:
        return f.astype(np.float64)
    hi = _bf(f)
    lo = _bf(f - hi)
    return hi.astype(np.float64) + lo.astype(np.float64)


def _store(x, bf16=True):
    f = np.asarray(x, dtype=np.float64).astype(np.float32)
    return (_bf(f) if bf16 else f).astype(np.float64)


def _w64(a):
    return (dg.bf16_bits_to_f32(a) if a.dtype == np.uint16 else a).astype(np.float64)


def _rmsnorm(x, g, eps):
    return x / np.sqrt(np.mean(x * x) + eps) * g.astype(np.float64)


def _rope(x, H, hd, pos, base):
    x = x.reshape(H, hd).copy()
    half = hd // 2
    i = np.arange(half)
    ang = pos * base ** (-2.0 * i / hd)
    c, s = np.cos(ang), np.sin(ang)
    a, b = x[:, :half].copy(), x[:, half:].copy()
    x[:, :half] = a * c - b * s
    x[:, half:] = b * c + a * s
    return x.reshape(-1)


class NumpyLlama:
    """The block with explicit rounding points.  Weights as float64 matrices (so merged adapter weights, which
    are not bf16 values, can be used too); the cache as lists of [H*hd] rows per layer."""

    def __init__(self, shape, w, bf16=True):
        self.s, self.bf16 = shape, bf16
        self.w = {k: ([_w64(a) for a in v] if isinstance(v, list) else _w64(v)) for k, v in w.items()}
        self.K = [[] for _ in range(shape.n_layers)]
        self.V = [[] for _ in range(shape.n_layers)]

    def forward(self, tokens):
        s, w, bf16 = self.s, self.w, self.bf16
        H, hd = s.n_heads, s.head_dim
        out = []
        for tok in tokens:
            pos = len(self.K[0])
            h = w["embed"][tok].copy()
            for l in range(s.n_layers):
                a = _act(_rmsnorm(h, w["norm_attn"][l], s.rms_eps), bf16)
                q = _act(_rope(w["wq"][l] @ a, H, hd, pos, s.rope_base), bf16)
                self.K[l].append(_store(_rope(w["wk"][l] @ a, H, hd, pos, s.rope_base), bf16))
                self.V[l].append(_store(w["wv"][l] @ a, bf16))
                Kc = np.stack(self.K[l]).reshape(-1, H, hd)
                Vc = np.stack(self.V[l]).reshape(-1, H, hd)
                o = np.empty(H * hd)
                for hh in range(H):
                    sc = Kc[:, hh] @ q[hh * hd:(hh + 1) * hd] / np.sqrt(hd)
                    p = np.exp(sc - sc.max())
                    o[hh * hd:(hh + 1) * hd] = (p / p.sum()) @ Vc[:, hh]
                o = _act(o, bf16)
                h = h + w["wo"][l] @ o
                f = _act(_rmsnorm(h, w["norm_ffn"][l], s.rms_eps), bf16)
                g = w["wgate"][l] @ f
                t = _act(g / (1.0 + np.exp(-g)) * (w["wup"][l] @ f), bf16)
                h = h + w["wdown"][l] @ t
            a = _act(_rmsnorm(h, w["final_norm"], s.rms_eps), bf16)
            out.append((w["lm_head"] @ a).astype(np.float32))
        return np.stack(out)


def _weights(shape, seed):
    """O(1) activations and attention that is far from uniform, so that every rounding site matters."""
    w = dg.make_weights(shape, seed=seed, lm_head_scale=5.0)
    for k in ("wq", "wk", "wv", "wo", "wgate", "wup", "wdown"):
        w[k] = [dg.f32_to_bf16_bits(dg.bf16_bits_to_f32(a) * np.float32(8.0)) for a in w[k]]
    return w


def _close(got, ref):
    """Equal up to the rounding of the fp32 logits (fp64 sums in another order move a value by ~1e-15)."""
    return np.abs(got.astype(np.float64) - ref).max() <= 2.0 ** -22 * np.abs(ref).max()


@pytest.mark.parametrize("shape", [ONE, TWO])
def test_bf16_rounding_points_match_library_casts(shape):
    w = _weights(shape, 21)
    toks = [int(t) for t in dg.make_prompt(21, 0, 7, shape.vocab)]
    ref = NumpyLlama(shape, w).forward(toks)
    got = oracle.OracleModel(shape, w).new_seq(16).forward(toks)
    assert np.abs(ref).max() > 0.5
    assert _close(got, ref), np.abs(got - ref).max() / np.abs(ref).max()


def test_every_rounding_site_matters_in_this_pin():
    """The pin's resolution: leaving out any one of the contract's roundings in the numpy model moves the
    logits by far more than the tolerance above, so the comparison would notice the same slip in the oracle."""
    w = _weights(ONE, 21)
    toks = [int(t) for t in dg.make_prompt(21, 0, 7, ONE.vocab)]
    ref = NumpyLlama(ONE, w).forward(toks)
    unrounded = NumpyLlama(ONE, w, bf16=False).forward(toks)
    assert np.abs(unrounded - ref).max() > 2.0 ** -18 * np.abs(ref).max()


def test_the_numpy_model_is_the_fp32_oracle_without_roundings():
    """The second implementation itself: with roundings off it is the fp32 oracle (pinned elsewhere against a
    third-party LLaMA) on the same weights."""
    shape = dataclasses.replace(TWO, dtype=dg.FP32, name="pin_f32_2l")
    wb = _weights(TWO, 22)
    wf = {k: ([dg.bf16_bits_to_f32(a) if a.dtype == np.uint16 else a for a in v] if isinstance(v, list)
              else (dg.bf16_bits_to_f32(v) if v.dtype == np.uint16 else v)) for k, v in wb.items()}
    toks = [int(t) for t in dg.make_prompt(22, 0, 6, shape.vocab)]
    ref = NumpyLlama(shape, wf, bf16=False).forward(toks)
    got = oracle.OracleModel(shape, wf).new_seq(16).forward(toks)
    assert np.abs(got - ref).max() < 1e-5 * np.abs(ref).max()


@pytest.mark.parametrize("shape", [ONE, dataclasses.replace(ONE, dtype=dg.FP32, name="pin_f32_1l")])
def test_set_kv_loads_rows_as_token_head_dim(shape):
    """Synthetic cache rows [len][n_heads][head_dim] loaded with set_kv must act exactly like rows a forward
    wrote.  The rows come from the numpy model (not from the oracle), the continuation from both."""
    wb = _weights(ONE, 23)
    w = wb if shape.dtype == dg.BF16 else {
        k: ([dg.bf16_bits_to_f32(a) if a.dtype == np.uint16 else a for a in v] if isinstance(v, list)
            else (dg.bf16_bits_to_f32(v) if v.dtype == np.uint16 else v)) for k, v in wb.items()}
    bf16 = shape.dtype == dg.BF16
    toks = [int(t) for t in dg.make_prompt(23, 0, 9, shape.vocab)]
    ref_model = NumpyLlama(shape, w, bf16=bf16)
    ref_model.forward(toks[:6])
    k_rows = np.stack(ref_model.K[0]).reshape(6, shape.n_heads, shape.head_dim).astype(np.float32)
    v_rows = np.stack(ref_model.V[0]).reshape(6, shape.n_heads, shape.head_dim).astype(np.float32)
    ref = ref_model.forward(toks[6:])
    seq = oracle.OracleModel(shape, w).new_seq(16)
    if bf16:
        seq.set_kv(0, dg.f32_to_bf16_bits(k_rows), dg.f32_to_bf16_bits(v_rows))   # exact: the rows are bf16 values
    else:
        seq.set_kv(0, k_rows, v_rows)
    assert seq.len == 6
    got = seq.forward(toks[6:])
    tol = 2.0 ** -22 if bf16 else 1e-5
    assert np.abs(got - ref).max() <= tol * np.abs(ref).max()
    # and a straight run of the oracle agrees with the loaded one
    straight = oracle.OracleModel(shape, w).new_seq(16)
    straight.forward(toks[:6])
    assert np.abs(straight.forward(toks[6:]) - got).max() <= tol * np.abs(ref).max()
    # a loader that exchanged heads and tokens would not get past this: swapping the axes changes the logits
    seq2 = oracle.OracleModel(shape, w).new_seq(16)
    k_t = np.ascontiguousarray(k_rows.reshape(6, -1).T).reshape(-1)[:k_rows.size].reshape(k_rows.shape)
    seq2.set_kv(0, dg.f32_to_bf16_bits(k_t) if bf16 else k_t, dg.f32_to_bf16_bits(v_rows) if bf16 else v_rows)
    assert np.abs(seq2.forward(toks[6:]) - ref).max() > 1e-3 * np.abs(ref).max()


def test_set_kv_validates_and_sets_length():
    w = _weights(ONE, 23)
    seq = oracle.OracleModel(ONE, w).new_seq(4)
    k, v = dg.make_kv_rows(1, 0, 0, 5, ONE.n_heads, ONE.head_dim, dg.BF16)
    with pytest.raises(ValueError):
        seq.set_kv(0, k, v)          # longer than the capacity
    with pytest.raises(ValueError):
        seq.set_kv(1, k[:2], v[:2])  # no such layer
    seq.set_kv(0, k[:3], v[:3])
    assert seq.len == 3


def test_adapters_with_bf16_factors_equal_merged_weights():
    """y = W x + s B (A x) with bf16 A, B: the adapter path must equal the numpy model run on the merged
    float64 matrices W + s B A (which are not bf16 values - only the second implementation can take them)."""
    shape = TWO
    w = _weights(shape, 24)
    lora = dg.make_lora(shape, 25, n_adapters=3, rank=4, std_a=0.5, std_b=0.5)
    scale = 1.5
    toks = [int(t) for t in dg.make_prompt(24, 0, 6, shape.vocab)]
    m = oracle.OracleModel(shape, w)
    m.set_lora(lora, scale)
    base = oracle.OracleModel(shape, w).new_seq(16).forward(toks)
    for a in (0, 2):
        wm = {k: ([_w64(x) for x in v] if isinstance(v, list) else _w64(v)) for k, v in w.items()}
        for pnm, key in (("q", "wq"), ("k", "wk"), ("v", "wv"), ("o", "wo")):
            wm[key] = [wm[key][l] + scale * _w64(lora["b_" + pnm][l][a]) @ _w64(lora["a_" + pnm][l][a])
                       for l in range(shape.n_layers)]
        ref = NumpyLlama(shape, wm).forward(toks)
        got = m.new_seq(16, a).forward(toks)
        assert _close(got, ref), (a, np.abs(got - ref).max() / np.abs(ref).max())
        assert np.abs(got - base).max() > 1e-2 * np.abs(base).max()
