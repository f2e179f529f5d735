"""Pins of the classifier oracle (Sections 2.4, 3.3.3) against things other than itself:
the unrolled solution of the state recurrence, library filters for the time-invariant
special case, one- and two-token prompts worked by hand, causality, and the pooling and
output layer's behaviour under a permutation of the classes, an empty prompt and ties."""
import dataclasses

import numpy as np
import pytest
from scipy.signal import lfilter
from scipy.special import expit

from oracle import mamba
from paper_2505_08600_amd import datagen as dg

TINY = dg.CLASSIFIER_TINY


def _weights(shape=TINY, seed=3):
    return {k: v.astype(np.float64) for k, v in dg.make_classifier(shape, seed).items()}


def _prompt(shape, seed, length):
    return dg.make_prompt(seed, 0, length, shape.vocab)


def test_scan_equals_the_unrolled_sum_with_cumulative_step_sizes():
    """h_t = sum_{s<=t} exp(A (S_t - S_s)) Delta_s B_s x_s with S the running sum of Delta:
    the recurrence solved in closed form, evaluated without any running state."""
    w = _weights()
    u = w["emb"][_prompt(TINY, 1, 11)]
    r = mamba.mamba_layer(w, u)
    A = -np.exp(w["a_log"])
    S = np.cumsum(r["delta"], axis=0)
    L = u.shape[0]
    for t in range(L):
        acc = np.zeros(TINY.d_inner)
        for s in range(t + 1):
            kernel = np.exp(A * (S[t] - S[s])[:, None])          # [d_inner][d_state]
            acc += (kernel * r["B"][s][None, :]) @ r["C"][t] * r["delta"][s] * r["x"][s]
        want = (acc + w["d"] * r["x"][t]) * mamba.silu(r["z"][t])
        np.testing.assert_allclose(r["y"][t], want, rtol=1e-11, atol=1e-13)


def test_time_invariant_case_reduces_to_library_filters():
    """With W_dt = 0 the step size is the constant softplus(b_dt), so each channel is a
    first-order IIR filter: the whole layer is matmuls, np.convolve and scipy's lfilter.
    B and C enter asymmetrically here (B scales the filter's input, C its output)."""
    shape = dataclasses.replace(TINY, d_state=1)
    w = _weights(shape, 5)
    w["w_dt"][:] = 0.0
    u = w["emb"][_prompt(shape, 2, 17)]
    L = u.shape[0]
    r = mamba.mamba_layer(w, u)

    xz = u @ w["w_in"]
    x_in, z = xz[:, :shape.d_inner], xz[:, shape.d_inner:]
    x = np.empty_like(x_in)
    for c in range(shape.d_inner):
        x[:, c] = np.convolve(x_in[:, c], w["conv_w"][c][::-1])[:L] + w["conv_b"][c]
    x = x / (1.0 + np.exp(-x))
    np.testing.assert_allclose(r["x"], x, rtol=1e-12, atol=1e-14)

    proj = x @ w["w_x"]
    B, C = proj[:, shape.dt_rank], proj[:, shape.dt_rank + 1]
    delta = np.logaddexp(0.0, w["b_dt"])
    np.testing.assert_allclose(r["delta"], np.broadcast_to(delta, (L, shape.d_inner)), rtol=1e-13)
    a = np.exp(-delta * np.exp(w["a_log"][:, 0]))
    y = np.empty_like(x)
    for c in range(shape.d_inner):
        h = lfilter([1.0], [1.0, -a[c]], delta[c] * B * x[:, c])
        y[:, c] = (C * h + w["d"][c] * x[:, c]) * (z[:, c] / (1.0 + np.exp(-z[:, c])))
    np.testing.assert_allclose(r["y"], y, rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(r["o"], y @ w["w_out"], rtol=1e-11, atol=1e-13)
    # the asymmetry is real: exchanging the two columns changes the output
    w2 = dict(w)
    w2["w_x"] = w["w_x"][:, [0, 1, 2, 4, 3]]
    assert np.abs(mamba.mamba_layer(w2, u)["y"] - r["y"]).max() > 1e-6


def test_two_token_prompt_by_hand():
    """Scalars only: every sum of the definition written as a loop for L = 2."""
    s = TINY
    w = _weights(s, 7)
    tok = _prompt(s, 3, 2)
    logits, label = mamba.classify(w, tok)

    sig = lambda v: 1.0 / (1.0 + np.exp(-v))
    xin = [[sum(w["emb"][tok[t]][k] * w["w_in"][k][c] for k in range(s.d_model)) for c in range(2 * s.d_inner)]
           for t in range(2)]
    x = [[0.0] * s.d_inner for _ in range(2)]
    for c in range(s.d_inner):
        pre0 = w["conv_b"][c] + w["conv_w"][c][s.d_conv - 1] * xin[0][c]
        pre1 = w["conv_b"][c] + w["conv_w"][c][s.d_conv - 1] * xin[1][c] + w["conv_w"][c][s.d_conv - 2] * xin[0][c]
        x[0][c], x[1][c] = pre0 * sig(pre0), pre1 * sig(pre1)
    J = s.dt_rank + 2 * s.d_state
    proj = [[sum(x[t][c] * w["w_x"][c][j] for c in range(s.d_inner)) for j in range(J)] for t in range(2)]
    o = [[0.0] * s.d_model for _ in range(2)]
    y = [[0.0] * s.d_inner for _ in range(2)]
    for c in range(s.d_inner):
        dl = [np.log1p(np.exp(w["b_dt"][c] + sum(proj[t][i] * w["w_dt"][i][c] for i in range(s.dt_rank))))
              for t in range(2)]
        acc0 = acc1 = 0.0
        for n in range(s.d_state):
            a = -np.exp(w["a_log"][c][n])
            b0, b1 = proj[0][s.dt_rank + n], proj[1][s.dt_rank + n]
            c0, c1 = proj[0][s.dt_rank + s.d_state + n], proj[1][s.dt_rank + s.d_state + n]
            h0 = dl[0] * b0 * x[0][c]
            h1 = np.exp(dl[1] * a) * h0 + dl[1] * b1 * x[1][c]
            acc0 += c0 * h0
            acc1 += c1 * h1
        for t, acc in ((0, acc0), (1, acc1)):
            zt = xin[t][s.d_inner + c]
            y[t][c] = (acc + w["d"][c] * x[t][c]) * zt * sig(zt)
    for t in range(2):
        for m in range(s.d_model):
            o[t][m] = sum(y[t][c] * w["w_out"][c][m] for c in range(s.d_inner))
    want = [w["b_fc"][k] + sum(w["w_fc"][k][m] * 0.5 * (o[0][m] + o[1][m]) for m in range(s.d_model))
            for k in range(s.n_classes)]
    np.testing.assert_allclose(logits, want, rtol=1e-11, atol=1e-13)
    assert label == int(np.argmax(want))


def test_layer_is_causal_and_prefix_consistent():
    w = _weights()
    tok = _prompt(TINY, 4, 13)
    full = mamba.mamba_layer(w, w["emb"][tok])["o"]
    for k in (1, 2, 5, 12):
        np.testing.assert_allclose(mamba.mamba_layer(w, w["emb"][tok[:k]])["o"], full[:k], rtol=1e-12, atol=1e-14)
    other = tok.copy()
    other[9] = (other[9] + 1) % TINY.vocab
    changed = mamba.mamba_layer(w, w["emb"][other])["o"]
    np.testing.assert_array_equal(changed[:9], full[:9])
    assert np.abs(changed[9:] - full[9:]).min(axis=1).max() > 0 and np.abs(changed[9] - full[9]).max() > 1e-9


def test_state_carries_information_beyond_the_convolution_window():
    """A token further back than d_conv still moves the output (through h only)."""
    w = _weights()
    tok = _prompt(TINY, 5, 12)
    other = tok.copy()
    other[0] = (other[0] + 1) % TINY.vocab
    a = mamba.mamba_layer(w, w["emb"][tok])["o"][11]
    b = mamba.mamba_layer(w, w["emb"][other])["o"][11]
    assert np.abs(a - b).max() > 1e-9
    # and with the state switched off (B = 0) it does not
    w0 = dict(w)
    w0["w_x"] = w["w_x"].copy()
    w0["w_x"][:, TINY.dt_rank:TINY.dt_rank + TINY.d_state] = 0.0
    a = mamba.mamba_layer(w0, w0["emb"][tok])["o"][11]
    b = mamba.mamba_layer(w0, w0["emb"][other])["o"][11]
    np.testing.assert_array_equal(a, b)


def test_pooling_is_the_mean_over_tokens_and_labels_follow_the_logits():
    w = _weights()
    tok = _prompt(TINY, 6, 9)
    logits, label = mamba.classify(w, tok)
    o = mamba.mamba_layer(w, w["emb"][tok])["o"]
    # linear output layer: logits - bias is additive over tokens, each weighted 1/L
    per_token = np.stack([w["w_fc"] @ o[t] for t in range(9)])
    np.testing.assert_allclose(logits - w["b_fc"], per_token.sum(axis=0) / 9, rtol=1e-12, atol=1e-14)
    assert label == int(np.argmax(logits))
    # permuting the classes permutes logits and relabels
    perm = np.array([2, 0, 1])
    wp = dict(w)
    wp["w_fc"], wp["b_fc"] = w["w_fc"][perm], w["b_fc"][perm]
    lp, labp = mamba.classify(wp, tok)
    np.testing.assert_allclose(lp, logits[perm], rtol=1e-13)
    assert perm[labp] == label
    # an empty prompt pools to zero
    le, labe = mamba.classify(w, [])
    np.testing.assert_array_equal(le, w["b_fc"])
    assert labe == int(np.argmax(w["b_fc"]))
    # ties go to the lowest index
    wt = dict(w)
    wt["w_fc"] = np.zeros_like(w["w_fc"])
    wt["b_fc"] = np.array([0.5, 0.5, 0.25])
    assert mamba.classify(wt, tok)[1] == 0


def test_activation_helpers_against_library_forms():
    v = np.linspace(-40, 40, 161)
    np.testing.assert_allclose(mamba.softplus(v), np.where(v > 30, v, np.log1p(np.exp(np.minimum(v, 30)))),
                               rtol=1e-12)
    np.testing.assert_allclose(mamba.silu(v), v * expit(v), rtol=1e-12, atol=1e-300)


@pytest.mark.parametrize("field,axis", [("conv_w", 1), ("w_dt", 0)])
def test_unused_history_and_rank_slots_do_not_matter(field, axis):
    """Widening the convolution with zero taps at the far end, or the step-size projection
    with zero rows, leaves the result unchanged: the index conventions are as stated."""
    w = _weights()
    tok = _prompt(TINY, 8, 10)
    base = mamba.classify(w, tok)[0]
    w2 = dict(w)
    if field == "conv_w":
        w2["conv_w"] = np.concatenate([np.zeros((TINY.d_inner, 2)), w["conv_w"]], axis=1)   # older taps
    else:
        w2["w_dt"] = np.concatenate([w["w_dt"], np.zeros((2, TINY.d_inner))], axis=0)
        wx = w["w_x"]
        w2["w_x"] = np.concatenate([wx[:, :TINY.dt_rank], np.ones((TINY.d_inner, 2)), wx[:, TINY.dt_rank:]], axis=1)
    np.testing.assert_allclose(mamba.classify(w2, tok)[0], base, rtol=1e-12, atol=1e-14)


# ---- planted mistakes: each plausible slip in the layer must be caught by at least one pin above

_PINS = [test_scan_equals_the_unrolled_sum_with_cumulative_step_sizes,
         test_time_invariant_case_reduces_to_library_filters,
         test_two_token_prompt_by_hand,
         test_layer_is_causal_and_prefix_consistent,
         test_state_carries_information_beyond_the_convolution_window,
         test_pooling_is_the_mean_over_tokens_and_labels_follow_the_logits]

_MISTAKES = {
    "convolution taps in reverse order": ('f["conv_w"][:, j] * x_in[s]', 'f["conv_w"][:, d_conv - 1 - j] * x_in[s]'),
    "convolution looks ahead": ("s = t - (d_conv - 1) + j", "s = t + j"),
    "convolution bias dropped": ('acc = f["conv_b"].copy()', 'acc = np.zeros_like(f["conv_b"])'),
    "B and C exchanged": ("B = proj[:, dt_rank:dt_rank + d_state]\n    C = proj[:, dt_rank + d_state:]",
                          "C = proj[:, dt_rank:dt_rank + d_state]\n    B = proj[:, dt_rank + d_state:]"),
    "step size without its bias": ('softplus(r @ f["w_dt"] + f["b_dt"])', 'softplus(r @ f["w_dt"])'),
    "exp instead of softplus": ('delta = softplus(r @ f["w_dt"] + f["b_dt"])', 'delta = np.exp(r @ f["w_dt"] + f["b_dt"])'),
    "growing instead of decaying state": ('A = -np.exp(f["a_log"])', 'A = np.exp(f["a_log"])'),
    "A used without the exponential": ('A = -np.exp(f["a_log"])', 'A = -f["a_log"]'),
    "input not scaled by the step size": ("(delta[t] * x[t])[:, None] * B[t][None, :]", "x[t][:, None] * B[t][None, :]"),
    "state read before it is updated": ("h = decay * h + (delta[t] * x[t])[:, None] * B[t][None, :]\n        y[t] = (h @ C[t]",
                                        "y[t] = (h @ C[t]"),
    "skip term dropped": ('(h @ C[t] + f["d"] * x[t])', "(h @ C[t])"),
    "gate without SiLU": ("* silu(z[t])", "* z[t]"),
    "gate and input halves exchanged": ("x_in, z = xz[:, :d_inner], xz[:, d_inner:]", "z, x_in = xz[:, :d_inner], xz[:, d_inner:]"),
    "decay applied to the new input as well":
        ("h = decay * h + (delta[t] * x[t])[:, None] * B[t][None, :]", "h = decay * (h + (delta[t] * x[t])[:, None] * B[t][None, :])"),
}


@pytest.mark.parametrize("name", sorted(_MISTAKES))
def test_planted_mistake_is_caught(name, monkeypatch):
    import inspect
    old, new = _MISTAKES[name]
    src = inspect.getsource(mamba.mamba_layer)
    assert src.count(old) == 1, f"the oracle no longer contains the text this mistake replaces: {old!r}"
    scope = dict(vars(mamba))
    exec(src.replace(old, new), scope)
    broken = scope["mamba_layer"]
    u = np.asarray(_weights()["emb"][_prompt(TINY, 1, 9)])
    try:
        changed = not np.allclose(broken(_weights(), u)["o"], mamba.mamba_layer(_weights(), u)["o"], rtol=1e-9, atol=1e-12)
    except IndexError:      # e.g. a convolution that reads past the end of the prompt
        return
    assert changed, "this edit does not change the result on the test input"
    monkeypatch.setattr(mamba, "mamba_layer", broken)
    caught = []
    for pin in _PINS:
        try:
            pin()
        except (AssertionError, IndexError):
            caught.append(pin.__name__)
    assert caught, f"no pin notices: {name}"
