"""Prompt classifier of Sections 2.4 and 3.3.3, written out in fp64 (test infrastructure).

Test infrastructure only: nothing in the product path imports this file.  It shares no
code with the HIP kernels; both sides read the same seeded weights and prompts.

The paper names the layers (embedding, one Mamba sequence layer, adaptive pooling, a fully
connected layer) and nothing else, so the layer itself follows the published selective
state-space block it cites.  With u the embedded prompt [L][d_model]:

    (x, z) = u W_in                                  two halves of width d_inner
    x_t    = SiLU(b_conv + sum_j w_conv[:, j] x_{t - (d_conv-1) + j})     causal, zero history
    (r_t, B_t, C_t) = x_t W_x                        widths dt_rank, d_state, d_state
    Delta_t = softplus(r_t W_dt + b_dt)              one step size per channel
    h_t    = exp(Delta_t A) * h_{t-1} + Delta_t B_t x_t,   A = -exp(A_log),  h_{-1} = 0
    y_t    = (C_t . h_t + D x_t) * SiLU(z_t)
    o_t    = y_t W_out

Readings where the paper is silent: no normalisation and no residual around the layer;
"adaptive pooling" is the average over the prompt's tokens (output length one); the label is
the arg max of the fully connected layer's output, the lowest index on ties; an empty
prompt pools to zero, so its logits are the bias.
"""
from __future__ import annotations

from typing import Dict

import numpy as np


def softplus(x):
    """log(1 + e^x)."""
    return np.logaddexp(0.0, x)


def silu(x):
    """x * sigmoid(x)."""
    return x / (1.0 + np.exp(-x))


def mamba_layer(w: Dict[str, np.ndarray], u: np.ndarray) -> Dict[str, np.ndarray]:
    """The sequence layer on one prompt; u is [L][d_model].  Returns every intermediate
    (x after the convolution and SiLU, Delta, B, C, the gated y, and the output o)."""
    f = {k: np.asarray(v, dtype=np.float64) for k, v in w.items()}
    u = np.asarray(u, dtype=np.float64)
    L = u.shape[0]
    d_inner, d_conv = f["conv_w"].shape
    d_state = f["a_log"].shape[1]
    dt_rank = f["w_dt"].shape[0]

    xz = u @ f["w_in"]
    x_in, z = xz[:, :d_inner], xz[:, d_inner:]

    x = np.zeros((L, d_inner))
    for t in range(L):
        acc = f["conv_b"].copy()
        for j in range(d_conv):
            s = t - (d_conv - 1) + j
            if s >= 0:
                acc += f["conv_w"][:, j] * x_in[s]
        x[t] = silu(acc)

    proj = x @ f["w_x"]
    r = proj[:, :dt_rank]
    B = proj[:, dt_rank:dt_rank + d_state]
    C = proj[:, dt_rank + d_state:]
    delta = softplus(r @ f["w_dt"] + f["b_dt"])

    A = -np.exp(f["a_log"])
    h = np.zeros((d_inner, d_state))
    y = np.zeros((L, d_inner))
    for t in range(L):
        decay = np.exp(delta[t][:, None] * A)
        h = decay * h + (delta[t] * x[t])[:, None] * B[t][None, :]
        y[t] = (h @ C[t] + f["d"] * x[t]) * silu(z[t])

    return {"x": x, "z": z, "delta": delta, "B": B, "C": C, "y": y, "o": y @ f["w_out"]}


def classify(w: Dict[str, np.ndarray], tokens) -> tuple:
    """Logits [n_classes] and label of one prompt given as token ids."""
    tokens = np.asarray(tokens, dtype=np.int64)
    d_model = w["emb"].shape[1]
    if tokens.size:
        u = np.asarray(w["emb"], dtype=np.float64)[tokens]
        pooled = mamba_layer(w, u)["o"].mean(axis=0)
    else:
        pooled = np.zeros(d_model)
    logits = np.asarray(w["w_fc"], dtype=np.float64) @ pooled + np.asarray(w["b_fc"], dtype=np.float64)
    return logits, int(np.argmax(logits))
