"""fp64 oracle: vanilla tanh RNN, sequential back-propagation.  TEST INFRASTRUCTURE.

Model (Section 4.1, the RNN equation): h_t = tanh(W_ih x_t + b + W_hh h_{t-1}),
h_0 = 0, t = 1..T (x is stored 0-based: x[t-1] feeds h_t).  The paper's two
biases are folded into b = b_ih + b_hh (their gradients coincide).  The head is
softmax cross-entropy on a linear map of the last hidden state, mean over the
batch.

Backward: Eq. 3 of Section 2.1 applied step by step as a vector-Jacobian
product (the transposed Jacobian is never formed in `backward_chain`), then
Eq. 2 summed over the steps because the parameters are shared.

Pins (tests/test_oracle_rnn.py): central finite differences of the loss with
respect to every parameter and to injected perturbations of hidden states;
`step_jacobian_T` against finite differences of a single step and against the
vector-Jacobian product of `backward_chain`.
"""
from __future__ import annotations

import numpy as np


def _f64(a):
    return np.asarray(a, dtype=np.float64)


def forward(x, w_ih, w_hh, b, h0=None, start=0, inject=None):
    """Hidden states h[0..T] of shape [T+1, B, H].

    `start`/`h0` let the recurrence restart from step `start` with state h0
    (used by finite differences on a hidden state).
    """
    x, w_ih, w_hh, b = _f64(x), _f64(w_ih), _f64(w_hh), _f64(b)
    T, B, _ = x.shape
    H = w_hh.shape[0]
    h = np.zeros((T + 1, B, H))
    if h0 is not None:
        h[start] = _f64(h0)
    for t in range(start + 1, T + 1):
        a = x[t - 1] @ w_ih.T + h[t - 1] @ w_hh.T + b
        h[t] = np.tanh(a)
    return h


def head(h_last, w_out, b_out, labels):
    """Mean softmax cross-entropy on z = W_out h_T + b_out and its gradient dL/dh_T."""
    h_last, w_out, b_out = _f64(h_last), _f64(w_out), _f64(b_out)
    labels = np.asarray(labels).astype(np.int64)
    B = h_last.shape[0]
    z = h_last @ w_out.T + b_out
    zmax = z.max(axis=1, keepdims=True)
    lse = zmax[:, 0] + np.log(np.exp(z - zmax).sum(axis=1))
    loss = float(np.mean(lse - z[np.arange(B), labels]))
    p = np.exp(z - lse[:, None])
    p[np.arange(B), labels] -= 1.0
    seed = (p / B) @ w_out
    return loss, seed


def loss(x, w_ih, w_hh, b, w_out, b_out, labels):
    h = forward(x, w_ih, w_hh, b)
    return head(h[-1], w_out, b_out, labels)[0]


def backward_chain(h, w_hh, seed):
    """Eq. 3: g_t = W_hh^T ((1 - h_{t+1}^2) o g_{t+1}), from g_T = seed down to g_0.

    Returns (G, g0) with G[t-1] = dL/dh_t for t = 1..T and g0 = dL/dh_0.
    """
    h, w_hh = _f64(h), _f64(w_hh)
    T = h.shape[0] - 1
    G = np.zeros((T,) + h.shape[1:])
    g = _f64(seed).copy()
    G[T - 1] = g
    for t in range(T - 1, -1, -1):
        g = ((1.0 - h[t + 1] ** 2) * g) @ w_hh
        if t >= 1:
            G[t - 1] = g
    return G, g


def param_grads(h, x, G):
    """Eq. 2 summed over steps: delta_t = (1 - h_t^2) o g_t, outer products with inputs."""
    h, x, G = _f64(h), _f64(x), _f64(G)
    T = G.shape[0]
    H, I = h.shape[2], x.shape[2]
    dw_hh = np.zeros((H, H))
    dw_ih = np.zeros((H, I))
    db = np.zeros(H)
    for t in range(1, T + 1):
        delta = (1.0 - h[t] ** 2) * G[t - 1]
        dw_hh += delta.T @ h[t - 1]
        dw_ih += delta.T @ x[t - 1]
        db += delta.sum(axis=0)
    return dw_ih, dw_hh, db


def step_jacobian_T(h_next, w_hh):
    """Transposed step Jacobian (dh_{t+1}/dh_t)^T per sample, shape [B, H, H].

    dh_{t+1}[j]/dh_t[i] = (1 - h_{t+1}[j]^2) W_hh[j][i], so the transpose has
    entry [i][j] = W_hh[j][i] (1 - h_{t+1}[j]^2): W_hh^T with column j scaled.
    """
    h_next, w_hh = _f64(h_next), _f64(w_hh)
    return w_hh.T[None, :, :] * (1.0 - h_next ** 2)[:, None, :]


def jacobians_T(h, w_hh):
    """All T transposed Jacobians, Jt[t] = (dh_{t+1}/dh_t)^T, shape [T, B, H, H]."""
    h = _f64(h)
    return np.stack([step_jacobian_T(h[t + 1], w_hh) for t in range(h.shape[0] - 1)])
