"""fp64 oracle: one training iteration of the tanh RNN on a mini-batch.  TEST INFRASTRUCTURE.

Section 4.1's procedure: forward recurrence, softmax cross-entropy on a linear map of the last
hidden state (mean over the batch), back-propagation (Eq. 3 step by step, Eq. 2 summed over the
steps), and one update of every parameter by the Adam optimiser with learning rate 1e-5.  The
optimiser is the published algorithm (Kingma & Ba, "Adam", Algorithm 1) with its default
constants: m <- b1 m + (1 - b1) g;  v <- b2 v + (1 - b2) g^2;  theta <- theta - lr * (m / (1 -
b1^t)) / (sqrt(v / (1 - b2^t)) + eps).  Everything here calls the plain functions of
`oracle.rnn`; nothing is fused.

Pins (tests/test_oracle_train.py): the first Adam step and a run of steps with a constant
gradient against their closed forms (-lr g / (|g| + eps) per step), invariance of the step under
rescaling of the gradient; the head's parameter gradients and the assembled gradient of every
parameter against central finite differences of `oracle.rnn.loss`; a falling loss over repeated
iterations on one batch.
"""
from __future__ import annotations

import numpy as np

from . import rnn as _rnn

PARAM_ORDER = ("w_ih", "w_hh", "b_ih", "b_hh", "w_out", "b_out")


def adam_step(theta, g, m, v, t, lr=1e-5, beta1=0.9, beta2=0.999, eps=1e-8):
    """One Adam update (t = 1 for the first).  Returns (theta, m, v), all new arrays."""
    theta, g, m, v = (np.asarray(a, dtype=np.float64) for a in (theta, g, m, v))
    m = beta1 * m + (1.0 - beta1) * g
    v = beta2 * v + (1.0 - beta2) * g * g
    m_hat = m / (1.0 - beta1 ** t)
    v_hat = v / (1.0 - beta2 ** t)
    return theta - lr * m_hat / (np.sqrt(v_hat) + eps), m, v


def head_backward(h_last, w_out, b_out, labels):
    """Loss, dL/dh_T, dL/dW_out and dL/db_out of the mean softmax cross-entropy on z = W_out h_T + b_out."""
    h_last, w_out, b_out = (np.asarray(a, dtype=np.float64) for a in (h_last, w_out, b_out))
    labels = np.asarray(labels).astype(np.int64)
    B = h_last.shape[0]
    z = h_last @ w_out.T + b_out
    z = z - z.max(axis=1, keepdims=True)
    p = np.exp(z) / np.exp(z).sum(axis=1, keepdims=True)
    loss = float(np.mean(-np.log(p[np.arange(B), labels])))
    dz = p.copy()
    dz[np.arange(B), labels] -= 1.0
    dz /= B                                           # d(mean loss) / dz
    return loss, dz @ w_out, dz.T @ h_last, dz.sum(axis=0)


def rnn_gradients(params, x, labels):
    """Loss and the gradient of every parameter for one mini-batch x [T,B,I], labels [B]."""
    p = {k: np.asarray(params[k], dtype=np.float64) for k in PARAM_ORDER}
    h = _rnn.forward(x, p["w_ih"], p["w_hh"], p["b_ih"] + p["b_hh"])
    loss, seed, dw_out, db_out = head_backward(h[-1], p["w_out"], p["b_out"], labels)
    G, _ = _rnn.backward_chain(h, p["w_hh"], seed)
    dw_ih, dw_hh, db = _rnn.param_grads(h, x, G)
    return loss, {"w_ih": dw_ih, "w_hh": dw_hh, "b_ih": db, "b_hh": db.copy(), "w_out": dw_out, "b_out": db_out}


def rnn_iteration(params, moments, x, labels, t, lr=1e-5, beta1=0.9, beta2=0.999, eps=1e-8):
    """One training iteration.  moments = {name: (m, v)} (zeros before the first), t = 1, 2, ...
    Returns (loss before the update, gradients, new params, new moments)."""
    loss, grads = rnn_gradients(params, x, labels)
    new_p, new_m = {}, {}
    for k in PARAM_ORDER:
        m, v = moments[k]
        new_p[k], m, v = adam_step(params[k], grads[k], m, v, t, lr, beta1, beta2, eps)
        new_m[k] = (m, v)
    return loss, grads, new_p, new_m


def zero_moments(params):
    return {k: (np.zeros(np.shape(params[k])), np.zeros(np.shape(params[k]))) for k in PARAM_ORDER}
