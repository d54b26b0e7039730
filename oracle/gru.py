"""fp64 oracle: single-layer GRU, sequential back-propagation.  TEST INFRASTRUCTURE.

Cell (Section 4.2, the GRU equations; Appendix E's rewrite with pre-activations
R, Z, M, N):
    R = W_ir x + b_ir + W_hr h' + b_hr,   r = sigmoid(R)
    Z = W_iz x + b_iz + W_hz h' + b_hz,   z = sigmoid(Z)
    M = W_hn h' + b_hn,  N = W_in x + b_in + r o M,  n = tanh(N)
    h = (1 - z) o n + z o h'
with h' the previous hidden state.  Weights are stacked in gate order (r, z, n):
w_ih [3H, I], w_hh [3H, H], b_ih [3H], b_hh [3H].

Backward is Eq. 3 applied as a vector-Jacobian product per step (chain rule on
the rewrite above), and Eq. 2 summed over steps.  The paper prints only the
hidden-state Jacobian (Appendix E); the parameter formulas are the chain rule
on the same rewrite.

Pins (tests/test_oracle_gru.py): central finite differences of the loss for
every parameter; `step_jacobian_T` (Appendix E's formula as printed) against
finite differences of one step and against the vector-Jacobian product.
"""
from __future__ import annotations

import numpy as np


def _f64(a):
    return np.asarray(a, dtype=np.float64)


def _sigmoid(a):
    return 1.0 / (1.0 + np.exp(-a))


def gates(h_prev, x_t, w_ih, w_hh, b_ih, b_hh):
    """r, z, n, M of one step for a batch: h_prev [B, H], x_t [B, I]."""
    h_prev, x_t = _f64(h_prev), _f64(x_t)
    w_ih, w_hh, b_ih, b_hh = _f64(w_ih), _f64(w_hh), _f64(b_ih), _f64(b_hh)
    H = h_prev.shape[1]
    gi = x_t @ w_ih.T + b_ih
    gh = h_prev @ w_hh.T + b_hh
    r = _sigmoid(gi[:, :H] + gh[:, :H])
    z = _sigmoid(gi[:, H:2 * H] + gh[:, H:2 * H])
    M = gh[:, 2 * H:]
    n = np.tanh(gi[:, 2 * H:] + r * M)
    return r, z, n, M


def step(h_prev, x_t, w_ih, w_hh, b_ih, b_hh):
    r, z, n, _ = gates(h_prev, x_t, w_ih, w_hh, b_ih, b_hh)
    return (1.0 - z) * n + z * _f64(h_prev)


def forward(x, w_ih, w_hh, b_ih, b_hh):
    x = _f64(x)
    T, B, _ = x.shape
    H = np.asarray(w_hh).shape[1]
    h = np.zeros((T + 1, B, H))
    for t in range(1, T + 1):
        h[t] = step(h[t - 1], x[t - 1], w_ih, w_hh, b_ih, b_hh)
    return h


def _step_deltas(g, h_prev, x_t, w_ih, w_hh, b_ih, b_hh):
    r, z, n, M = gates(h_prev, x_t, w_ih, w_hh, b_ih, b_hh)
    dN = g * (1.0 - z) * (1.0 - n * n)
    dZ = g * (_f64(h_prev) - n) * z * (1.0 - z)
    dM = dN * r
    dR = dN * M * r * (1.0 - r)
    return dR, dZ, dN, dM, z


def backward_chain(h, x, w_ih, w_hh, b_ih, b_hh, seed):
    """g_{t-1} = W_hr^T dR + W_hz^T dZ + W_hn^T dM + z o g_t, from g_T = seed.

    Returns (G, g0) with G[t-1] = dL/dh_t.
    """
    h, w_hh = _f64(h), _f64(w_hh)
    T = h.shape[0] - 1
    H = h.shape[2]
    G = np.zeros((T,) + h.shape[1:])
    g = _f64(seed).copy()
    G[T - 1] = g
    for t in range(T, 0, -1):
        dR, dZ, dN, dM, z = _step_deltas(g, h[t - 1], x[t - 1], w_ih, w_hh, b_ih, b_hh)
        g = dR @ w_hh[:H] + dZ @ w_hh[H:2 * H] + dM @ w_hh[2 * H:] + z * g
        if t >= 2:
            G[t - 2] = g
    return G, g


def param_grads(h, x, G, w_ih, w_hh, b_ih, b_hh):
    """Eq. 2 summed over steps.  Returns dW_ih [3H, I], dW_hh [3H, H], db_ih, db_hh [3H]."""
    h, x, G = _f64(h), _f64(x), _f64(G)
    T = G.shape[0]
    H, I = h.shape[2], x.shape[2]
    dw_ih = np.zeros((3 * H, I))
    dw_hh = np.zeros((3 * H, H))
    db_ih = np.zeros(3 * H)
    db_hh = np.zeros(3 * H)
    for t in range(1, T + 1):
        dR, dZ, dN, dM, _ = _step_deltas(G[t - 1], h[t - 1], x[t - 1], w_ih, w_hh, b_ih, b_hh)
        d_i = np.concatenate([dR, dZ, dN], axis=1)       # what reaches W_i* and b_i*
        d_h = np.concatenate([dR, dZ, dM], axis=1)       # what reaches W_h* and b_h*
        dw_ih += d_i.T @ x[t - 1]
        dw_hh += d_h.T @ h[t - 1]
        db_ih += d_i.sum(axis=0)
        db_hh += d_h.sum(axis=0)
    return dw_ih, dw_hh, db_ih, db_hh


def step_jacobian_T(h_prev, x_t, w_ih, w_hh, b_ih, b_hh):
    """Appendix E's formula for (dh_t/dh_{t-1})^T, per sample: [B, H, H].

    (J1 o (j2 o j3)^T + J4 o j5^T) o (j6 o j7)^T + J8 o (j9 o j10)^T + J11,
    where "J o v^T" scales column j of J by v_j.
    """
    r, z, n, M = gates(h_prev, x_t, w_ih, w_hh, b_ih, b_hh)
    w_hh = _f64(w_hh)
    H = w_hh.shape[1]
    J1, J8, J4 = w_hh[:H].T, w_hh[H:2 * H].T, w_hh[2 * H:].T
    j2, j3, j5 = r * (1.0 - r), M, r
    j6, j7 = 1.0 - n * n, 1.0 - z
    j9, j10 = z * (1.0 - z), _f64(h_prev) - n

    def cols(J, v):                      # J o v^T, batched over v's first axis
        return J[None, :, :] * v[:, None, :]

    out = (cols(J1, j2 * j3) + cols(J4, j5)) * (j6 * j7)[:, None, :] + cols(J8, j9 * j10)
    idx = np.arange(H)
    out[:, idx, idx] += z
    return out


def jacobians_T(h, x, w_ih, w_hh, b_ih, b_hh):
    """Jt[t] = (dh_{t+1}/dh_t)^T for t = 0..T-1, shape [T, B, H, H]."""
    h, x = _f64(h), _f64(x)
    T = h.shape[0] - 1
    return np.stack([step_jacobian_T(h[t], x[t], w_ih, w_hh, b_ih, b_hh) for t in range(T)])
