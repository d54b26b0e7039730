"""Pins for oracle/rnn.py: finite differences and explicit Jacobians (CPU only)."""
import numpy as np
import pytest

import workloads
from oracle import rnn, scan


def _setup(T=7, B=3, H=5, I=2, C=4, seed=11):
    w = workloads.rnn_inputs(T, B, H, I, C, seed=seed)
    w = {k: (np.asarray(v, dtype=np.float64) if isinstance(v, np.ndarray) and v.dtype == np.float32 else v)
         for k, v in w.items()}
    return w


def _loss(w, **over):
    p = dict(w)
    p.update(over)
    return rnn.loss(p["x"], p["w_ih"], p["w_hh"], p["b"], p["w_out"], p["b_out"], p["labels"])


def _central_fd(f, a, eps=1e-6):
    g = np.zeros_like(a)
    it = np.nditer(a, flags=["multi_index"])
    for _ in it:
        idx = it.multi_index
        ap, am = a.copy(), a.copy()
        ap[idx] += eps
        am[idx] -= eps
        g[idx] = (f(ap) - f(am)) / (2 * eps)
    return g


def _grads(w):
    h = rnn.forward(w["x"], w["w_ih"], w["w_hh"], w["b"])
    _, seed = rnn.head(h[-1], w["w_out"], w["b_out"], w["labels"])
    G, g0 = rnn.backward_chain(h, w["w_hh"], seed)
    return h, seed, G, g0, rnn.param_grads(h, w["x"], G)


def test_param_grads_match_finite_differences():
    w = _setup()
    _, _, _, _, (dw_ih, dw_hh, db) = _grads(w)
    for name, got in (("w_ih", dw_ih), ("w_hh", dw_hh), ("b", db)):
        fd = _central_fd(lambda a: _loss(w, **{name: a}), w[name])
        assert np.max(np.abs(fd - got)) <= 1e-7 * max(1.0, np.max(np.abs(fd))), name
        assert np.max(np.abs(fd - got)) <= 2e-6 * np.max(np.abs(fd)), name


def test_hidden_state_grads_match_finite_differences():
    w = _setup()
    h, _, G, g0, _ = _grads(w)
    T = w["T"]

    def loss_with_h(t, ht):
        hh = rnn.forward(w["x"], w["w_ih"], w["w_hh"], w["b"], h0=ht, start=t)
        return rnn.head(hh[-1], w["w_out"], w["b_out"], w["labels"])[0]

    for t in (0, 1, T // 2, T - 1, T):
        fd = _central_fd(lambda a: loss_with_h(t, a), h[t])
        got = g0 if t == 0 else G[t - 1]
        assert np.max(np.abs(fd - got)) <= 2e-6 * np.max(np.abs(fd)) + 1e-12, t


def test_seed_is_gradient_of_head():
    w = _setup()
    h = rnn.forward(w["x"], w["w_ih"], w["w_hh"], w["b"])
    _, seed = rnn.head(h[-1], w["w_out"], w["b_out"], w["labels"])
    fd = _central_fd(lambda a: rnn.head(a, w["w_out"], w["b_out"], w["labels"])[0], h[-1])
    assert np.allclose(fd, seed, rtol=1e-6, atol=1e-10)
    # uniform logits: the loss of an all-zero head is log(C)
    l0, _ = rnn.head(h[-1], 0 * w["w_out"], 0 * w["b_out"], w["labels"])
    assert abs(l0 - np.log(w["C"])) < 1e-12


def test_step_jacobian_matches_finite_differences_of_one_step():
    w = _setup(T=1, B=2, H=4, I=1)
    rng = np.random.default_rng(0)
    h_prev = rng.standard_normal((2, 4)) * 0.5

    def one_step(hp):
        return np.tanh(w["x"][0] @ w["w_ih"].T + hp @ w["w_hh"].T + w["b"])

    h_next = one_step(h_prev)
    jt = rnn.step_jacobian_T(h_next, w["w_hh"])
    eps = 1e-6
    for b in range(2):
        for i in range(4):
            hp, hm = h_prev.copy(), h_prev.copy()
            hp[b, i] += eps
            hm[b, i] -= eps
            col = (one_step(hp)[b] - one_step(hm)[b]) / (2 * eps)   # d h_next[:] / d h_prev[i]
            assert np.allclose(jt[b, i, :], col, rtol=1e-6, atol=1e-9)


def test_matrix_free_chain_equals_linear_scan_on_explicit_jacobians():
    w = _setup(T=23, B=2, H=6, I=1)
    h, seed, G, g0, _ = _grads(w)
    jt = rnn.jacobians_T(h, w["w_hh"])
    G2, g02 = scan.linear_scan(jt, seed)
    assert np.allclose(G, G2, rtol=1e-12, atol=1e-300)
    assert np.allclose(g0, g02, rtol=1e-12, atol=1e-300)


def test_single_step_closed_form():
    # T = 1, H = 1: dL/dw_hh = 0 because h_0 = 0; dL/db = (1 - h_1^2) * seed.
    w = _setup(T=1, B=1, H=1, I=1, C=2)
    h, seed, G, g0, (dw_ih, dw_hh, db) = _grads(w)
    assert G.shape == (1, 1, 1) and G[0, 0, 0] == seed[0, 0]
    assert dw_hh[0, 0] == 0.0
    assert np.isclose(db[0], (1 - h[1, 0, 0] ** 2) * seed[0, 0])
    assert np.isclose(dw_ih[0, 0], db[0] * w["x"][0, 0, 0])
    assert np.isclose(g0[0, 0], w["w_hh"][0, 0] * db[0])
