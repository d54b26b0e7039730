"""Pins for oracle/gru.py: finite differences, Appendix E's Jacobian (CPU only)."""
import numpy as np

import workloads
from oracle import gru, rnn, scan


def _setup(T=6, B=2, H=3, I=2, C=4, seed=5):
    w = workloads.gru_inputs(T, B, H, I, C, seed=seed, audio=False)
    return {k: (np.asarray(v, dtype=np.float64) if isinstance(v, np.ndarray) and v.dtype == np.float32 else v)
            for k, v in w.items()}


def _loss(w, **over):
    p = dict(w)
    p.update(over)
    h = gru.forward(p["x"], p["w_ih"], p["w_hh"], p["b_ih"], p["b_hh"])
    return rnn.head(h[-1], p["w_out"], p["b_out"], p["labels"])[0]


def _central_fd(f, a, eps=1e-6):
    g = np.zeros_like(a)
    for idx in np.ndindex(*a.shape):
        ap, am = a.copy(), a.copy()
        ap[idx] += eps
        am[idx] -= eps
        g[idx] = (f(ap) - f(am)) / (2 * eps)
    return g


def test_gru_param_grads_match_finite_differences():
    w = _setup()
    h = gru.forward(w["x"], w["w_ih"], w["w_hh"], w["b_ih"], w["b_hh"])
    _, seed = rnn.head(h[-1], w["w_out"], w["b_out"], w["labels"])
    G, _ = gru.backward_chain(h, w["x"], w["w_ih"], w["w_hh"], w["b_ih"], w["b_hh"], seed)
    got = dict(zip(("w_ih", "w_hh", "b_ih", "b_hh"),
                   gru.param_grads(h, w["x"], G, w["w_ih"], w["w_hh"], w["b_ih"], w["b_hh"])))
    for name in got:
        fd = _central_fd(lambda a: _loss(w, **{name: a}), w[name])
        assert np.max(np.abs(fd - got[name])) <= 2e-6 * np.max(np.abs(fd)), name
    H = w["H"]
    # the r and z gates see b_ih and b_hh only through their sum
    assert np.allclose(got["b_ih"][:2 * H], got["b_hh"][:2 * H], rtol=0, atol=0)
    assert not np.allclose(got["b_ih"][2 * H:], got["b_hh"][2 * H:])


def test_gru_step_jacobian_as_printed_matches_finite_differences():
    w = _setup(T=1, B=2, H=4, I=1)
    rng = np.random.default_rng(3)
    h_prev = rng.standard_normal((2, 4)) * 0.7
    args = (w["x"][0], w["w_ih"], w["w_hh"], w["b_ih"], w["b_hh"])
    jt = gru.step_jacobian_T(h_prev, *args)
    eps = 1e-6
    for b in range(2):
        for i in range(4):
            hp, hm = h_prev.copy(), h_prev.copy()
            hp[b, i] += eps
            hm[b, i] -= eps
            col = (gru.step(hp, *args)[b] - gru.step(hm, *args)[b]) / (2 * eps)
            assert np.allclose(jt[b, i, :], col, rtol=1e-6, atol=1e-9)


def test_gru_chain_equals_linear_scan_on_explicit_jacobians():
    w = _setup(T=19, B=2, H=5, I=1)
    h = gru.forward(w["x"], w["w_ih"], w["w_hh"], w["b_ih"], w["b_hh"])
    _, seed = rnn.head(h[-1], w["w_out"], w["b_out"], w["labels"])
    G, g0 = gru.backward_chain(h, w["x"], w["w_ih"], w["w_hh"], w["b_ih"], w["b_hh"], seed)
    jt = gru.jacobians_T(h, w["x"], w["w_ih"], w["w_hh"], w["b_ih"], w["b_hh"])
    G2, g02 = scan.linear_scan(jt, seed)
    assert np.allclose(G, G2, rtol=1e-11, atol=1e-300)
    assert np.allclose(g0, g02, rtol=1e-11, atol=1e-300)


def test_gru_hidden_grads_match_finite_differences():
    w = _setup(T=5, B=2, H=3, I=1)
    args = (w["w_ih"], w["w_hh"], w["b_ih"], w["b_hh"])
    h = gru.forward(w["x"], *args)
    _, seed = rnn.head(h[-1], w["w_out"], w["b_out"], w["labels"])
    G, g0 = gru.backward_chain(h, w["x"], *args, seed)

    def loss_from(t, ht):
        cur = ht
        for s in range(t + 1, w["T"] + 1):
            cur = gru.step(cur, w["x"][s - 1], *args)
        return rnn.head(cur, w["w_out"], w["b_out"], w["labels"])[0]

    for t in range(0, w["T"] + 1):
        fd = _central_fd(lambda a: loss_from(t, a), h[t])
        got = g0 if t == 0 else G[t - 1]
        assert np.max(np.abs(fd - got)) <= 2e-6 * np.max(np.abs(fd)) + 1e-12, t
