"""CPU: pins of the training-iteration oracle (oracle/train.py)."""
import numpy as np
import pytest

import workloads
from oracle import rnn, train


def test_adam_first_step_and_constant_gradient_closed_forms():
    rng = np.random.default_rng(0)
    theta, g = rng.standard_normal(50), rng.standard_normal(50) * 1e-3
    lr, eps = 1e-5, 1e-8
    t1, m, v = train.adam_step(theta, g, np.zeros(50), np.zeros(50), 1, lr=lr, eps=eps)
    # t = 1: the bias-corrected moments are g and g^2 exactly
    assert np.allclose(t1, theta - lr * g / (np.abs(g) + eps), rtol=0, atol=1e-18)
    assert np.allclose(m, 0.1 * g) and np.allclose(v, 0.001 * g * g)
    # a constant gradient keeps the corrected moments at g and g^2, so every step is the same
    th, m, v = theta, np.zeros(50), np.zeros(50)
    for t in range(1, 8):
        th, m, v = train.adam_step(th, g, m, v, t, lr=lr, eps=eps)
    assert np.allclose(th, theta - 7 * lr * g / (np.abs(g) + eps), rtol=0, atol=1e-15)
    # the step does not depend on the scale of the gradient (up to eps)
    a = train.adam_step(theta, g, np.zeros(50), np.zeros(50), 1, eps=0.0)[0]
    b = train.adam_step(theta, 1e3 * g, np.zeros(50), np.zeros(50), 1, eps=0.0)[0]
    assert np.allclose(a, b, rtol=0, atol=1e-18)
    # a zero gradient moves nothing and a sign flip mirrors the step
    assert np.array_equal(train.adam_step(theta, np.zeros(50), np.zeros(50), np.zeros(50), 1)[0], theta)
    c = train.adam_step(theta, -g, np.zeros(50), np.zeros(50), 1)[0]
    assert np.allclose(c - theta, -(t1 - theta), rtol=0, atol=1e-18)


def test_adam_second_step_by_hand():
    # two different gradients, written out from the algorithm's four lines
    g1, g2, lr, b1, b2, eps = 0.5, -0.25, 0.1, 0.9, 0.999, 1e-8
    th, m, v = train.adam_step(np.array([1.0]), np.array([g1]), np.zeros(1), np.zeros(1), 1, lr, b1, b2, eps)
    th, m, v = train.adam_step(th, np.array([g2]), m, v, 2, lr, b1, b2, eps)
    m2 = b1 * (1 - b1) * g1 + (1 - b1) * g2
    v2 = b2 * (1 - b2) * g1 * g1 + (1 - b2) * g2 * g2
    want = (1.0 - lr * g1 / (abs(g1) + eps)) - lr * (m2 / (1 - b1 ** 2)) / (np.sqrt(v2 / (1 - b2 ** 2)) + eps)
    assert np.allclose(th, want, rtol=0, atol=1e-15)


def _fd(f, a, idx, h=1e-6):
    a = a.copy()
    old = a[idx]
    a[idx] = old + h
    up = f(a)
    a[idx] = old - h
    dn = f(a)
    return (up - dn) / (2 * h)


def test_gradients_of_every_parameter_against_finite_differences():
    T, B = 12, 3
    x, labels = workloads.bitstream_batch(T, B, first_sample=5)
    p = {k: v.astype(np.float64) for k, v in workloads.rnn_parameters().items()}
    loss, grads = train.rnn_gradients(p, x, labels)
    assert np.isclose(loss, rnn.loss(x, p["w_ih"], p["w_hh"], p["b_ih"] + p["b_hh"], p["w_out"], p["b_out"], labels))
    rng = np.random.default_rng(1)
    for name in train.PARAM_ORDER:
        for _ in range(6):
            idx = tuple(int(rng.integers(0, s)) for s in p[name].shape)

            def f(a, name=name):
                q = dict(p)
                q[name] = a
                return rnn.loss(x, q["w_ih"], q["w_hh"], q["b_ih"] + q["b_hh"], q["w_out"], q["b_out"], labels)

            assert np.isclose(grads[name][idx], _fd(f, p[name], idx), rtol=1e-5, atol=1e-9), (name, idx)


def test_bitstream_batch_follows_the_recipe():
    x, labels = workloads.bitstream_batch(4000, 24, first_sample=100)
    assert x.shape == (4000, 24, 1) and set(np.unique(x)) <= {0.0, 1.0} and labels.min() >= 0 and labels.max() <= 9
    rate = x[:, :, 0].mean(axis=0)
    assert np.all(np.abs(rate - (0.05 + 0.1 * labels)) < 5 * np.sqrt(0.25 / 4000))       # five sigma
    # a sample is the same whatever batch it sits in
    x2, l2 = workloads.bitstream_batch(4000, 4, first_sample=110)
    assert np.array_equal(x2[:, 0], x[:, 10]) and l2[0] == labels[10]


def test_loss_falls_over_iterations_on_one_batch():
    x, labels = workloads.bitstream_batch(30, 16)
    p = {k: v.astype(np.float64) for k, v in workloads.rnn_parameters().items()}
    mom = train.zero_moments(p)
    losses = []
    for t in range(1, 41):
        loss, _, p, mom = train.rnn_iteration(p, mom, x, labels, t, lr=1e-2)
        losses.append(loss)
    assert losses[-1] < 0.5 * losses[0] and np.all(np.diff(losses[:25]) < 0)
