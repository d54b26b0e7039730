"""Pins for oracle/scan.py: textbook special cases, brute force over n, bracketings."""
import numpy as np
import pytest

import workloads
from oracle import scan


def test_h1_reduces_to_cumulative_product():
    rng = np.random.default_rng(1)
    T, B = 37, 3
    jt = rng.uniform(0.5, 1.5, size=(T, B, 1, 1))
    seed = rng.standard_normal((B, 1))
    G, g0 = scan.linear_scan(jt, seed)
    # g_t = seed * prod_{s=t}^{T-1} jt[s]  ->  reversed cumulative product
    cp = np.cumprod(jt[::-1, :, 0, 0], axis=0)[::-1]          # cp[t] = prod_{s>=t} jt[s]
    for t in range(1, T):
        assert np.allclose(G[t - 1, :, 0], seed[:, 0] * cp[t], rtol=1e-12)
    assert np.allclose(G[T - 1], seed)
    assert np.allclose(g0[:, 0], seed[:, 0] * cp[0], rtol=1e-12)


def test_identity_jacobians_return_seed_everywhere():
    T, B, H = 20, 2, 4
    jt = np.broadcast_to(np.eye(H), (T, B, H, H)).copy()
    seed = np.random.default_rng(2).standard_normal((B, H))
    G, g0 = scan.linear_scan(jt, seed)
    assert all(np.array_equal(G[t], seed) for t in range(T)) and np.array_equal(g0, seed)
    out = scan.tree_scan(scan.to_paper_array(jt, seed))
    assert np.array_equal(scan.from_paper_array(out), G)


def test_diagonal_jacobians_reduce_to_elementwise_cumprod():
    rng = np.random.default_rng(3)
    T, B, H = 15, 2, 3
    d = rng.uniform(0.5, 1.5, size=(T, B, H))
    jt = np.zeros((T, B, H, H))
    jt[..., np.arange(H), np.arange(H)] = d
    seed = rng.standard_normal((B, H))
    G, _ = scan.linear_scan(jt, seed)
    cp = np.cumprod(d[::-1], axis=0)[::-1]
    for t in range(1, T):
        assert np.allclose(G[t - 1], seed * cp[t], rtol=1e-12)


def test_operand_order_is_reversed_product():
    # A <> B = B A, not A B: a transposed operand or swapped order must fail this.
    rng = np.random.default_rng(4)
    A = rng.standard_normal((1, 3, 3))
    Bm = rng.standard_normal((1, 3, 3))
    v = rng.standard_normal((1, 3))
    assert np.allclose(scan.op(A, Bm)[0], Bm[0] @ A[0])
    assert not np.allclose(scan.op(A, Bm)[0], A[0] @ Bm[0])
    assert np.allclose(scan.op(v, Bm)[0], Bm[0] @ v[0])
    with pytest.raises(ValueError):
        scan.op(A, v)
    # two-step chain written out by hand: g_1 = Jt[1] g_2 (seed), g_0 = Jt[0] g_1
    jt = rng.standard_normal((2, 1, 3, 3))
    G, g0 = scan.linear_scan(jt, v)
    assert np.allclose(G[1, 0], v[0])
    assert np.allclose(G[0, 0], jt[1, 0] @ v[0])
    assert np.allclose(g0[0], jt[0, 0] @ (jt[1, 0] @ v[0]))


@pytest.mark.parametrize("n", list(range(1, 131)))
def test_tree_scan_and_definition_equal_linear_scan_for_every_n(n):
    B, H = 2, 3
    jt, seed = workloads.random_jacobian_chain(n, B, H, seed=100 + n, dtype=np.float64)
    G, _ = scan.linear_scan(jt, seed)
    a = scan.to_paper_array(jt, seed)
    counts = {}
    out = scan.tree_scan(a, None, counts)
    assert out[0] is None
    Gb = scan.from_paper_array(out)
    assert np.allclose(Gb, G, rtol=1e-10, atol=1e-13)
    Gd = scan.from_paper_array(scan.scan_by_definition(a))
    assert np.allclose(Gd, G, rtol=1e-10, atol=1e-13)
    # only the up-sweep holds matrix-matrix products (Section 3.2)
    assert counts["down_mm"] == 0
    # work stays linear: never more than one product per element and phase
    assert counts["up_mm"] + counts["up_mv"] <= n
    assert counts["down_mv"] <= n


@pytest.mark.parametrize("n", [1, 2, 3, 5, 8, 13, 31, 64])
def test_random_bracketings_agree(n):
    rng = np.random.default_rng(n)
    jt, seed = workloads.random_jacobian_chain(n, 2, 4, seed=7 * n, dtype=np.float64)
    G, g0 = scan.linear_scan(jt, seed)
    a = scan.to_paper_array(jt, seed)
    for _ in range(5):
        for k in (1, n // 2 + 1, n):
            val = scan.random_bracketing(a[:k + 1], rng)   # g_T <> Jt_{T-1} <> ... (k factors)
            want = G[n - k - 1] if k < n else g0
            assert np.allclose(val, want, rtol=1e-9, atol=1e-12)


def test_last_jacobian_never_reaches_an_output():
    jt, seed = workloads.random_jacobian_chain(9, 1, 3, seed=5, dtype=np.float64)
    jt2 = jt.copy()
    jt2[0] = 123.0                       # a[n] in the paper's array
    G1 = scan.from_paper_array(scan.tree_scan(scan.to_paper_array(jt, seed)))
    G2 = scan.from_paper_array(scan.tree_scan(scan.to_paper_array(jt2, seed)))
    assert np.array_equal(G1, G2)


@pytest.mark.parametrize("n", list(range(1, 70)) + [100, 127, 128, 129])
def test_truncated_schedule_equals_linear_scan_for_every_level_count(n):
    jt, seed = workloads.random_jacobian_chain(n, 1, 3, seed=300 + n, dtype=np.float64)
    G, _ = scan.linear_scan(jt, seed)
    a = scan.to_paper_array(jt, seed)
    for U in range(0, 9):
        counts = {}
        out = scan.tree_scan(a, U, counts)
        assert out[0] is None
        assert np.allclose(scan.from_paper_array(out), G, rtol=1e-10, atol=1e-13), (n, U)
        assert counts["down_mm"] == 0
        if U == 0:
            assert counts["up_mm"] == 0 and counts["up_mv"] == 0      # pure linear scan
