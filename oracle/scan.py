"""fp64 oracle: back-propagation as an exclusive scan.  TEST INFRASTRUCTURE.

Section 3.1 defines A <> B = B A (A a matrix or a vector, B a matrix) with the
identity matrix as neutral element, and states that the gradients are the
exclusive scan of the array
    [ g_n, Jt_n, Jt_{n-1}, ..., Jt_1 ],   Jt_i = (d x_i / d x_{i-1})^T
(Eq. 5), whose output is [ I, g_n, g_{n-1}, ..., g_1 ] (Eq. 4, Algorithm 1's
post-condition).  The method reaches exactly the result of Eq. 3, so the
reference result here is `linear_scan`: the serial scan written out.

`tree_scan` does the work of Algorithm 1 (up-sweep totals of a binary tree,
prefixes handed down with the operands in the down-sweep's order, a symbolic
identity that is never multiplied), written as a recursion over the tree, and
with a block size the hybrid schedule of Section 5.3; it serves purely as a
second, independent opinion and to count which products are matrix-matrix and
which are matrix-vector.

Index convention used by the library (time-indexed, 0-based storage):
Jt[t] = (d h_{t+1} / d h_t)^T for t = 0..T-1, g_t = Jt[t] g_{t+1}, g_T = seed,
output G[t-1] = g_t for t = 1..T and g0 = g_0.  In the paper's array that is
a[0] = g_T and a[k] = Jt[T-k].

Pins (tests/test_oracle_scan.py): H = 1 reduces to numpy's cumulative product;
identity Jacobians return the seed everywhere; diagonal Jacobians reduce to an
element-wise cumulative product; `tree_scan`, `scan_by_definition` and random
bracketings agree with `linear_scan` for every n up to 130 (`tree_scan` with a
block size for every n and every number of up-sweep levels); the RNN oracle's matrix-free
chain equals `linear_scan` on its explicit Jacobians.
"""
from __future__ import annotations

import math

import numpy as np


def linear_scan(jt, seed):
    """Serial scan (Section 3.6, "linear scan"): g_t = Jt[t] g_{t+1}.

    jt: [T, B, H, H], seed: [B, H].  Returns (G [T, B, H], g0 [B, H]).
    """
    jt = np.asarray(jt, dtype=np.float64)
    g = np.asarray(seed, dtype=np.float64).copy()
    T = jt.shape[0]
    G = np.zeros((T,) + g.shape)
    G[T - 1] = g
    for t in range(T - 1, -1, -1):
        g = np.einsum("bij,bj->bi", jt[t], g)
        if t >= 1:
            G[t - 1] = g
    return G, g


# ---- the operator and the paper's array form ------------------------------

def op(a, b):
    """A <> B = B A.  `None` stands for the symbolic identity (never multiplied)."""
    if a is None:
        return b
    if b is None:
        return a
    if b.ndim != 3:
        raise ValueError("right operand of <> must be a (batched) matrix")
    if a.ndim == 3:
        return np.matmul(b, a)
    return np.einsum("bij,bj->bi", b, a)


def to_paper_array(jt, seed):
    """[g_T, Jt[T-1], Jt[T-2], ..., Jt[0]] as a python list of fp64 arrays (Eq. 5)."""
    jt = np.asarray(jt, dtype=np.float64)
    T = jt.shape[0]
    return [np.asarray(seed, dtype=np.float64)] + [jt[T - k] for k in range(1, T + 1)]


def from_paper_array(out):
    """Map [I, g_T, ..., g_1] (Eq. 4) back to G[t-1] = g_t."""
    assert out[0] is None
    n = len(out) - 1
    return np.stack([out[n - t + 1] for t in range(1, n + 1)])


def scan_by_definition(a):
    """Exclusive scan per Section 2.3: out[k] = a[0] <> a[1] <> ... <> a[k-1], out[0] = I."""
    out = [None]
    acc = None
    for k in range(len(a) - 1):
        acc = op(acc, a[k])
        out.append(acc)
    return out


def tree_scan(a, up_levels=None, counts=None, combine=None, is_matrix=None, on_step=None):
    """Exclusive scan of `a` over a balanced binary tree (the work Algorithm 1 does), with the
    hybrid schedule of Section 5.3 when `up_levels` is given.

    len(a) = n + 1.  The array is cut into blocks of 2**up_levels elements (one block holding
    everything when up_levels is None: the full scan).  Inside a block the elements are the leaves
    of a binary tree split at powers of two; `total` of a node is the <>-product of its leaves (the
    up-sweep: node of 2**(d+1) leaves = level d) and is formed only when something asks for it.
    `spread` hands a node's exclusive prefix down (the down-sweep): the left child inherits it, the
    right child gets prefix <> total(left).  Between blocks the prefix advances serially,
    prefix <> total(block): with the gradient vector in the first block these are all matrix-vector
    products.  The total of the last block, and with it anything built on a[n], is never needed.

    counts: dict receiving the number of matrix-matrix ("mm") and matrix-vector ("mv") products per
    phase ("up", "linear", "down").  combine(x, y) = x <> y (default `op`) and is_matrix(v) (default:
    a batched dense matrix) let the same recursion run on other element types; on_step(phase,
    level, x, y) is called before every product of two non-identity operands.
    """
    a = list(a)
    n = len(a) - 1
    combine = op if combine is None else combine
    is_matrix = (lambda v: v.ndim == 3) if is_matrix is None else is_matrix
    depth = math.ceil(math.log2(n + 1)) if n >= 1 else 0
    U = depth if up_levels is None else max(0, min(int(up_levels), max(depth - 1, 0)))
    block = 1 << U
    if counts is not None:
        counts.update({"up_mm": 0, "up_mv": 0, "linear_mv": 0, "linear_mm": 0, "down_mm": 0, "down_mv": 0})
    out = [None] * (n + 1)
    totals = {}

    def product(phase, level, x, y):
        if x is not None and y is not None:
            if counts is not None:
                counts[phase + ("_mm" if is_matrix(x) and is_matrix(y) else "_mv")] += 1
            if on_step is not None:
                on_step(phase, level, x, y)
        return combine(x, y)

    def total(lo, size):
        if size == 1:
            return a[lo]
        half = size // 2
        if lo + half > n:                            # nothing in the right half
            return total(lo, half)
        if (lo, size) not in totals:
            totals[(lo, size)] = product("up", half.bit_length() - 1, total(lo, half), total(lo + half, half))
        return totals[(lo, size)]

    def spread(lo, size, prefix):
        if size == 1:
            out[lo] = prefix
            return
        half = size // 2
        if lo + half > n:
            spread(lo, half, prefix)
            return
        right_prefix = product("down", half.bit_length() - 1, prefix, total(lo, half))
        spread(lo, half, prefix)
        spread(lo + half, half, right_prefix)

    prefix = None                                    # the symbolic identity, never multiplied
    for j, lo in enumerate(range(0, n + 1, block)):
        spread(lo, block, prefix)
        if lo + block <= n:                          # a later block exists
            prefix = product("linear", j, prefix, total(lo, block))
    return out


def random_bracketing(items, rng):
    """Evaluate items[0] <> items[1] <> ... <> items[-1] under a random bracketing."""
    items = list(items)
    while len(items) > 1:
        k = int(rng.integers(0, len(items) - 1))
        items[k:k + 2] = [op(items[k], items[k + 1])]
    return items[0]
