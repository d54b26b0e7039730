"""fp64 oracle: back-propagation as an exclusive scan.  TEST INFRASTRUCTURE.

Section 3.1 defines A <> B = B A (A a matrix or a vector, B a matrix) with the
identity matrix as neutral element, and states that the gradients are the
exclusive scan of the array
    [ g_n, Jt_n, Jt_{n-1}, ..., Jt_1 ],   Jt_i = (d x_i / d x_{i-1})^T
(Eq. 5), whose output is [ I, g_n, g_{n-1}, ..., g_1 ] (Eq. 4, Algorithm 1's
post-condition).  The method reaches exactly the result of Eq. 3, so the
reference result here is `linear_scan`: the serial scan written out.

`blelloch` follows the up-sweep / down-sweep schedule of Algorithm 1 (with the
reversed operands in the down-sweep and a symbolic identity that is never
multiplied) purely as a second, independent opinion and to count which
products are matrix-matrix and which are matrix-vector.

Index convention used by the library (time-indexed, 0-based storage):
Jt[t] = (d h_{t+1} / d h_t)^T for t = 0..T-1, g_t = Jt[t] g_{t+1}, g_T = seed,
output G[t-1] = g_t for t = 1..T and g0 = g_0.  In the paper's array that is
a[0] = g_T and a[k] = Jt[T-k].

Pins (tests/test_oracle_scan.py): H = 1 reduces to numpy's cumulative product;
identity Jacobians return the seed everywhere; diagonal Jacobians reduce to an
element-wise cumulative product; `blelloch`, `scan_by_definition` and random
bracketings agree with `linear_scan` for every n up to 130 (`blelloch_truncated`
for every n and every number of up-sweep levels); the RNN oracle's matrix-free
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


def blelloch(a, counts=None):
    """Modified Blelloch scan with Algorithm 1's level structure, on a copy of `a`.

    len(a) = n + 1.  `counts`, if given, is a dict that receives the number of
    matrix-matrix ("mm") and matrix-vector ("mv") products per phase.
    """
    a = list(a)
    n = len(a) - 1
    levels = math.ceil(math.log2(n + 1)) if n >= 1 else 0
    if counts is not None:
        counts.update({"up_mm": 0, "up_mv": 0, "down_mm": 0, "down_mv": 0})

    def tally(phase, x, y):
        if counts is None or x is None or y is None:
            return
        kind = "mm" if (x.ndim == 3 and y.ndim == 3) else "mv"
        counts[phase + "_" + kind] += 1

    def pairs(d):
        step, half = 1 << (d + 1), 1 << d
        i = 0
        while i <= n - half:
            yield i + half - 1, min(i + step - 1, n)
            i += step

    for d in range(0, levels - 1):                 # up-sweep
        for l, r in pairs(d):
            tally("up", a[l], a[r])
            a[r] = op(a[l], a[r])
    a[n] = None                                    # symbolic identity
    for d in range(levels - 1, -1, -1):            # down-sweep, operands reversed
        for l, r in pairs(d):
            t = a[l]
            a[l] = a[r]
            tally("down", a[r], t)
            a[r] = op(a[r], t)
    return a


def blelloch_truncated(a, up_levels, counts=None):
    """The hybrid schedule of Section 5.3 on a copy of `a`.

    Only the first `up_levels` up-sweep levels run; the block totals they leave
    behind are then combined by a linear scan (matrix-vector products only,
    because the first block holds the gradient vector), which deposits every
    block's exclusive prefix where the down-sweep expects it; the down-sweep then
    runs its last `up_levels` levels.  up_levels = 0 is the pure linear scan.
    """
    a = list(a)
    n = len(a) - 1
    levels = math.ceil(math.log2(n + 1)) if n >= 1 else 0
    U = max(0, min(up_levels, levels - 1)) if levels >= 1 else 0
    if counts is not None:
        counts.update({"up_mm": 0, "up_mv": 0, "linear_mv": 0, "down_mm": 0, "down_mv": 0})

    def tally(phase, x, y):
        if counts is None or x is None or y is None:
            return
        kind = "mm" if (x.ndim == 3 and y.ndim == 3) else "mv"
        counts[phase + "_" + kind] += 1

    def pairs(d):
        step, half = 1 << (d + 1), 1 << d
        i = 0
        while i <= n - half:
            yield i + half - 1, min(i + step - 1, n)
            i += step

    for d in range(0, U):
        for l, r in pairs(d):
            tally("up", a[l], a[r])
            a[r] = op(a[l], a[r])
    block = 1 << U
    prefix = None                                  # exclusive prefix of the current block
    for i in range(0, n + 1, block):
        r = min(i + block - 1, n)
        total = a[r]
        a[r] = prefix
        if i + block <= n:                         # a later block needs prefix <> total
            if prefix is not None:
                tally("linear", prefix, total)
            prefix = op(prefix, total)
    for d in range(U - 1, -1, -1):
        for l, r in pairs(d):
            t = a[l]
            a[l] = a[r]
            tally("down", a[r], t)
            a[r] = op(a[r], t)
    return a


def random_bracketing(items, rng):
    """Evaluate items[0] <> items[1] <> ... <> items[-1] under a random bracketing."""
    items = list(items)
    while len(items) > 1:
        k = int(rng.integers(0, len(items) - 1))
        items[k:k + 2] = [op(items[k], items[k + 1])]
    return items[0]
