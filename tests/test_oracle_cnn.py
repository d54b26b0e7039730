"""Pins for oracle/cnn.py (CPU only): the paper's printed values, brute force, finite differences."""
import os

import numpy as np
import pytest
import scipy.sparse as sp

import workloads
from oracle import cnn

GOLD = os.path.join(os.path.dirname(__file__), "golden", "table1_sparsity.txt")


def _gold():
    vals = {}
    for line in open(GOLD):
        line = line.split("#")[0].split()
        if line:
            vals[line[0]] = [float(v) for v in line[1:]]
    return vals


def test_table1_sparsity_values_and_section33_storage():
    g = _gold()
    rng = np.random.default_rng(0)
    w = rng.standard_normal((64, 3, 3, 3))
    jt = cnn.conv_jacobian_T(w, None, 32, 32)
    rows, cols, want = g["conv1"]
    assert jt.shape == (rows, cols)
    # true non-zero count c_i c_o (3h-2)(3w-2) reproduces the printed sparsity and the 6.5 MB
    assert jt.nnz == 3 * 64 * 94 * 94 == 1696512
    assert round(1 - jt.nnz / (rows * cols), 5) == want
    assert rows * cols * 4 / 2 ** 20 == g["conv1_dense_mb"][0]
    assert round(jt.nnz * 4 / 2 ** 20, 1) == g["conv1_csr_mb"][0]
    # ReLU: one stored entry per element
    x = rng.standard_normal(65536)
    jr = cnn.relu_jacobian_T(x)
    assert jr.nnz == 65536 and round(1 - jr.nnz / 65536 ** 2, 5) == g["relu1"][2]
    # max-pooling: the guaranteed zeros are everything outside the 4-candidate windows
    rows, cols, want = g["pool1"]
    assert round(1 - 4 * 16384 / (rows * cols), 5) == want
    _, idx = cnn.maxpool2x2_fast(x.reshape(64, 32, 32))
    jp = cnn.pool_jacobian_T(idx, (64, 32, 32))
    assert jp.shape == (rows, cols) and jp.nnz == 16384 and np.all(jp.data == 1.0)


def test_conv_interior_row_lengths_match_algorithm2():
    # Algorithm 2 allots 6 c_o entries to pixels of the first and last image row and 9 c_o to
    # the others; away from the left/right edge the in-image reading has the same lengths.
    co, ci, h, w = 5, 2, 6, 7
    jt = cnn.conv_jacobian_T(np.ones((co, ci, 3, 3)), None, h, w)
    lens = np.diff(jt.indptr).reshape(ci, h, w)
    assert np.all(lens[:, 1:-1, 1:-1] == 9 * co)
    assert np.all(lens[:, 0, 1:-1] == 6 * co) and np.all(lens[:, -1, 1:-1] == 6 * co)
    assert np.all(lens[:, 1:-1, 0] == 6 * co) and np.all(lens[:, 0, 0] == 4 * co)
    assert jt.nnz == ci * co * (3 * h - 2) * (3 * w - 2)
    assert jt.indptr.size == ci * h * w + 1


def _impulse_jacobian_T(f, n_in):
    cols = []
    for i in range(n_in):
        e = np.zeros(n_in)
        e[i] = 1.0
        cols.append(np.asarray(f(e)).reshape(-1))
    return np.stack(cols)          # row i = d out / d in[i]


@pytest.mark.parametrize("ci,co,h,w", [(2, 3, 4, 5), (1, 1, 1, 1), (3, 2, 2, 2), (1, 2, 1, 4)])
def test_conv_jacobian_matches_unit_impulses(ci, co, h, w):
    rng = np.random.default_rng(ci * 10 + co)
    wt = rng.standard_normal((co, ci, 3, 3))
    mask = rng.random((co, ci, 3, 3)) < 0.6
    wm = np.where(mask, wt, 0.0)
    dense = _impulse_jacobian_T(lambda e: cnn.conv3x3(e.reshape(ci, h, w), wm), ci * h * w)
    jt = cnn.conv_jacobian_T(wm, mask, h, w)
    assert np.allclose(jt.toarray(), dense, atol=0, rtol=0)
    # structure = where the mask (not the value) allows an entry
    pat = _impulse_jacobian_T(lambda e: cnn.conv3x3(e.reshape(ci, h, w), mask.astype(float)), ci * h * w)
    assert np.array_equal(jt.toarray() != 0, (pat != 0) & (dense != 0))
    got_pat = sp.csr_matrix((np.ones(jt.nnz), jt.indices, jt.indptr), shape=jt.shape).toarray()
    assert np.array_equal(got_pat != 0, pat != 0)
    assert all(np.all(np.diff(jt.indices[jt.indptr[r]:jt.indptr[r + 1]]) > 0) for r in range(jt.shape[0]))


GEOMETRIES = [  # (ci, co, h, w, kh, kw, stride, padding, dilation)
    (2, 3, 5, 6, 3, 3, (1, 1), (1, 1), (1, 1)),
    (1, 2, 7, 5, 5, 3, (2, 1), (2, 0), (1, 1)),
    (2, 2, 8, 8, 2, 2, (2, 2), (0, 0), (1, 1)),
    (1, 1, 9, 7, 3, 2, (3, 2), (1, 1), (2, 3)),
    (3, 1, 4, 4, 1, 1, (1, 1), (0, 0), (1, 1)),
    (1, 2, 6, 6, 4, 4, (1, 1), (3, 3), (1, 1)),
    (2, 1, 5, 5, 7, 7, (1, 1), (0, 0), (1, 1)),     # kernel larger than the image: no output
]


@pytest.mark.parametrize("ci,co,h,w,kh,kw,stride,padding,dilation", GEOMETRIES)
def test_generic_conv_and_its_jacobian(ci, co, h, w, kh, kw, stride, padding, dilation):
    from scipy.signal import correlate2d
    rng = np.random.default_rng(kh * 10 + kw)
    wt = rng.standard_normal((co, ci, kh, kw))
    mask = rng.random((co, ci, kh, kw)) < 0.7
    wm = np.where(mask, wt, 0.0)
    x = rng.standard_normal((ci, h, w))
    out = cnn.conv2d(x, wm, stride, padding, dilation)
    oh, ow = cnn.conv2d_out_size(h, kh, stride[0], padding[0], dilation[0]), \
        cnn.conv2d_out_size(w, kw, stride[1], padding[1], dilation[1])
    assert out.shape == (co, oh, ow)
    if dilation == (1, 1) and oh > 0 and ow > 0:
        # SciPy's full-padded correlation, cropped to this padding and sampled at this stride
        xp = np.pad(x, ((0, 0), (padding[0],) * 2, (padding[1],) * 2))
        ref = np.stack([sum(correlate2d(xp[c], wm[o, c], mode="valid") for c in range(ci)) for o in range(co)])
        assert np.allclose(out, ref[:, ::stride[0], ::stride[1]], rtol=1e-12, atol=1e-12)
    jt = cnn.conv2d_jacobian_T(wm, mask, h, w, stride, padding, dilation)
    assert jt.shape == (ci * h * w, co * oh * ow)
    dense = _impulse_jacobian_T(lambda e: cnn.conv2d(e.reshape(ci, h, w), wm, stride, padding, dilation), ci * h * w)
    assert np.array_equal(jt.toarray(), dense.reshape(ci * h * w, co * oh * ow))
    pat = _impulse_jacobian_T(lambda e: cnn.conv2d(e.reshape(ci, h, w), mask.astype(float), stride, padding, dilation),
                              ci * h * w).reshape(ci * h * w, -1)
    got_pat = sp.csr_matrix((np.ones(jt.nnz), jt.indices, jt.indptr), shape=jt.shape).toarray()
    assert np.array_equal(got_pat != 0, pat != 0)
    assert all(np.all(np.diff(jt.indices[jt.indptr[r]:jt.indptr[r + 1]]) > 0) for r in range(jt.shape[0]))


def test_generic_conv_reduces_to_the_3x3_case():
    rng = np.random.default_rng(9)
    wt = rng.standard_normal((4, 3, 3, 3))
    mask = rng.random(wt.shape) < 0.5
    x = rng.standard_normal((3, 6, 5))
    assert np.allclose(cnn.conv2d(x, wt, (1, 1), (1, 1)), cnn.conv3x3(x, wt), rtol=1e-13, atol=1e-13)
    a = cnn.conv2d_jacobian_T(wt, mask, 6, 5, (1, 1), (1, 1))
    b = cnn.conv_jacobian_T(wt, mask, 6, 5)
    assert np.array_equal(a.indptr, b.indptr) and np.array_equal(a.indices, b.indices) and np.array_equal(a.data, b.data)


def test_kept_zero_weight_stays_structural():
    w = np.zeros((1, 1, 3, 3))
    jt = cnn.conv_jacobian_T(w, np.ones((1, 1, 3, 3), bool), 2, 2)
    assert jt.nnz == 16 and np.all(jt.data == 0)


def test_pool_relu_fc_jacobians_match_definitions():
    rng = np.random.default_rng(5)
    x = rng.standard_normal((2, 4, 6))
    x[0, :2, :2] = 0.0                                   # a tie: first element of the window wins
    out, idx = cnn.maxpool2x2(x)
    out2, idx2 = cnn.maxpool2x2_fast(x)
    assert np.array_equal(out, out2) and np.array_equal(idx, idx2) and idx[0, 0, 0] == 0
    jp = cnn.pool_jacobian_T(idx, x.shape).toarray()
    eps = 1e-6
    fd = _impulse_jacobian_T(lambda e: (cnn.maxpool2x2(x + eps * e.reshape(x.shape))[0] - out) / eps, x.size)
    fd[0 * 24 + 1] = 0; fd[0 * 24 + 6] = 0; fd[0 * 24 + 7] = 0   # perturbing a tied loser flips the argmax
    fd[0] = jp[0]
    assert np.allclose(jp, fd, atol=1e-6)
    jr = cnn.relu_jacobian_T(x)
    assert np.array_equal(jr.indices, np.arange(x.size)) and np.array_equal(jr.data, (x.reshape(-1) > 0) * 1.0)
    w = rng.standard_normal((3, 5))
    m = rng.random((3, 5)) < 0.5
    jf = cnn.fc_jacobian_T(np.where(m, w, 0), m)
    assert np.array_equal(jf.toarray(), np.where(m, w, 0).T) and jf.nnz == m.sum()


def _tiny_net(seed=0):
    return workloads.cnn_layers(conv_channels=(3, 4), pool_after=(1, 2), fc=(6, 5), in_shape=(2, 8, 8),
                                prune=0.5, seed=seed)


def test_backward_matches_finite_differences_and_sparse_chain():
    layers, image, label = _tiny_net()
    acts, aux = cnn.forward(layers, image)
    grads = cnn.backward(layers, acts, aux, label)

    def loss_of(img):
        a, _ = cnn.forward(layers, img)
        return cnn.loss_and_seed(a[-1], label)[0]

    eps = 1e-6
    img = np.asarray(image, np.float64)
    fd = np.zeros_like(img)
    for idx in np.ndindex(*img.shape):
        p, m = img.copy(), img.copy()
        p[idx] += eps
        m[idx] -= eps
        fd[idx] = (loss_of(p) - loss_of(m)) / (2 * eps)
    assert np.allclose(grads[0], fd, rtol=1e-5, atol=1e-9)
    # the CSR chain (Jt[k] ... Jt[0] seed) reproduces every layer-boundary gradient
    jts = cnn.network_jacobians_T(layers, acts, aux)
    chain = cnn.sparse_linear_scan(jts, grads[-1])
    n = len(layers)
    for k in range(n):
        assert np.allclose(chain[k], np.asarray(grads[n - 1 - k]).reshape(-1), rtol=1e-12, atol=1e-15)


def test_csr_product_is_structural_and_matches_dense_loops():
    rng = np.random.default_rng(2)
    a = sp.random(7, 9, density=0.3, random_state=1, format="csr")
    b = sp.random(9, 6, density=0.3, random_state=2, format="csr")
    b.data[:] = rng.standard_normal(b.nnz)
    a.data[:] = rng.standard_normal(a.nnz)
    # force an exact cancellation: the entry must stay, with value 0
    a = sp.csr_matrix(np.array([[1.0, 1.0, 0.0]]))
    b2 = sp.csr_matrix(np.array([[2.0, 0.0], [-2.0, 3.0], [0.0, 5.0]]))
    c = cnn.csr_product(a, b2)
    assert c.nnz == 2 and np.array_equal(c.indices, [0, 1]) and np.array_equal(c.data, [0.0, 3.0])
    a = sp.random(7, 9, density=0.3, random_state=3, format="csr")
    b = sp.random(9, 6, density=0.3, random_state=4, format="csr")
    c = cnn.csr_product(a, b)
    da, db = a.toarray(), b.toarray()
    dense = np.zeros((7, 6))
    pat = np.zeros((7, 6), bool)
    for i in range(7):
        for k in range(9):
            for j in range(6):
                if da[i, k] != 0 and db[k, j] != 0:
                    pat[i, j] = True
                dense[i, j] += da[i, k] * db[k, j]
    got_pat = np.zeros((7, 6), bool)
    for i in range(7):
        got_pat[i, c.indices[c.indptr[i]:c.indptr[i + 1]]] = True
    assert np.array_equal(got_pat, pat) and np.allclose(c.toarray(), dense)


def test_scan_step_flops_against_closed_forms_and_brute_force():
    """The static FLOP analysis (Sections 4.3 and 5.3).  Pins: with no up-sweep level the scan is the
    chain of matrix-vector products, 2 nnz each; fully dense operands give the textbook 2 m k n of a
    matrix product (and 2 m k of a matrix-vector product) at the places a tree over four elements
    must have them; on random patterns every matrix-matrix record equals a brute-force count of the
    index triples (i, k, j) with both entries stored."""
    dims = [5, 7, 6, 8, 4, 9, 3]                       # jts[k] is dims[k+1] x dims[k]
    jts = [sp.random(dims[k + 1], dims[k], density=0.4, random_state=k, format="csr") for k in range(6)]
    steps = cnn.scan_step_flops(jts, 0)
    assert [s[:3] for s in steps] == [("linear", j, "mv") for j in range(1, 6)]
    assert [s[3] for s in steps] == [2 * jts[k].nnz for k in range(5)]     # jts[5] only feeds the tail
    # dense chain over 1 + 5 elements with two levels: blocks [seed, J0, J1, J2] and [J3, J4]
    dense = [sp.csr_matrix(np.ones((dims[k + 1], dims[k]))) for k in range(5)]
    steps = cnn.scan_step_flops(dense, 2)
    d = dims
    kinds = {}
    for ph, lv, kd, fl in steps:
        kinds.setdefault((ph, lv, kd), []).append(fl)
    # up level 0: seed <> J0 (matrix-vector) and J1 <> J2 = J2 J1 (matrix-matrix, d3 x d2 x d1)
    assert kinds[("up", 0, "mv")] == [2 * d[1] * d[0]]
    assert kinds[("up", 0, "mm")] == [2 * d[3] * d[2] * d[1]]
    # up level 1: (J0 seed) <> (J2 J1): a d3 x d1 matrix applied to a vector
    assert kinds[("up", 1, "mv")] == [2 * d[3] * d[1]]
    # down: inside the first block the right half's prefix is the left half's total itself (the
    # block's own prefix is the identity: no product at level 1); the prefix of J2 is
    # (J0 seed) <> J1 (level 0: d2 x d1); in the second block [J3, J4] the prefix of J4 is
    # (block prefix) <> J3 (level 0: d4 x d3)
    assert kinds[("down", 0, "mv")] == [2 * d[2] * d[1], 2 * d[4] * d[3]]
    assert not any(k[0] == "linear" for k in kinds) and ("down", 1, "mv") not in kinds
    assert sum(len(v) for v in kinds.values()) == 5
    # brute force on random patterns, as many levels as the length allows
    steps = cnn.scan_step_flops(jts, 3)
    got_mm = sorted(f for ph, lv, kd, f in steps if kd == "mm")

    def triples(a, b):
        da, db = a.toarray() != 0, b.toarray() != 0
        return int(sum(1 for i in range(da.shape[0]) for k in range(da.shape[1]) for j in range(db.shape[1])
                       if da[i, k] and db[k, j]))
    # seven elements allow at most two levels: blocks [seed, J0, J1, J2] and [J3, J4, J5].  The
    # first block's total needs J1 <> J2 = J2 J1; in the second the prefix of J5 needs
    # J3 <> J4 = J4 J3; nothing else multiplies two matrices
    p21 = triples(jts[2], jts[1])
    p43 = triples(jts[4], jts[3])
    assert got_mm == sorted([2 * p21, 2 * p43])


def test_full_network_shapes_and_counts():
    layers, image, label = workloads.cnn_layers()
    kinds = [L.kind for L in layers]
    assert kinds.count("conv") == 8 and kinds.count("pool") == 5 and kinds.count("fc") == 3
    assert kinds.count("relu") == 10 and len(layers) == 26
    for L in layers:
        if L.weight is not None:
            keep = L.mask.mean()
            assert 0.0999 <= keep <= 0.1005 + 1.0 / L.mask.size
            assert np.all(L.weight[~L.mask] == 0)
