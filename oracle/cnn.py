"""fp64 oracle: pruned VGG-11-style CNN, textbook backward and CSR Jacobians.  TEST INFRASTRUCTURE.

Two independent things live here.

1. `forward` / `backward`: the network of Section 4.3 (3x3 convolutions with
   padding 1 as cross-correlation, ReLU, 2x2/2 max-pooling, fully connected
   layers, softmax cross-entropy) and its per-layer backward rules written
   without any sparse matrix: Eq. 3 of Section 2.1 applied layer by layer.
   This is what the sparse scan must reproduce.

2. `jacobian_T_csr`: the transposed Jacobian of one layer, (d out / d in)^T with
   rows = input elements and columns = output elements (Appendix D), written
   from the derivative of the layer's definition entry by entry and put into
   canonical CSR (row pointers, ascending column indices).  Readings of the
   appendix taken here: only in-image neighbours are stored for a convolution
   (which is what reproduces the sparsity and memory figures of Section 3.3 and
   Table 1); pruned weights are structurally absent (decided by the mask, never
   by the value); ReLU keeps its full diagonal with data in {0, 1}; max-pooling
   stores one unit entry per output at the first maximum of its window in
   row-major window order.

`conv2d` / `conv2d_jacobian_T` are the same pair for a convolution with any kernel size, stride,
zero padding and dilation (the generic routine Appendix D.1's footnote leaves open), written as
the definition's loops.

`csr_product` is the structural product: its pattern is the boolean product of
the patterns (explicit zeros propagate, nothing is dropped by value).

Pins (tests/test_oracle_cnn.py): Table 1's sparsity values and the 768 MB /
6.5 MB figures of Section 3.3; Algorithm 2's interior row lengths (6 c_o, 9 c_o);
dense Jacobians obtained by pushing unit impulses / finite differences through
`forward` on tiny shapes; finite differences of the loss for `backward`;
`CSR -> dense . g` equals `backward`'s layer rule; dense triple loops for
`csr_product`; `conv2d` against SciPy's 2-D correlation where stride and dilation are 1 and
against `conv3x3`; `conv2d_jacobian_T` against unit impulses pushed through `conv2d` and, for the
3x3 / padding 1 case, against `conv_jacobian_T` (itself pinned to Table 1).
"""
from __future__ import annotations

import numpy as np
import scipy.sparse as sp


def _f64(a):
    return np.asarray(a, dtype=np.float64)


# ---------------------------------------------------------------------------
# layer definitions (forward)
# ---------------------------------------------------------------------------

def conv3x3(x, w, b=None):
    """Cross-correlation, 3x3, padding 1, stride 1.  x [ci,h,w], w [co,ci,3,3] -> [co,h,w]."""
    x, w = _f64(x), _f64(w)
    ci, h, wd = x.shape
    co = w.shape[0]
    xp = np.zeros((ci, h + 2, wd + 2))
    xp[:, 1:-1, 1:-1] = x
    out = np.zeros((co, h, wd))
    for ky in range(3):
        for kx in range(3):
            out += np.einsum("oc,chw->ohw", w[:, :, ky, kx], xp[:, ky:ky + h, kx:kx + wd])
    if b is not None:
        out += _f64(b)[:, None, None]
    return out


def maxpool2x2(x):
    """2x2 window, stride 2.  Returns (out [c,h/2,w/2], pool_indices [c,h/2,w/2]).

    pool_indices holds the flat index (y * w + x) within the channel plane of the
    first maximum in row-major window order.
    """
    x = _f64(x)
    c, h, w = x.shape
    ho, wo = h // 2, w // 2
    out = np.zeros((c, ho, wo))
    idx = np.zeros((c, ho, wo), dtype=np.int64)
    for ch in range(c):
        for y in range(ho):
            for xx in range(wo):
                best, bi = -np.inf, -1
                for dy in range(2):
                    for dx in range(2):
                        v = x[ch, 2 * y + dy, 2 * xx + dx]
                        if v > best:
                            best, bi = v, (2 * y + dy) * w + (2 * xx + dx)
                out[ch, y, xx] = best
                idx[ch, y, xx] = bi
    return out, idx


def maxpool2x2_fast(x):
    """Vectorised equivalent of `maxpool2x2` (same tie rule), for full-size layers."""
    x = _f64(x)
    c, h, w = x.shape
    ho, wo = h // 2, w // 2
    win = x[:, :2 * ho, :2 * wo].reshape(c, ho, 2, wo, 2).transpose(0, 1, 3, 2, 4).reshape(c, ho, wo, 4)
    k = np.argmax(win, axis=-1)                      # first maximum, window order (dy, dx)
    out = np.take_along_axis(win, k[..., None], axis=-1)[..., 0]
    yy = 2 * np.arange(ho)[None, :, None] + k // 2
    xx = 2 * np.arange(wo)[None, None, :] + k % 2
    return out, yy * w + xx


def forward(layers, image):
    """Activations at every layer boundary: acts[0] = image, acts[i+1] = layer i output.

    Also returns aux[i] (pool_indices for pooling layers, else None).
    """
    acts = [_f64(image)]
    aux = []
    for L in layers:
        x = acts[-1]
        if L.kind == "conv":
            y, a = conv3x3(x.reshape(L.in_shape), L.weight, L.bias), None
        elif L.kind == "relu":
            y, a = np.maximum(x, 0.0), None
        elif L.kind == "pool":
            y, a = maxpool2x2_fast(x.reshape(L.in_shape))
        elif L.kind == "fc":
            y, a = _f64(L.weight) @ x.reshape(-1) + _f64(L.bias), None
        else:
            raise ValueError(L.kind)
        acts.append(y)
        aux.append(a)
    return acts, aux


def loss_and_seed(logits, label):
    z = _f64(logits).reshape(-1)
    m = z.max()
    lse = m + np.log(np.exp(z - m).sum())
    p = np.exp(z - lse)
    p[label] -= 1.0
    return float(lse - z[label]), p


# ---------------------------------------------------------------------------
# textbook backward, no sparse matrices
# ---------------------------------------------------------------------------

def layer_backward(L, x_in, aux, g_out):
    """Gradient w.r.t. the layer input given the gradient w.r.t. its output."""
    g_out = _f64(g_out)
    if L.kind == "conv":
        co, h, w = L.out_shape
        g = g_out.reshape(co, h, w)
        gp = np.zeros((co, h + 2, w + 2))
        gp[:, 1:-1, 1:-1] = g
        wgt = _f64(L.weight)
        gin = np.zeros(L.in_shape)
        # in[ci, y, x] feeds out[co, y - ky + 1, x - kx + 1] through w[co, ci, ky, kx]
        for ky in range(3):
            for kx in range(3):
                gin += np.einsum("oc,ohw->chw", wgt[:, :, ky, kx], gp[:, 2 - ky:2 - ky + h, 2 - kx:2 - kx + w])
        return gin
    if L.kind == "relu":
        return g_out.reshape(np.shape(x_in)) * (_f64(x_in) > 0)
    if L.kind == "pool":
        c, h, w = L.in_shape
        gin = np.zeros((c, h * w))
        idx = aux.reshape(c, -1)
        g = g_out.reshape(c, -1)
        for ch in range(c):
            gin[ch, idx[ch]] = g[ch]          # windows do not overlap: plain scatter
        return gin.reshape(c, h, w)
    if L.kind == "fc":
        return _f64(L.weight).T @ g_out.reshape(-1)
    raise ValueError(L.kind)


def backward(layers, acts, aux, label):
    """grads[i] = dL/d acts[i] for i = 0..len(layers), by Eq. 3 from the last layer down."""
    _, seed = loss_and_seed(acts[-1], label)
    grads = [None] * (len(layers) + 1)
    grads[len(layers)] = seed
    for i in range(len(layers) - 1, -1, -1):
        grads[i] = layer_backward(layers[i], acts[i], aux[i], grads[i + 1])
    return grads


# ---------------------------------------------------------------------------
# transposed Jacobians in canonical CSR
# ---------------------------------------------------------------------------

def _canonical(rows, cols, vals, shape):
    """COO triples without duplicates -> CSR with ascending column indices."""
    order = np.lexsort((cols, rows))
    rows, cols, vals = rows[order], cols[order], vals[order]
    indptr = np.zeros(shape[0] + 1, dtype=np.int64)
    np.add.at(indptr, rows + 1, 1)
    indptr = np.cumsum(indptr)
    m = sp.csr_matrix((vals.astype(np.float64), cols.astype(np.int32), indptr.astype(np.int32)), shape=shape)
    return m


def conv_jacobian_T(w, mask, h, wd):
    """rows (ci, y, x), columns (co, y + dy, x + dx) for in-image neighbours; value w[co, ci, 1-dy, 1-dx]."""
    w = _f64(w)
    co, ci = w.shape[:2]
    mask = np.ones(w.shape, bool) if mask is None else np.asarray(mask, bool)
    rows, cols, vals = [], [], []
    ys, xs = np.meshgrid(np.arange(h), np.arange(wd), indexing="ij")
    for dy in (-1, 0, 1):
        for dx in (-1, 0, 1):
            ok = (ys + dy >= 0) & (ys + dy < h) & (xs + dx >= 0) & (xs + dx < wd)
            y0, x0 = ys[ok], xs[ok]
            src = y0 * wd + x0                       # input pixel
            dst = (y0 + dy) * wd + (x0 + dx)         # output pixel it feeds through tap (1-dy, 1-dx)
            o, c = np.nonzero(mask[:, :, 1 - dy, 1 - dx])   # kept (co, ci) pairs of this tap
            if o.size == 0 or src.size == 0:
                continue
            rows.append((c[:, None] * (h * wd) + src[None, :]).reshape(-1))
            cols.append((o[:, None] * (h * wd) + dst[None, :]).reshape(-1))
            vals.append(np.repeat(w[o, c, 1 - dy, 1 - dx], src.size))
    if not rows:
        return sp.csr_matrix((ci * h * wd, co * h * wd))
    return _canonical(np.concatenate(rows), np.concatenate(cols), np.concatenate(vals),
                      (ci * h * wd, co * h * wd))


def conv2d_out_size(n, k, stride, pad, dil):
    """Number of output positions along one axis of a convolution (0 if the kernel does not fit)."""
    span = n + 2 * pad - dil * (k - 1) - 1
    return span // stride + 1 if span >= 0 else 0


def conv2d(x, w, stride=(1, 1), padding=(0, 0), dilation=(1, 1)):
    """Cross-correlation with any kernel size, stride, zero padding and dilation, from its definition:
    out[o, oy, ox] = sum_{c, ky, kx} w[o, c, ky, kx] x[c, oy sh - ph + ky dh, ox sw - pw + kx dw]."""
    x, w = _f64(x), _f64(w)
    ci, h, wd = x.shape
    co, _, kh, kw = w.shape
    (sh, sw), (ph, pw), (dh, dw) = stride, padding, dilation
    oh, ow = conv2d_out_size(h, kh, sh, ph, dh), conv2d_out_size(wd, kw, sw, pw, dw)
    out = np.zeros((co, oh, ow))
    for oy in range(oh):
        for ox in range(ow):
            for ky in range(kh):
                for kx in range(kw):
                    y, xx = oy * sh - ph + ky * dh, ox * sw - pw + kx * dw
                    if 0 <= y < h and 0 <= xx < wd:
                        out[:, oy, ox] += w[:, :, ky, kx] @ x[:, y, xx]
    return out


def conv2d_jacobian_T(w, mask, h, wd, stride=(1, 1), padding=(0, 0), dilation=(1, 1)):
    """Transposed Jacobian of `conv2d` (the generic routine the footnote of Appendix D.1 leaves open):
    rows (c, y, x), columns (o, oy, ox); entry w[o, c, ky, kx] wherever y = oy sh - ph + ky dh and
    x = ox sw - pw + kx dw for a kept (mask) weight.  One input/output pair meets through at most
    one tap, so no entry is a sum.  Canonical CSR, pruned weights structurally absent."""
    w = _f64(w)
    co, ci, kh, kw = w.shape
    mask = np.ones(w.shape, bool) if mask is None else np.asarray(mask, bool)
    (sh, sw), (ph, pw), (dh, dw) = stride, padding, dilation
    oh, ow = conv2d_out_size(h, kh, sh, ph, dh), conv2d_out_size(wd, kw, sw, pw, dw)
    rows, cols, vals = [], [], []
    for o in range(co):
        for c in range(ci):
            for ky in range(kh):
                for kx in range(kw):
                    if not mask[o, c, ky, kx]:
                        continue
                    for oy in range(oh):
                        y = oy * sh - ph + ky * dh
                        if not 0 <= y < h:
                            continue
                        for ox in range(ow):
                            x = ox * sw - pw + kx * dw
                            if 0 <= x < wd:
                                rows.append((c * h + y) * wd + x)
                                cols.append((o * oh + oy) * ow + ox)
                                vals.append(w[o, c, ky, kx])
    shape = (ci * h * wd, co * oh * ow)
    if not rows:
        return sp.csr_matrix(shape)
    return _canonical(np.asarray(rows), np.asarray(cols), np.asarray(vals), shape)


def relu_jacobian_T(x):
    x = _f64(x).reshape(-1)
    d = x.size
    return sp.csr_matrix(((x > 0).astype(np.float64), np.arange(d, dtype=np.int32),
                          np.arange(d + 1, dtype=np.int32)), shape=(d, d))


def pool_jacobian_T(pool_indices, in_shape):
    c, h, w = in_shape
    ho, wo = h // 2, w // 2
    idx = np.asarray(pool_indices).reshape(c, ho * wo)
    rows = (np.arange(c)[:, None] * h * w + idx).reshape(-1)
    cols = np.arange(c * ho * wo)
    return _canonical(rows, cols, np.ones(rows.size), (c * h * w, c * ho * wo))


def fc_jacobian_T(w, mask):
    w = _f64(w)
    mask = np.ones(w.shape, bool) if mask is None else np.asarray(mask, bool)
    j, i = np.nonzero(mask)                    # out index j, in index i
    return _canonical(i, j, w[j, i], (w.shape[1], w.shape[0]))


def jacobian_T_csr(L, x_in, aux):
    if L.kind == "conv":
        return conv_jacobian_T(L.weight, L.mask, L.in_shape[1], L.in_shape[2])
    if L.kind == "relu":
        return relu_jacobian_T(x_in)
    if L.kind == "pool":
        return pool_jacobian_T(aux, L.in_shape)
    if L.kind == "fc":
        return fc_jacobian_T(L.weight, L.mask)
    raise ValueError(L.kind)


def network_jacobians_T(layers, acts, aux):
    """Transposed Jacobians in scan order: element 0 belongs to the last layer."""
    return [jacobian_T_csr(layers[i], acts[i], aux[i]) for i in range(len(layers) - 1, -1, -1)]


# ---------------------------------------------------------------------------
# structural CSR product and the sparse linear scan
# ---------------------------------------------------------------------------

def csr_product(a, b):
    """a @ b keeping every structurally possible entry (pattern = boolean product)."""
    a = sp.csr_matrix(a)
    b = sp.csr_matrix(b)
    pa = sp.csr_matrix((np.ones(a.nnz), a.indices, a.indptr), shape=a.shape)
    pb = sp.csr_matrix((np.ones(b.nnz), b.indices, b.indptr), shape=b.shape)
    pat = (pa @ pb).tocsr()                     # counts >= 1 on the structural pattern
    pat.sort_indices()
    val = (a @ b).tocsr()                       # may have dropped entries that summed to zero
    val.sort_indices()
    data = np.zeros(pat.nnz)
    for i in range(pat.shape[0]):
        ps, pe = pat.indptr[i], pat.indptr[i + 1]
        vs, ve = val.indptr[i], val.indptr[i + 1]
        if ve > vs:
            pos = np.searchsorted(pat.indices[ps:pe], val.indices[vs:ve])
            data[ps + pos] = val.data[vs:ve]
    return sp.csr_matrix((data, pat.indices.astype(np.int32), pat.indptr.astype(np.int32)), shape=pat.shape)


def sparse_linear_scan(jts, seed):
    """grads[k] = Jt[k] Jt[k-1] ... Jt[0] seed, by matrix-vector products in order (Section 3.6)."""
    g = _f64(seed).reshape(-1)
    out = []
    for m in jts:
        g = sp.csr_matrix(m) @ g
        out.append(g)
    return out


def scan_step_flops(jts, up_levels):
    """Static FLOP analysis of the scan over CSR transposed Jacobians (Sections 4.3 and 5.3).

    Runs the tree scan of `oracle.scan.tree_scan` with `up_levels` up-sweep levels on the patterns
    of jts (scan order: jts[0] is the last layer's) and a vector in place of the seed, and returns
    one record per product of two non-identity operands, in the order the recursion meets them:
    (phase, level, kind, flops) with phase in {"up", "linear", "down"}, kind "mm" or "mv", and flops
    = 2 per multiply-add: for C = A B every stored entry (i, k) of A meets every stored entry of row
    k of B; for y = A x every stored entry of A is used once.  The product that would give the
    gradient of the first layer's input (the inclusive tail) is not part of the scan and not listed.
    """
    from . import scan as _scan
    mats = [sp.csr_matrix(m) for m in jts]
    steps = []

    def combine(x, y):                          # x <> y = y x
        if sp.issparse(x):
            return csr_product(y, x)
        return np.ones(y.shape[0])              # only the length of a vector matters here

    def on_step(phase, level, x, y):
        if sp.issparse(x):
            row_len = np.diff(x.indptr)
            flops = 2 * int(row_len[y.indices].sum())
            steps.append((phase, level, "mm", flops))
        else:
            steps.append((phase, level, "mv", 2 * int(y.nnz)))

    a = [np.ones(mats[0].shape[1])] + mats
    _scan.tree_scan(a, up_levels, combine=combine, is_matrix=sp.issparse, on_step=on_step)
    return steps
