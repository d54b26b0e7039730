"""GPU parity: CSR Jacobian builders (bit-exact structure), SpMV, SpGEMM structure and the sparse scan."""
import numpy as np
import pytest
import scipy.sparse as sp

import workloads
from oracle import cnn as ocnn
from util import TOL, rel_err, to_gpu, to_np

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def bp():
    import torch
    assert torch.cuda.is_available()
    import paper_1907_10134_amd as lib
    return lib


def _assert_same_csr(got, ref, values=True):
    """got: binding CsrMatrix on the GPU; ref: scipy CSR from the oracle.  Index arrays bit-exact."""
    ref = sp.csr_matrix(ref)
    assert (got.rows, got.cols) == ref.shape
    assert np.array_equal(to_np(got.indptr), ref.indptr.astype(np.int32))
    assert np.array_equal(to_np(got.indices), ref.indices.astype(np.int32))
    if values:
        d = to_np(got.data)
        assert d.shape == ref.data.shape
        if d.size:
            assert rel_err(d, ref.data) <= 1e-6


def _rounded_forward(layers, image):
    """Oracle forward, then every activation rounded to fp32 once: both sides decide ReLU masks and
    pooling winners on exactly these values."""
    acts, _ = ocnn.forward(layers, image)
    acts32 = [np.asarray(a, np.float32) for a in acts]
    aux = [ocnn.maxpool2x2_fast(acts32[i].reshape(L.in_shape))[1] if L.kind == "pool" else None
           for i, L in enumerate(layers)]
    return acts32, aux


def _gpu_jacobians(bp, layers, acts32):
    """Transposed Jacobians in scan order (last layer first), built on the GPU."""
    out = []
    for i in range(len(layers) - 1, -1, -1):
        L = layers[i]
        if L.kind == "conv":
            m = bp.csr_conv3x3(to_gpu(L.weight), to_gpu(L.mask.astype(np.uint8)), L.in_shape[1], L.in_shape[2])
        elif L.kind == "fc":
            m = bp.csr_linear(to_gpu(L.weight), to_gpu(L.mask.astype(np.uint8)))
        elif L.kind == "relu":
            m = bp.csr_relu(to_gpu(acts32[i].reshape(-1)))
        else:
            m = bp.csr_maxpool2x2(to_gpu(acts32[i].reshape(L.in_shape)))
        out.append(m)
    return out


@pytest.mark.parametrize("ci,co,h,w,keep", [(2, 3, 4, 5, 0.6), (1, 1, 1, 1, 1.0), (3, 2, 2, 2, 0.5), (1, 2, 1, 4, 1.0),
                                            (3, 64, 32, 32, 1.0), (5, 70, 6, 3, 0.1), (4, 8, 3, 3, 0.0)])
def test_conv_builder_bit_exact(bp, ci, co, h, w, keep):
    rng = np.random.default_rng(ci * 100 + co)
    wt = rng.standard_normal((co, ci, 3, 3)).astype(np.float32)
    mask = rng.random((co, ci, 3, 3)) < keep if keep < 1.0 else None
    ref = ocnn.conv_jacobian_T(wt, mask, h, w)
    got = bp.csr_conv3x3(to_gpu(wt), None if mask is None else to_gpu(mask.astype(np.uint8)), h, w)
    _assert_same_csr(got, ref)
    if mask is None:
        assert got.nnz == ci * co * (3 * h - 2) * (3 * w - 2)      # the count behind Table 1's example


def test_relu_pool_linear_builders_bit_exact(bp):
    rng = np.random.default_rng(1)
    x = rng.standard_normal((6, 8, 10)).astype(np.float32)
    x[0, :2, :2] = 0.0
    x[1, 2:4, 4:6] = 1.5           # ties: the first element of the window wins
    x[2] = np.maximum(x[2], 0)     # many zero ties, as after a ReLU
    _assert_same_csr(bp.csr_relu(to_gpu(x.reshape(-1))), ocnn.relu_jacobian_T(x))
    _, idx = ocnn.maxpool2x2(x)
    _assert_same_csr(bp.csr_maxpool2x2(to_gpu(x)), ocnn.pool_jacobian_T(idx, x.shape))
    w = rng.standard_normal((37, 70)).astype(np.float32)
    m = rng.random((37, 70)) < 0.3
    _assert_same_csr(bp.csr_linear(to_gpu(w), to_gpu(m.astype(np.uint8))), ocnn.fc_jacobian_T(w, m))
    _assert_same_csr(bp.csr_linear(to_gpu(w), None), ocnn.fc_jacobian_T(w, None))


def test_spmv_matches_scipy(bp):
    rng = np.random.default_rng(2)
    for rows, cols, dens in [(50, 70, 0.3), (1000, 300, 0.002), (7, 5, 1.0), (300, 4000, 0.05)]:
        a = sp.random(rows, cols, density=dens, random_state=rows, format="csr", dtype=np.float32)
        a.sort_indices()
        x = rng.standard_normal(cols).astype(np.float32)
        A = bp.CsrMatrix(rows, cols, to_gpu(a.indptr.astype(np.int32)), to_gpu(a.indices.astype(np.int32)),
                         to_gpu(a.data))
        y = to_np(bp.spmv(A, to_gpu(x)))
        ref = a.astype(np.float64) @ x.astype(np.float64)
        assert rel_err(y, ref) <= 1e-5 or np.max(np.abs(ref)) == 0


def _check_products(bp, plan, jts_ref):
    """Every planned CSR x CSR product: structure bit-exact against the oracle's structural product."""
    n = len(jts_ref)
    mats = list(jts_ref)
    for k in range(plan.num_products()):
        got, l, r = plan.product(k)
        ref = ocnn.csr_product(mats[l], mats[r])
        mats.append(ref)
        _assert_same_csr(got, ref, values=False)
        d = to_np(got.data)
        if d.size and np.max(np.abs(ref.data)) > 0:
            assert rel_err(d, ref.data) <= 1e-5
    return len(mats) - n


def _run_spscan(bp, jts, seed, up_levels, n, want_tail=True):
    import torch
    arena = torch.empty((1 << 30,), dtype=torch.uint8, device="cuda")
    plan = bp.SpscanPlan(jts, up_levels, arena)
    grads = [torch.full((m.rows,), float("nan"), dtype=torch.float32, device="cuda") for m in jts]
    if not want_tail:
        grads[-1] = None
    plan.run(jts, seed, grads)
    torch.cuda.synchronize()
    return plan, grads


@pytest.mark.parametrize("up_levels", [0, 1, 2, 3, 4, 9])
def test_spscan_tiny_network(bp, up_levels):
    layers, image, label = workloads.cnn_layers(conv_channels=(3, 4, 4), pool_after=(1, 3), fc=(6, 5),
                                                in_shape=(2, 8, 8), prune=0.5, seed=up_levels)
    acts32, aux = _rounded_forward(layers, image)
    grads_ref = ocnn.backward(layers, acts32, aux, label)
    jts_ref = ocnn.network_jacobians_T(layers, acts32, aux)
    jts = _gpu_jacobians(bp, layers, acts32)
    for g, r in zip(jts, jts_ref):
        _assert_same_csr(g, r)
    n = len(layers)
    seed = to_gpu(np.asarray(grads_ref[n], np.float32))
    plan, grads = _run_spscan(bp, jts, seed, up_levels, n, want_tail=(up_levels % 2 == 0))
    for k in range(n):
        if grads[k] is None:
            continue
        ref = np.asarray(grads_ref[n - 1 - k]).reshape(-1)
        assert rel_err(to_np(grads[k]), ref) <= TOL, (k, layers[n - 1 - k].kind)
    nprod = _check_products(bp, plan, jts_ref)
    assert (nprod == 0) == (up_levels == 0)
    mm, mv = plan.flops()
    assert (mm == 0) == (up_levels == 0) and mv > 0
    plan.close()


def test_spscan_one_shot_and_error_paths(bp):
    import torch
    layers, image, label = workloads.cnn_layers(conv_channels=(2,), pool_after=(1,), fc=(4, 3),
                                                in_shape=(1, 4, 4), prune=0.0, seed=3)
    acts32, aux = _rounded_forward(layers, image)
    grads_ref = ocnn.backward(layers, acts32, aux, label)
    jts = _gpu_jacobians(bp, layers, acts32)
    n = len(layers)
    seed = to_gpu(np.asarray(grads_ref[n], np.float32))
    grads = [torch.empty((m.rows,), dtype=torch.float32, device="cuda") for m in jts]
    ws = torch.empty((1 << 22,), dtype=torch.uint8, device="cuda")
    bp.spscan(jts, seed, grads, 2, ws)
    for k in range(n):
        assert rel_err(to_np(grads[k]), np.asarray(grads_ref[n - 1 - k]).reshape(-1)) <= TOL
    with pytest.raises(bp.BppsaError) as e:      # arena too small: reported, nothing half-done is returned
        bp.spscan(jts, seed, grads, 2, ws[:256])
    assert e.value.code == 3
    with pytest.raises(bp.BppsaError) as e:      # chain whose shapes do not compose
        bp.spscan([jts[0], jts[0]], seed, grads[:2], 0, ws)
    assert e.value.code == 2


@pytest.mark.parametrize("up_levels", [0, 2])
def test_spscan_config4_full_network(bp, up_levels):
    """configs[4]: the pruned VGG-11-style network on one 32x32x3 image, 26 transposed Jacobians."""
    layers, image, label = workloads.cnn_layers()
    acts32, aux = _rounded_forward(layers, image)
    grads_ref = ocnn.backward(layers, acts32, aux, label)
    jts_ref = ocnn.network_jacobians_T(layers, acts32, aux)
    jts = _gpu_jacobians(bp, layers, acts32)
    assert len(jts) == 26
    for g, r in zip(jts, jts_ref):
        _assert_same_csr(g, r)                       # all CSR index structures bit-exact
    n = len(layers)
    seed = to_gpu(np.asarray(grads_ref[n], np.float32))
    plan, grads = _run_spscan(bp, jts, seed, up_levels, n)
    for k in range(n):
        ref = np.asarray(grads_ref[n - 1 - k]).reshape(-1)
        assert rel_err(to_np(grads[k]), ref) <= TOL, (k, layers[n - 1 - k].kind)
    if up_levels:
        assert _check_products(bp, plan, jts_ref) > 0
    plan.close()


def _csr_to_gpu(bp, m):
    m = sp.csr_matrix(m)
    m.sort_indices()
    return bp.CsrMatrix(m.shape[0], m.shape[1], to_gpu(m.indptr.astype(np.int32)), to_gpu(m.indices.astype(np.int32)),
                        to_gpu(m.data.astype(np.float32)))


def _chain_with_one_product(bp, left, right, rng):
    """A five-matrix chain in scan order whose level-0 up-sweep forms exactly left * right as a live
    product: [D0, right, left, D3, D4] with small dense end pieces."""
    d0 = sp.csr_matrix(rng.standard_normal((right.shape[1], 3)).astype(np.float32))
    d3 = sp.csr_matrix(rng.standard_normal((5, left.shape[0])).astype(np.float32))
    d4 = sp.csr_matrix(rng.standard_normal((4, 5)).astype(np.float32))
    return [d0, sp.csr_matrix(right), sp.csr_matrix(left), d3, d4]


@pytest.mark.parametrize("case", ["wave", "block_dense", "block_staged", "block_global"])
def test_spgemm_numeric_kinds_match_oracle_and_repeat_bit_identically(bp, case):
    """The numeric phase of the CSR x CSR product, one case per kernel that sums terms: values against
    the oracle's product, and the same bits on every run (each value is formed by one wave in a fixed
    order).  A workgroup takes at most 64 KiB of LDS: 4 bytes per column of the right operand, or 4
    bytes per entry of the longest row plus 8 bytes per 32 columns; block_global is a product that
    fits neither, which is what sends a row to accumulators in global memory."""
    import torch
    rng = np.random.default_rng(len(case))
    if case == "wave":                      # short rows with real sums
        left = sp.random(300, 200, density=0.1, random_state=1, format="csr", dtype=np.float32)
        right = sp.random(200, 500, density=0.05, random_state=2, format="csr", dtype=np.float32)
    elif case == "block_dense":             # rows longer than 1024 entries, one accumulator per column fits
        left = sp.random(40, 300, density=0.3, random_state=3, format="csr", dtype=np.float32)
        right = sp.random(300, 9000, density=0.02, random_state=4, format="csr", dtype=np.float32)
    elif case == "block_staged":            # too many columns for that, but the longest row fits
        left = sp.random(30, 200, density=0.2, random_state=5, format="csr", dtype=np.float32)
        right = sp.random(200, 20000, density=0.005, random_state=6, format="csr", dtype=np.float32)
    else:                                   # neither fits
        left = sp.random(6, 120, density=0.9, random_state=7, format="csr", dtype=np.float32)
        right = sp.random(120, 20000, density=0.03, random_state=8, format="csr", dtype=np.float32)
    left.sort_indices()
    right.sort_indices()
    ref = ocnn.csr_product(left, right)
    longest = int(np.max(np.diff(ref.indptr)))
    dense_bytes = 4 * right.shape[1]
    ranked_bytes = 4 * longest + 8 * ((right.shape[1] + 31) // 32)
    if case == "wave":
        assert longest <= 1024 and ref.nnz < left.nnz * right.nnz
    elif case == "block_dense":
        assert longest > 1024 and dense_bytes <= 65536 and 4 * dense_bytes <= 5 * ranked_bytes
    elif case == "block_staged":
        assert longest > 1024 and dense_bytes > 65536 and ranked_bytes <= 65536
    else:
        assert longest > 1024 and dense_bytes > 65536 and ranked_bytes > 65536
    chain = _chain_with_one_product(bp, left, right, rng)
    jts = [_csr_to_gpu(bp, m) for m in chain]
    seed = to_gpu(rng.standard_normal(chain[0].shape[1]).astype(np.float32))
    arena = torch.empty((1 << 28,), dtype=torch.uint8, device="cuda")
    plan = bp.SpscanPlan(jts, 1, arena)
    grads = [torch.empty((m.rows,), dtype=torch.float32, device="cuda") for m in jts]
    found = None
    runs = []
    for _ in range(3):
        plan.run(jts, seed, grads)
        torch.cuda.synchronize()
        for k in range(plan.num_products()):
            got, l, r = plan.product(k)
            if (l, r) == (2, 1):
                found = got
                runs.append(to_np(got.data).copy())
    assert found is not None, "the chain did not produce left * right"
    _assert_same_csr(found, ref, values=False)
    assert rel_err(runs[0], ref.data) <= 1e-5
    assert all(np.array_equal(runs[0], r) for r in runs[1:])
    # and the gradients of the whole chain against the oracle's serial sparse scan
    g_ref = ocnn.sparse_linear_scan([sp.csr_matrix(m, dtype=np.float64) for m in chain], to_np(seed).astype(np.float64))
    for k in range(len(chain)):
        assert rel_err(to_np(grads[k]), g_ref[k]) <= TOL
    plan.close()


def test_spscan_config4_products_repeat_bit_identically(bp):
    """configs[4] with two up-sweep levels: the values of every CSR x CSR product are the same bits
    on two runs."""
    import torch
    layers, image, label = workloads.cnn_layers()
    acts32, aux = _rounded_forward(layers, image)
    jts = _gpu_jacobians(bp, layers, acts32)
    seed = to_gpu(np.random.default_rng(0).standard_normal(jts[0].cols).astype(np.float32))
    arena = torch.empty((1 << 30,), dtype=torch.uint8, device="cuda")
    plan = bp.SpscanPlan(jts, 2, arena)
    grads = [torch.empty((m.rows,), dtype=torch.float32, device="cuda") for m in jts]
    snaps = []
    for _ in range(2):
        plan.run(jts, seed, grads)
        torch.cuda.synchronize()
        snaps.append([plan.product(k)[0].data.clone() for k in range(plan.num_products())] + [g.clone() for g in grads])
        for k in range(plan.num_products()):
            plan.product(k)[0].data.zero_()
    assert all(torch.equal(a, b) for a, b in zip(*snaps))
    plan.close()


def _step_series(steps):
    """(phase, level, kind) -> sorted FLOP counts, leaving out the inclusive tail."""
    out = {}
    for s in steps:
        if s["phase"] != "tail":
            out.setdefault((s["phase"], s["level"], s["kind"]), []).append(s["flops"])
    return {k: sorted(v) for k, v in out.items()}


@pytest.mark.parametrize("up_levels", [0, 1, 2, 3])
def test_plan_step_flops_match_the_oracle_analysis(bp, up_levels):
    """bppsa_spscan_plan_step_flops against counts the oracle derives from its own structural
    products (Sections 4.3 and 5.3): the same products at the same tree levels, each with the same
    number of multiply-adds, and totals that agree with bppsa_spscan_plan_flops."""
    import torch
    layers, image, label = workloads.cnn_layers(conv_channels=(3, 4, 4), pool_after=(1, 3), fc=(6, 5),
                                                in_shape=(2, 8, 8), prune=0.5, seed=11)
    acts32, aux = _rounded_forward(layers, image)
    jts_ref = ocnn.network_jacobians_T(layers, acts32, aux)
    jts = _gpu_jacobians(bp, layers, acts32)
    arena = torch.empty((1 << 26,), dtype=torch.uint8, device="cuda")
    plan = bp.SpscanPlan(jts, up_levels, arena)
    steps = plan.steps()
    ref = [{"phase": ph, "level": lv, "kind": kd, "flops": fl} for ph, lv, kd, fl in ocnn.scan_step_flops(jts_ref, up_levels)]
    assert _step_series(steps) == _step_series(ref)
    assert steps[-1]["phase"] == "tail" and steps[-1]["flops"] == 2 * jts_ref[-1].nnz
    mm, mv = plan.flops()
    assert mm == sum(s["flops"] for s in ref if s["kind"] == "mm")
    assert mv == sum(s["flops"] for s in ref if s["kind"] == "mv")
    assert sum(1 for s in steps if s["kind"] == "mm") == plan.num_products()
    plan.close()


def test_plan_step_flops_config4_two_levels(bp):
    """configs[4] with the two up-sweep levels of Section 5.3: per-level FLOP series against the oracle."""
    import torch
    layers, image, label = workloads.cnn_layers()
    acts32, aux = _rounded_forward(layers, image)
    jts_ref = ocnn.network_jacobians_T(layers, acts32, aux)
    jts = _gpu_jacobians(bp, layers, acts32)
    arena = torch.empty((1 << 30,), dtype=torch.uint8, device="cuda")
    plan = bp.SpscanPlan(jts, 2, arena)
    ref = [{"phase": ph, "level": lv, "kind": kd, "flops": fl} for ph, lv, kd, fl in ocnn.scan_step_flops(jts_ref, 2)]
    assert _step_series(plan.steps()) == _step_series(ref)
    plan.close()


def test_plan_cache_reuses_the_symbolic_phase(bp):
    """A second plan for the same patterns comes from the cache: no product structure is computed
    again (counted by the library), the structures are the same device arrays, and its results
    equal those of an uncached plan; other patterns, or another level count, miss."""
    import torch
    layers, image, label = workloads.cnn_layers(conv_channels=(3, 4, 4), pool_after=(1, 3), fc=(6, 5),
                                                in_shape=(2, 8, 8), prune=0.5, seed=21)
    acts32, aux = _rounded_forward(layers, image)
    grads_ref = ocnn.backward(layers, acts32, aux, label)
    jts_ref = ocnn.network_jacobians_T(layers, acts32, aux)
    jts = _gpu_jacobians(bp, layers, acts32)
    n = len(layers)
    seed = to_gpu(np.asarray(grads_ref[n], np.float32))
    cache = bp.SpscanCache()
    assert cache.stats() == (0, 0, 0, 0)
    arenas = [torch.empty((1 << 26,), dtype=torch.uint8, device="cuda") for _ in range(3)]
    first = bp.SpscanPlan(jts, 2, arenas[0], cache=cache)
    hits, misses, computed, held = cache.stats()
    assert (hits, misses) == (0, 1) and computed == first.num_products() > 0 and held > 0
    second = bp.SpscanPlan(jts, 2, arenas[1], cache=cache)
    assert cache.stats() == (1, 1, computed, held)
    plain = bp.SpscanPlan(jts, 2, arenas[2])
    assert second.arena_used() < plain.arena_used()          # structures are not in the arena
    assert second.steps() == first.steps() == plain.steps()
    for k in range(first.num_products()):
        a, b = first.product(k)[0], second.product(k)[0]
        assert a.indices.data_ptr() == b.indices.data_ptr() and a.data.data_ptr() != b.data.data_ptr()
    outs = []
    for plan in (first, second, plain):
        grads = [torch.full((m.rows,), float("nan"), dtype=torch.float32, device="cuda") for m in jts]
        plan.run(jts, seed, grads)
        torch.cuda.synchronize()
        outs.append(grads)
    for k in range(n):
        assert rel_err(to_np(outs[0][k]), np.asarray(grads_ref[n - 1 - k]).reshape(-1)) <= TOL
        assert torch.equal(outs[0][k], outs[1][k]) and torch.equal(outs[0][k], outs[2][k])
    _check_products(bp, second, jts_ref)
    # same shapes and entry counts, one pattern changed: a fully connected layer whose mask is
    # rotated by one input, so only the fingerprint of the index arrays can tell the difference
    moved = list(jts)
    fc_at = min(i for i, L in enumerate(reversed(layers)) if L.kind == "fc" and not L.mask.all())
    L = list(reversed(layers))[fc_at]
    moved[fc_at] = bp.csr_linear(to_gpu(L.weight), to_gpu(np.roll(L.mask, 1, axis=1).astype(np.uint8)))
    assert moved[fc_at].nnz == jts[fc_at].nnz and not torch.equal(moved[fc_at].indices, jts[fc_at].indices)
    third = bp.SpscanPlan(moved, 2, arenas[2], cache=cache)
    assert cache.stats()[:2] == (1, 2)
    third.close()
    fourth = bp.SpscanPlan(jts, 1, arenas[2], cache=cache)      # another schedule: its own entry
    assert cache.stats()[0] == 1
    for p in (first, second, plain, fourth):
        p.close()
    cache.close()


CONV_GEOMETRIES = [  # (ci, co, h, w, kh, kw, stride, padding, dilation, keep)
    (2, 3, 5, 6, 3, 3, (1, 1), (1, 1), (1, 1), 0.7),
    (1, 2, 7, 5, 5, 3, (2, 1), (2, 0), (1, 1), 1.0),
    (2, 2, 8, 8, 2, 2, (2, 2), (0, 0), (1, 1), 0.5),
    (1, 1, 9, 7, 3, 2, (3, 2), (1, 1), (2, 3), 1.0),
    (3, 1, 4, 4, 1, 1, (1, 1), (0, 0), (1, 1), 0.6),
    (1, 2, 6, 6, 4, 4, (1, 1), (3, 3), (1, 1), 0.8),
    (3, 16, 17, 19, 5, 5, (2, 2), (2, 2), (1, 1), 0.3),      # 400 candidates per row: several wave passes
    (4, 8, 12, 10, 3, 3, (1, 2), (2, 1), (2, 1), 0.5),
    (2, 40, 6, 6, 3, 3, (1, 1), (0, 0), (1, 1), 0.0),        # everything pruned: an empty matrix
]


@pytest.mark.parametrize("ci,co,h,w,kh,kw,stride,padding,dilation,keep", CONV_GEOMETRIES)
def test_generic_conv_builder_bit_exact(bp, ci, co, h, w, kh, kw, stride, padding, dilation, keep):
    """bppsa_csr_conv2d_* against the oracle's entry-by-entry Jacobian: row pointers, column indices
    and values, all bit-exact (no entry is a sum)."""
    rng = np.random.default_rng(ci * 100 + co * 10 + kh)
    wt = rng.standard_normal((co, ci, kh, kw)).astype(np.float32)
    mask = rng.random(wt.shape) < keep
    ref = ocnn.conv2d_jacobian_T(wt, mask, h, w, stride, padding, dilation)
    got = bp.csr_conv2d(to_gpu(wt), to_gpu(mask.astype(np.uint8)), h, w, stride, padding, dilation)
    assert (got.rows, got.cols) == ref.shape
    _assert_same_csr(got, ref)


def test_generic_conv_builder_equals_the_3x3_builder(bp):
    import torch
    rng = np.random.default_rng(77)
    wt = to_gpu(rng.standard_normal((64, 3, 3, 3)).astype(np.float32))
    mask = to_gpu((rng.random((64, 3, 3, 3)) < 0.4).astype(np.uint8))
    a = bp.csr_conv3x3(wt, mask, 32, 32)
    b = bp.csr_conv2d(wt, mask, 32, 32, (1, 1), (1, 1), (1, 1))
    assert torch.equal(a.indptr, b.indptr) and torch.equal(a.indices, b.indices) and torch.equal(a.data, b.data)
    full = bp.csr_conv2d(wt, None, 32, 32, (1, 1), (1, 1), (1, 1))
    assert full.nnz == 1696512                                 # Table 1's first convolution of VGG-11


def test_spscan_through_strided_and_dilated_convolutions(bp):
    """A chain conv(5x5, stride 2) -> ReLU -> conv(3x3, dilation 2) -> ReLU -> fc: the sparse scan
    over the generic builder's Jacobians against the oracle's matrix-vector chain on its own."""
    import torch
    rng = np.random.default_rng(12)
    w1 = rng.standard_normal((4, 2, 5, 5)).astype(np.float32)
    w2 = rng.standard_normal((3, 4, 3, 3)).astype(np.float32)
    m1, m2 = rng.random(w1.shape) < 0.6, rng.random(w2.shape) < 0.6
    h0 = w0 = 15
    h1 = ocnn.conv2d_out_size(h0, 5, 2, 2, 1)                 # 8
    h2 = ocnn.conv2d_out_size(h1, 3, 1, 2, 2)                 # 8
    wf = rng.standard_normal((5, 3 * h2 * h2)).astype(np.float32)
    mf = rng.random(wf.shape) < 0.5
    a1 = rng.standard_normal(4 * h1 * h1).astype(np.float32)
    a2 = rng.standard_normal(3 * h2 * h2).astype(np.float32)
    ref = [ocnn.fc_jacobian_T(wf, mf), ocnn.relu_jacobian_T(a2),
           ocnn.conv2d_jacobian_T(w2, m2, h1, h1, (1, 1), (2, 2), (2, 2)), ocnn.relu_jacobian_T(a1),
           ocnn.conv2d_jacobian_T(w1, m1, h0, w0, (2, 2), (2, 2), (1, 1))]
    jts = [bp.csr_linear(to_gpu(wf), to_gpu(mf.astype(np.uint8))), bp.csr_relu(to_gpu(a2)),
           bp.csr_conv2d(to_gpu(w2), to_gpu(m2.astype(np.uint8)), h1, h1, (1, 1), (2, 2), (2, 2)),
           bp.csr_relu(to_gpu(a1)),
           bp.csr_conv2d(to_gpu(w1), to_gpu(m1.astype(np.uint8)), h0, w0, (2, 2), (2, 2), (1, 1))]
    for g, r in zip(jts, ref):
        _assert_same_csr(g, r)
    seed = rng.standard_normal(5).astype(np.float32)
    want = ocnn.sparse_linear_scan(ref, seed)
    for U in (0, 1, 2):
        arena = torch.empty((1 << 26,), dtype=torch.uint8, device="cuda")
        plan = bp.SpscanPlan(jts, U, arena)
        grads = [torch.empty((m.rows,), dtype=torch.float32, device="cuda") for m in jts]
        plan.run(jts, to_gpu(seed), grads)
        torch.cuda.synchronize()
        for k in range(len(jts)):
            assert rel_err(to_np(grads[k]), want[k]) <= TOL, (U, k)
        plan.close()
