"""GPU parity: GRU builder, scan and parameter gradients against the fp64 oracle."""
import numpy as np
import pytest

import workloads
from oracle import gru as ogru
from oracle import rnn as orn
from oracle import scan as oscan
from util import TOL, per_step_err, rel_err, to_gpu, to_np

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def bp():
    import torch
    assert torch.cuda.is_available()
    import paper_1907_10134_amd as lib
    return lib


def _dev(w):
    return {k: to_gpu(w[k]) for k in ("x", "w_ih", "w_hh", "b_ih", "b_hh", "w_out", "b_out", "labels")}


def _gpu_forward(bp, w, d):
    import torch
    h = torch.zeros((w["T"] + 1, w["B"], w["H"]), dtype=torch.float32, device="cuda")
    bp.forward(bp.GRU, d["x"], d["w_ih"], d["w_hh"], d["b_ih"], d["b_hh"], h)
    return h


SHAPES = [(6, 2, 3, 2), (9, 3, 20, 1), (5, 2, 33, 3), (20, 16, 64, 1), (7, 5, 128, 1), (1, 1, 1, 1), (3, 17, 8, 2),
          (9, 3, 128, 3), (11, 2, 128, 5), (300, 3, 128, 2)]


@pytest.mark.parametrize("T,B,H,I", SHAPES)
def test_gru_forward_matches_oracle(bp, T, B, H, I):
    w = workloads.gru_inputs(T, B, H, I, 11, seed=T + H, audio=False)
    h = _gpu_forward(bp, w, _dev(w))
    ref = ogru.forward(w["x"], w["w_ih"], w["w_hh"], w["b_ih"], w["b_hh"])
    assert rel_err(to_np(h), ref) <= 1e-5


@pytest.mark.parametrize("T,B,H,I", SHAPES)
def test_gru_build_jacobians(bp, T, B, H, I):
    w = workloads.gru_inputs(T, B, H, I, 11, seed=2 * T + H, audio=False)
    d = _dev(w)
    h32 = ogru.forward(w["x"], w["w_ih"], w["w_hh"], w["b_ih"], w["b_hh"]).astype(np.float32)
    Jt = bp.build_jacobians(bp.GRU, to_gpu(h32), d["x"], d["w_ih"], d["w_hh"], d["b_ih"], d["b_hh"])
    ref = ogru.jacobians_T(h32, w["x"], w["w_ih"], w["w_hh"], w["b_ih"], w["b_hh"])
    assert rel_err(to_np(Jt), ref) <= 2e-6


@pytest.mark.parametrize("T,B,H,I", SHAPES + [(300, 4, 20, 2)])
def test_gru_param_grads(bp, T, B, H, I):
    w = workloads.gru_inputs(T, B, H, I, 11, seed=3 * T + H, audio=False)
    d = _dev(w)
    args = (w["w_ih"], w["w_hh"], w["b_ih"], w["b_hh"])
    h = ogru.forward(w["x"], *args)
    _, seed = orn.head(h[-1], w["w_out"], w["b_out"], w["labels"])
    G, _ = ogru.backward_chain(h, w["x"], *args, seed)
    h32, G32 = h.astype(np.float32), G.astype(np.float32)
    ref = ogru.param_grads(h32, w["x"], G32, *args)
    got = bp.param_grads(bp.GRU, to_gpu(h32), d["x"], to_gpu(G32), d["w_ih"], d["w_hh"], d["b_ih"], d["b_hh"])
    for g, r, name in zip(got, ref, ("dW_ih", "dW_hh", "db_ih", "db_hh")):
        assert rel_err(to_np(g), r) <= TOL, name


def _end_to_end(bp, w):
    import torch
    d = _dev(w)
    h = _gpu_forward(bp, w, d)
    seed, _ = bp.head_seed(h[-1].contiguous(), d["w_out"], d["b_out"], d["labels"])
    Jt = bp.build_jacobians(bp.GRU, h, d["x"], d["w_ih"], d["w_hh"], d["b_ih"], d["b_hh"])
    g0 = torch.empty((w["B"], w["H"]), dtype=torch.float32, device="cuda")
    G = bp.scan(Jt, seed, g0=g0)
    grads = bp.param_grads(bp.GRU, h, d["x"], G, d["w_ih"], d["w_hh"], d["b_ih"], d["b_hh"])
    torch.cuda.synchronize()
    return Jt, to_np(h), to_np(G), to_np(g0), [to_np(g) for g in grads]


def _oracle(w):
    args = (w["w_ih"], w["w_hh"], w["b_ih"], w["b_hh"])
    h = ogru.forward(w["x"], *args)
    _, seed = orn.head(h[-1], w["w_out"], w["b_out"], w["labels"])
    G, g0 = ogru.backward_chain(h, w["x"], *args, seed)
    return h, G, g0, ogru.param_grads(h, w["x"], G, *args)


@pytest.mark.parametrize("T,B,H,I", [(40, 2, 20, 2), (150, 3, 32, 1), (70, 2, 128, 1)])
def test_gru_end_to_end_small(bp, T, B, H, I):
    w = workloads.gru_inputs(T, B, H, I, 11, seed=T)
    _, h, G, g0, grads = _end_to_end(bp, w)
    h_ref, G_ref, g0_ref, grads_ref = _oracle(w)
    assert rel_err(G, G_ref) <= TOL
    assert per_step_err(G, G_ref) <= 2 * TOL
    for g, r in zip(grads, grads_ref):
        assert rel_err(g, r) <= TOL


def test_gru_config3_full_size(bp):
    """configs[3]: H=128, T=4096, B=16 (4 GiB of Jacobians), in the launch shape bench uses."""
    w = workloads.config_inputs(3)
    Jt, h, G, g0, grads = _end_to_end(bp, w)
    h_ref, G_ref, g0_ref, grads_ref = _oracle(w)
    assert rel_err(h, h_ref) <= 1e-4
    assert rel_err(G, G_ref) <= TOL
    assert per_step_err(G, G_ref) <= 2 * TOL
    for g, r in zip(grads, grads_ref):
        assert rel_err(g, r) <= TOL
    # sampled Jacobians, one (t, b) matrix at a time from the oracle's closed form
    rng = np.random.default_rng(0)
    args = (w["w_ih"], w["w_hh"], w["b_ih"], w["b_hh"])
    for t in [0, 1, 4095] + list(rng.integers(2, 4095, size=5)):
        ref = ogru.step_jacobian_T(h[t], w["x"][t], *args)
        assert rel_err(to_np(Jt[int(t)]), ref) <= 2e-6


def _oracle_scan_in_chunks(Jt, seed, chunk=64):
    """oracle.scan.linear_scan over a device-resident chain, `chunk` steps at a time from the seed
    end (each chunk's last vector seeds the next), so that the fp64 copy of the Jacobians stays small."""
    T = Jt.shape[0]
    G = np.zeros((T,) + tuple(seed.shape))
    g = np.asarray(seed, dtype=np.float64)
    G[T - 1] = g
    for t1 in range(T, 0, -chunk):
        t0 = max(t1 - chunk, 0)
        Gc, g_next = oscan.linear_scan(to_np(Jt[t0:t1]), g)
        # Gc[k-1] = g[t0+k] for k = 1 .. t1-t0, so Gc[:-1] are g[t0+1 .. t1-1]
        G[t0:t1 - 1] = Gc[:t1 - t0 - 1]
        g = g_next
        if t0 >= 1:
            G[t0 - 1] = g
    return G, g


@pytest.mark.parametrize("T,B", [(2304, 16), (700, 64), (11000, 3), (260, 256), (200, 128), (450, 1)])
def test_h128_long_scan_matches_oracle_and_replays_in_a_hip_graph(bp, T, B):
    """The H=128 scan as its cost model schedules it, on chains of several shapes (up to 4 GB of
    Jacobians): a serial chain beside two slabs of 15 segments (B=16), beside one slab of 3 (B=64),
    beside two slabs of 84 (B=3); the two-level form without a serial chain where the batch alone
    fills the device (B=256); the largest batch that still gets a compute unit per sample (B=128,
    T=200: the model walks the whole chain serially) and a single sample (a short chain, then one
    slab cut into 16-step segments).  Every element of G and g0 is
    compared with the oracle's serial scan of the same chain; repeated calls and replays of a
    captured graph return the same bits whatever the workspace held."""
    import torch
    H = 128
    gen = torch.Generator(device="cuda")
    gen.manual_seed(1234)
    Jt = torch.empty((T, B, H, H), dtype=torch.float32, device="cuda")
    for t0 in range(0, T, 64):                   # near-isometries: identity plus a small random part
        blk = Jt[t0:t0 + 64]
        blk.normal_(0.0, 0.03 / np.sqrt(H), generator=gen)
        blk.diagonal(dim1=-2, dim2=-1).add_(1.0)
    seed = torch.randn((B, H), dtype=torch.float32, device="cuda", generator=gen)
    ws = torch.empty(bp.scan_workspace_bytes(T, B, H), dtype=torch.uint8, device="cuda")
    G = torch.empty((T, B, H), dtype=torch.float32, device="cuda")
    g0 = torch.empty((B, H), dtype=torch.float32, device="cuda")
    bp.scan(Jt, seed, G=G, g0=g0, workspace=ws)
    torch.cuda.synchronize()
    ref, ref0 = G.clone(), g0.clone()
    assert torch.equal(G[T - 1], seed)
    G_ref, g0_ref = _oracle_scan_in_chunks(Jt, to_np(seed))
    assert rel_err(to_np(G), G_ref) <= TOL
    assert per_step_err(to_np(G), G_ref) <= 2 * TOL
    assert rel_err(to_np(g0), g0_ref) <= TOL

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        bp.scan(Jt, seed, G=G, g0=g0, workspace=ws)
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        bp.scan(Jt, seed, G=G, g0=g0, workspace=ws)
    for _ in range(3):
        G.zero_()
        g0.zero_()
        ws.fill_(0x5A)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(G, ref) and torch.equal(g0, ref0)
        bp.scan(Jt, seed, G=G, g0=g0, workspace=ws)      # eager work between the replays
        torch.cuda.synchronize()
        assert torch.equal(G, ref) and torch.equal(g0, ref0)


def _near_isometries(T, B, seed_value):
    import torch
    H = 128
    gen = torch.Generator(device="cuda")
    gen.manual_seed(seed_value)
    Jt = torch.empty((T, B, H, H), dtype=torch.float32, device="cuda")
    for t0 in range(0, T, 64):                   # identity plus a small random part
        blk = Jt[t0:t0 + 64]
        blk.normal_(0.0, 0.03 / np.sqrt(H), generator=gen)
        blk.diagonal(dim1=-2, dim2=-1).add_(1.0)
    seed = torch.randn((B, H), dtype=torch.float32, device="cuda", generator=gen)
    return Jt, seed


@pytest.mark.parametrize("T,B,want_g0", [(700, 4, True), (641, 3, False), (130, 5, True)])
def test_h128_forced_schedules_match_oracle(bp, T, B, want_g0):
    """Every form of the H=128 schedule on one chain, forced through bppsa_scan_h128_diag: no serial
    chain (totals of all interior segments, scanned recursively), serial chains of 1, 2, 3 and 5
    segments with slabs of 1, 2, 3 or all remaining segments, the slab farthest from the seed cut
    into segments of 64, 32 and 16 steps, and the whole chain walked serially.  T = 641 without g0
    is ten full segments (no short segment at the seed end); T = 130 has three segments, so that
    slabs end on segments 1 and 0 in every way.  Every element is compared with the oracle's
    serial scan."""
    import torch
    H = 128
    Jt, seed = _near_isometries(T, B, 77 + T)
    G_ref, g0_ref = _oracle_scan_in_chunks(Jt, to_np(seed))
    ws = torch.empty(bp.scan_workspace_bytes(T, B, H), dtype=torch.uint8, device="cuda")
    nseg = -(-(T - (0 if want_g0 else 1)) // 64)
    forms = [(0, 0, 0), (1, 0, 0), (1, 1, 64), (1, 2, 32), (2, 3, 16), (3, 2, 64), (2, 0, 32), (5, 1, 16),
             (nseg - 1, 0, 0), (nseg - 1, 0, 16), (nseg, 0, 0), (nseg + 3, 0, 0)]
    for chain, slab, last in forms:
        G = torch.zeros((T, B, H), dtype=torch.float32, device="cuda")
        g0 = torch.zeros((B, H), dtype=torch.float32, device="cuda") if want_g0 else None
        ws.fill_(0xA5)
        bp.scan_h128_diag(Jt, seed, G=G, g0=g0, workspace=ws, chain_segments=chain, slab_segments=slab,
                          last_slab_steps=last)
        torch.cuda.synchronize()
        what = "chain_segments=%d slab_segments=%d last_slab_steps=%d" % (chain, slab, last)
        assert torch.equal(G[T - 1], seed), what
        assert rel_err(to_np(G), G_ref) <= TOL, what
        assert per_step_err(to_np(G), G_ref) <= 2 * TOL, what
        if want_g0:
            assert rel_err(to_np(g0), g0_ref) <= TOL, what


def test_h128_many_slabs(bp):
    """A chain cut into the largest number of slabs the launcher handles (a forced slab of one
    segment is raised to two: 31 slabs, one event each), against the oracle's serial scan."""
    import torch
    T, B, H = 4000, 8, 128
    Jt, seed = _near_isometries(T, B, 4242)
    G = bp.scan_h128_diag(Jt, seed, chain_segments=2, slab_segments=1, last_slab_steps=64)
    torch.cuda.synchronize()
    G_ref, _ = _oracle_scan_in_chunks(Jt, to_np(seed))
    assert rel_err(to_np(G), G_ref) <= TOL
    assert per_step_err(to_np(G), G_ref) <= 2 * TOL


def test_h128_diag_rejects_what_it_cannot_run(bp):
    """Argument checks of bppsa_scan_h128_diag happen on the host, before any launch."""
    import torch
    from paper_1907_10134_amd.binding import BppsaError
    T, B, H = 3000, 2, 128
    Jt = torch.empty((T, B, H, H), dtype=torch.float32, device="cuda")    # never read
    seed = torch.zeros((B, H), dtype=torch.float32, device="cuda")
    G = torch.empty((T, B, H), dtype=torch.float32, device="cuda")
    ws = torch.empty(bp.scan_workspace_bytes(T, B, H), dtype=torch.uint8, device="cuda")
    with pytest.raises(BppsaError):          # not a segment length
        bp.scan_h128_diag(Jt, seed, G=G, workspace=ws, chain_segments=1, last_slab_steps=48)
    with pytest.raises(BppsaError):          # 46 segments in one slab, cut in two: more than 32 fine segments
        bp.scan_h128_diag(Jt, seed, G=G, workspace=ws, chain_segments=1, slab_segments=127, last_slab_steps=32)
    with pytest.raises(BppsaError):
        bp.scan_h128_diag(Jt, seed, G=G, workspace=ws, chain_segments=-1)
    with pytest.raises(BppsaError):          # workspace too small
        bp.scan_h128_diag(Jt, seed, G=G, workspace=ws[:4096], chain_segments=1)
    Bbig = 200                                # no compute unit per sample beside the matrix-core work
    Jb = torch.empty((70, Bbig, H, H), dtype=torch.float32, device="cuda")
    with pytest.raises(BppsaError):
        bp.scan_h128_diag(Jb, torch.zeros((Bbig, H), device="cuda"), chain_segments=1)


def test_h128_long_scan_from_two_host_threads(bp):
    """Two host threads call bppsa_scan at H=128 at the same time, each on its own stream, seed,
    outputs and workspace (the Jacobians are shared, read-only).  Both use the library's second
    stream of the device; each must return the oracle's result for its own seed."""
    import threading
    import torch
    T, B, H = 700, 64, 128
    gen = torch.Generator(device="cuda")
    gen.manual_seed(99)
    Jt = torch.empty((T, B, H, H), dtype=torch.float32, device="cuda")
    for t0 in range(0, T, 64):
        blk = Jt[t0:t0 + 64]
        blk.normal_(0.0, 0.03 / np.sqrt(H), generator=gen)
        blk.diagonal(dim1=-2, dim2=-1).add_(1.0)
    seeds = [torch.randn((B, H), dtype=torch.float32, device="cuda", generator=gen) for _ in range(2)]
    outs = [(torch.zeros((T, B, H), dtype=torch.float32, device="cuda"),
             torch.zeros((B, H), dtype=torch.float32, device="cuda"),
             torch.empty(bp.scan_workspace_bytes(T, B, H), dtype=torch.uint8, device="cuda")) for _ in range(2)]
    streams = [torch.cuda.Stream() for _ in range(2)]
    torch.cuda.synchronize()
    errors = []
    gate = threading.Barrier(2)

    def work(i):
        try:
            gate.wait()
            for _ in range(3):
                bp.scan(Jt, seeds[i], G=outs[i][0], g0=outs[i][1], workspace=outs[i][2], stream=streams[i])
            streams[i].synchronize()
        except Exception as exc:                      # surfaced in the main thread below
            errors.append(exc)

    threads = [threading.Thread(target=work, args=(i,)) for i in range(2)]
    for th in threads:
        th.start()
    for th in threads:
        th.join()
    torch.cuda.synchronize()
    assert not errors, errors
    for i in range(2):
        G_ref, g0_ref = _oracle_scan_in_chunks(Jt, to_np(seeds[i]))
        assert rel_err(to_np(outs[i][0]), G_ref) <= TOL
        assert rel_err(to_np(outs[i][1]), g0_ref) <= TOL


def _fused_vs_oracle(bp, w, want_g0=True):
    import torch
    d = _dev(w)
    h = _gpu_forward(bp, w, d)
    seed, _ = bp.head_seed(h[-1].contiguous(), d["w_out"], d["b_out"], d["labels"])
    g0 = torch.empty((w["B"], w["H"]), dtype=torch.float32, device="cuda") if want_g0 else None
    G = bp.gru_scan_fused(h, d["x"], d["w_ih"], d["w_hh"], d["b_ih"], d["b_hh"], seed, g0=g0)
    torch.cuda.synchronize()
    return h, seed, to_np(G), None if g0 is None else to_np(g0)


@pytest.mark.parametrize("T,B,I", [(7, 5, 1), (64, 2, 3), (65, 3, 1), (70, 2, 1), (300, 3, 2), (1000, 2, 1), (129, 33, 1),
                                   (200, 130, 1)])
def test_gru_scan_fused_matches_oracle_chain(bp, T, B, I):
    """bppsa_gru_scan_fused (Jacobians generated inside the scan's kernels) against the oracle's
    matrix-free chain, every element; sizes cover one segment, a ragged last segment, the chain of
    totals and the two-stream form."""
    w = workloads.gru_inputs(T, B, 128, I, 11, seed=5 * T + B)
    h, seed, G, g0 = _fused_vs_oracle(bp, w)
    h_ref, G_ref, g0_ref, _ = _oracle(w)
    assert rel_err(G, G_ref) <= TOL
    assert per_step_err(G, G_ref) <= 2 * TOL
    if np.max(np.abs(g0_ref)) > 1e-30:            # below that the gradient has left fp32's range
        assert rel_err(g0, g0_ref) <= 5 * TOL
    else:
        assert np.max(np.abs(g0)) <= 1e-30
    # and equal, up to rounding, to the two calls on the same hidden states
    d = _dev(w)
    Jt = bp.build_jacobians(bp.GRU, h, d["x"], d["w_ih"], d["w_hh"], d["b_ih"], d["b_hh"])
    G2 = to_np(bp.scan(Jt, seed))
    assert rel_err(G, G2) <= 1e-5


def test_gru_scan_fused_config3_full_size(bp):
    """configs[3] (H=128, T=4096, B=16) through the fused call, every element against the oracle."""
    w = workloads.config_inputs(3)
    h, seed, G, g0 = _fused_vs_oracle(bp, w)
    h_ref, G_ref, g0_ref, _ = _oracle(w)
    assert rel_err(G, G_ref) <= TOL
    assert per_step_err(G, G_ref) <= 2 * TOL
    if np.max(np.abs(g0_ref)) > 1e-30:
        assert rel_err(g0, g0_ref) <= 5 * TOL


def test_gru_scan_fused_rejects_other_sizes(bp):
    import torch
    w = workloads.gru_inputs(10, 2, 64, 1, 11, seed=1)
    d = _dev(w)
    h = _gpu_forward(bp, w, d)
    seed = torch.zeros((2, 64), dtype=torch.float32, device="cuda")
    assert bp.gru_scan_fused_workspace_bytes(10, 2, 64) == 0
    with pytest.raises(bp.BppsaError) as e:
        bp.gru_scan_fused(h, d["x"], d["w_ih"], d["w_hh"], d["b_ih"], d["b_hh"], seed,
                          workspace=torch.empty((1 << 20,), dtype=torch.uint8, device="cuda"))
    assert e.value.code == 6
