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
    assert per_step_err(G, G_ref) <= 50 * TOL
    for g, r in zip(grads, grads_ref):
        assert rel_err(g, r) <= TOL


def test_gru_config3_full_size(bp):
    """configs[3]: H=128, T=4096, B=16 (4 GiB of Jacobians), in the launch shape bench uses."""
    w = workloads.config_inputs(3)
    Jt, h, G, g0, grads = _end_to_end(bp, w)
    h_ref, G_ref, g0_ref, grads_ref = _oracle(w)
    assert rel_err(h, h_ref) <= 1e-4
    assert rel_err(G, G_ref) <= TOL
    assert per_step_err(G, G_ref) <= 100 * TOL
    for g, r in zip(grads, grads_ref):
        assert rel_err(g, r) <= TOL
    # sampled Jacobians, one (t, b) matrix at a time from the oracle's closed form
    rng = np.random.default_rng(0)
    args = (w["w_ih"], w["w_hh"], w["b_ih"], w["b_hh"])
    for t in [0, 1, 4095] + list(rng.integers(2, 4095, size=5)):
        ref = ogru.step_jacobian_T(h[t], w["x"][t], *args)
        assert rel_err(to_np(Jt[int(t)]), ref) <= 2e-6
