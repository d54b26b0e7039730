#!/usr/bin/env python3
"""Benchmark of the BPPSA hot path on one MI355X.

One "step" = bppsa_build_jacobians + bppsa_scan + bppsa_param_grads on the
vanilla tanh RNN workload H=20, I=1, T=1000, B=16 (the paper's headline point,
Section 5.1), with hidden states, inputs and weights already resident in HBM.
Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0   # MI355X published HBM3E bandwidth


# HBM traffic of one scan_h20_kernel launch, from two `rocprofv3 --pmc` runs (FETCH_SIZE, then
# WRITE_SIZE, KiB per dispatch), each scaled by what the same counter reads for the 768,000,000-byte
# calibration copy (FETCH_SIZE reads 375,011.5 KiB for 750,000 KiB fetched: scale 2.000; WRITE_SIZE
# reads 750,006.6 for 750,000 written: scale 1.000).  Offline figures: the counters cannot be read
# inside this process.  Keyed by (T, B, H); the summaries are the profiles/*.txt of the same workloads.
PMC_COPY_SCALE = {"FETCH_SIZE": 750000.0 / 375011.5703, "WRITE_SIZE": 750000.0 / 750006.6250}
PMC_SCAN_KIB = {
    (1000, 16, 20): {"FETCH_SIZE": 13651.1809, "WRITE_SIZE": 2362.0000},
    (30000, 16, 20): {"FETCH_SIZE": 397468.7030, "WRITE_SIZE": 57931.9031},
}


def measured_traffic_bytes(T, B, H):
    kib = PMC_SCAN_KIB.get((T, B, H))
    if kib is None:
        return None
    return int(round(1024 * sum(kib[c] * PMC_COPY_SCALE[c] for c in kib)))


def scan_algorithmic_bytes(T, B, H):
    """Each Jacobian read once, each gradient written once, the seed read once."""
    return T * B * (4 * H * H + 4 * H) + 4 * B * H


def scan_h20_work(T, B, want_g0, hops, resident=768):
    """Products the H=20 scan executes for these sizes: matrix-matrix (2 H^3 FLOP each) and
    matrix-vector (2 H^2 FLOP each).  A unit is one or two halves of 32 steps; every half costs the
    31 products of Algorithm 1's up-sweep on 32 elements, a two-half unit one more for its total;
    the down-sweep is one matrix-vector product per element plus the few of the levels above a
    wave's eight elements that the waves repeat, the unit's outgoing vector and, for two halves,
    the vector between them; `hops` (measured) is the number of totals all look-backs applied."""
    n = T if want_g0 else T - 1
    halves = 2 if -(-n // 32) * B > resident else 1
    nunit = -(-n // (32 * halves))
    mm = nunit * B * (31 * halves + (1 if halves == 2 else 0))
    per_half_mv = 28 + 4          # seven per wave and sub-tree, plus the entering vectors of the four sub-trees
    mv = nunit * B * (per_half_mv * halves + 1 + (1 if halves == 2 else 0)) + int(hops)
    return {"unit_steps": 32 * halves, "units": nunit * B, "matrix_matrix": mm, "matrix_vector": mv,
            "flop": mm * 2 * 20 ** 3 + mv * 2 * 20 ** 2}


def lookback_hops(bp, b):
    """Hops (unit totals applied) of all look-backs of one scan of this workload, measured."""
    import torch
    stats = torch.zeros(3, dtype=torch.int64, device="cuda")
    bp.scan_h20_diag(b["Jt"], b["seed"], G=b["G"], workspace=b["scan_ws"], lookback_stats=stats)
    torch.cuda.synchronize()
    assert int(b["scan_ws"][:4].view(torch.int32).item()) == 0, "a bounded wait inside the scan expired"
    hops, count, most = (int(v) for v in stats.cpu())
    return {"total": hops, "lookbacks": count, "mean": round(hops / max(count, 1), 2), "max": most}


def prepare(bp, w):
    """Upload a workload and run the (untimed) forward pass and head on the GPU."""
    import torch
    dev = "cuda"
    t = {k: torch.from_numpy(v).to(dev) for k, v in w.items() if hasattr(v, "dtype")}
    T, B, H = w["T"], w["B"], w["H"]
    h = torch.zeros((T + 1, B, H), dtype=torch.float32, device=dev)
    bp.forward(bp.RNN_TANH, t["x"], t["w_ih"], t["w_hh"], t["b"], None, h)
    seed, _ = bp.head_seed(h[-1].contiguous(), t["w_out"], t["b_out"], t["labels"])
    bufs = dict(
        h=h, x=t["x"], w_hh=t["w_hh"], seed=seed,
        Jt=torch.empty((T, B, H, H), dtype=torch.float32, device=dev),
        G=torch.empty((T, B, H), dtype=torch.float32, device=dev),
        g0=torch.empty((B, H), dtype=torch.float32, device=dev),
        scan_ws=torch.empty(max(bp.scan_workspace_bytes(T, B, H), 256), dtype=torch.uint8, device=dev),
        pg_ws=torch.empty(max(bp.param_grads_workspace_bytes(bp.RNN_TANH, T, B, H, w["I"]), 256),
                          dtype=torch.uint8, device=dev),
        out=(torch.empty((H, w["I"]), dtype=torch.float32, device=dev),
             torch.empty((H, H), dtype=torch.float32, device=dev),
             torch.empty((H,), dtype=torch.float32, device=dev),
             torch.empty((H,), dtype=torch.float32, device=dev)),
    )
    torch.cuda.synchronize()
    return bufs


def time_steps(bp, b, steps, warmup):
    """Whole-path wall time over exactly `steps` steps plus per-call HIP-event times."""
    import torch

    def step(ev=None):
        if ev:
            ev[0].record()
        bp.build_jacobians(bp.RNN_TANH, b["h"], w_hh=b["w_hh"], Jt=b["Jt"])
        if ev:
            ev[1].record()
        bp.scan(b["Jt"], b["seed"], G=b["G"], g0=None, workspace=b["scan_ws"])
        if ev:
            ev[2].record()
        bp.param_grads(bp.RNN_TANH, b["h"], b["x"], b["G"], out=b["out"], workspace=b["pg_ws"])
        if ev:
            ev[3].record()

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / steps

    # per-call durations on the launch stream (HIP events), same number of steps
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(steps)]
    for e in evs:
        step(e)
    torch.cuda.synchronize()
    parts = {name: statistics.mean(e[i].elapsed_time(e[i + 1]) for e in evs)
             for i, name in enumerate(("build_jacobians_ms", "scan_ms", "param_grads_ms"))}
    return wall_ms, parts


def time_fused(bp, b, steps, warmup):
    """The tanh-RNN path without materialised Jacobians: bppsa_rnn_scan_fused + bppsa_param_grads."""
    import torch

    def step():
        bp.rnn_scan_fused(b["h"], b["w_hh"], b["seed"], G=b["G"], g0=None, workspace=b["scan_ws"])
        bp.param_grads(bp.RNN_TANH, b["h"], b["x"], b["G"], out=b["out"], workspace=b["pg_ws"])

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / steps
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    for a, z in evs:
        a.record()
        bp.rnn_scan_fused(b["h"], b["w_hh"], b["seed"], G=b["G"], g0=None, workspace=b["scan_ws"])
        z.record()
    torch.cuda.synchronize()
    return wall_ms, statistics.mean(a.elapsed_time(z) for a, z in evs)


def time_steps_cold(bp, b, steps):
    """Per-step HIP-event time when a 1 GiB buffer is overwritten before every step, so that
    neither the 256 MB memory-side cache nor the L2s hold any of the step's inputs."""
    import torch
    evict = torch.empty(1 << 28, dtype=torch.float32, device="cuda")
    times = []
    for i in range(steps):
        evict.fill_(float(i))
        a, z = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        bp.build_jacobians(bp.RNN_TANH, b["h"], w_hh=b["w_hh"], Jt=b["Jt"])
        bp.scan(b["Jt"], b["seed"], G=b["G"], g0=None, workspace=b["scan_ws"])
        bp.param_grads(bp.RNN_TANH, b["h"], b["x"], b["G"], out=b["out"], workspace=b["pg_ws"])
        z.record()
        torch.cuda.synchronize()
        times.append(a.elapsed_time(z))
    del evict
    return statistics.median(times)


def time_scan_only(bp, b, steps, warmup):
    """Mean HIP-event duration of bppsa_scan over `steps` back-to-back calls after `warmup` untimed
    ones.  On a fresh device the first hundred or so launches of a 0.3 ms kernel run up to 20 %
    slower than the steady state (clock ramp), so the long scan warms up accordingly."""
    import torch
    for _ in range(warmup):
        bp.scan(b["Jt"], b["seed"], G=b["G"], g0=None, workspace=b["scan_ws"])
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    for a, z in evs:
        a.record()
        bp.scan(b["Jt"], b["seed"], G=b["G"], g0=None, workspace=b["scan_ws"])
        z.record()
    torch.cuda.synchronize()
    return statistics.mean(a.elapsed_time(z) for a, z in evs)


def long_scan(bp, workloads, steps, fused=True):
    """bppsa_scan alone on configs[2] (T=30000): the HBM-bound case of the scan."""
    w2 = workloads.config_inputs(2)
    b2 = prepare(bp, w2)
    bp.build_jacobians(bp.RNN_TANH, b2["h"], w_hh=b2["w_hh"], Jt=b2["Jt"])
    ms = time_scan_only(bp, b2, steps=max(5, min(50, steps)), warmup=150)
    fused_ms = time_fused(bp, b2, max(5, min(50, steps)), 50)[1] if fused else None
    nbytes = scan_algorithmic_bytes(w2["T"], w2["B"], w2["H"])
    gbps = nbytes / (ms * 1e-3) / 1e9
    hops = lookback_hops(bp, b2)
    work = scan_h20_work(w2["T"], w2["B"], False, hops["total"])
    return {"workload": "rnn_tanh_H20_I1_T30000_B16 (configs[2])", "scan_ms": round(ms, 5),
            "algorithmic_bytes": nbytes, "gbps": round(gbps, 2),
            "frac_of_hbm_peak": round(gbps / HBM_PEAK_GBPS, 5),
            "traffic": measured_traffic_bytes(w2["T"], w2["B"], w2["H"]),
            "products": work, "gflops": round(work["flop"] / (ms * 1e-3) / 1e9, 1),
            "lookback_hops": hops,
            "fused_scan_ms": None if fused_ms is None else round(fused_ms, 5)}


def copy_calibration(bp, steps):
    """A plain copy of exactly the bytes of configs[2]'s Jacobian array (768,000,000 B each way)."""
    import torch
    n = 30000 * 16 * 20 * 20
    src = torch.ones(n, dtype=torch.float32, device="cuda")
    dst = torch.empty_like(src)
    for _ in range(3):
        bp.calibration_copy(src, dst)
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    for a, z in evs:
        a.record()
        bp.calibration_copy(src, dst)
        z.record()
    torch.cuda.synchronize()
    ms = statistics.mean(a.elapsed_time(z) for a, z in evs)
    return {"workload": "calibration copy", "bytes_read": 4 * n, "bytes_written": 4 * n,
            "copy_ms": round(ms, 5), "gbps_read_plus_write": round(8 * n / (ms * 1e-3) / 1e9, 2)}


def gru_workload(bp, workloads, steps):
    """configs[3] (GRU H=128, T=4096, B=16): per-call times of the three hot-path calls.

    The scan's schedule (how many steps nearest the seed one serial matrix-vector chain per sample
    walks, how many segments get matrix-matrix totals) is the library's own choice, read back with
    bppsa_scan_h128_schedule; a total costs S - 1 products of 2 H^3 FLOP per sample."""
    import torch
    w = workloads.config_inputs(3)
    T, B, H, I = w["T"], w["B"], w["H"], w["I"]
    d = {k: torch.from_numpy(w[k]).cuda() for k in ("x", "w_ih", "w_hh", "b_ih", "b_hh", "w_out", "b_out", "labels")}
    h = torch.zeros((T + 1, B, H), dtype=torch.float32, device="cuda")
    bp.forward(bp.GRU, d["x"], d["w_ih"], d["w_hh"], d["b_ih"], d["b_hh"], h)
    torch.cuda.synchronize()
    fw = (torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
    fw[0].record()
    bp.forward(bp.GRU, d["x"], d["w_ih"], d["w_hh"], d["b_ih"], d["b_hh"], h)   # not part of the backward pass
    fw[1].record()
    torch.cuda.synchronize()
    forward_ms = fw[0].elapsed_time(fw[1])
    seed, _ = bp.head_seed(h[-1].contiguous(), d["w_out"], d["b_out"], d["labels"])
    Jt = torch.empty((T, B, H, H), dtype=torch.float32, device="cuda")
    G = torch.empty((T, B, H), dtype=torch.float32, device="cuda")
    ws = torch.empty(bp.scan_workspace_bytes(T, B, H), dtype=torch.uint8, device="cuda")
    pws = torch.empty(max(bp.param_grads_workspace_bytes(bp.GRU, T, B, H, I), 256), dtype=torch.uint8, device="cuda")
    out = (torch.empty((3 * H, I), device="cuda"), torch.empty((3 * H, H), device="cuda"),
           torch.empty((3 * H,), device="cuda"), torch.empty((3 * H,), device="cuda"))

    def step(ev=None):
        if ev:
            ev[0].record()
        bp.build_jacobians(bp.GRU, h, d["x"], d["w_ih"], d["w_hh"], d["b_ih"], d["b_hh"], Jt=Jt)
        if ev:
            ev[1].record()
        bp.scan(Jt, seed, G=G, g0=None, workspace=ws)
        if ev:
            ev[2].record()
        bp.param_grads(bp.GRU, h, d["x"], G, d["w_ih"], d["w_hh"], d["b_ih"], d["b_hh"], out=out, workspace=pws)
        if ev:
            ev[3].record()

    steps = max(3, min(10, steps))
    step()
    torch.cuda.synchronize()
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(steps)]
    for e in evs:
        step(e)
    torch.cuda.synchronize()
    parts = {name: statistics.mean(e[i].elapsed_time(e[i + 1]) for e in evs)
             for i, name in enumerate(("build_jacobians_ms", "scan_ms", "param_grads_ms"))}
    # the same scan without the serial chain (totals of all interior segments, scanned recursively)
    two_level = lambda: bp.scan_h128_diag(Jt, seed, G=G, workspace=ws, chain_segments=0)
    two_level()
    torch.cuda.synchronize()
    tev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    for a, z in tev:
        a.record()
        two_level()
        z.record()
    torch.cuda.synchronize()
    two_level_ms = statistics.mean(a.elapsed_time(z) for a, z in tev)
    sched = bp.scan_h128_schedule(T, B, want_g0=False, generated=False)
    fsched = bp.scan_h128_schedule(T, B, want_g0=False, generated=True)
    mm = sched["matrix_products"]
    flop = mm * 2 * H ** 3 + T * B * 2 * H * H
    tf = flop / (parts["scan_ms"] * 1e-3) / 1e12
    # the same backward pass with the Jacobians generated inside the scan (no Jt array)
    del Jt
    torch.cuda.empty_cache()
    fws = torch.empty(bp.gru_scan_fused_workspace_bytes(T, B, H), dtype=torch.uint8, device="cuda")
    fused = lambda: bp.gru_scan_fused(h, d["x"], d["w_ih"], d["w_hh"], d["b_ih"], d["b_hh"], seed, G=G, workspace=fws)
    fused()
    torch.cuda.synchronize()
    fev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    for a, z in fev:
        a.record()
        fused()
        z.record()
    torch.cuda.synchronize()
    fused_ms = statistics.mean(a.elapsed_time(z) for a, z in fev)
    return {"workload": "gru_H128_I1_T4096_B16 (configs[3])", **{k: round(v, 4) for k, v in parts.items()},
            "fused_scan_ms": round(fused_ms, 4), "two_level_scan_ms": round(two_level_ms, 4),
            "forward_ms": round(forward_ms, 4),
            "fused_vs_build_plus_scan": round((parts["build_jacobians_ms"] + parts["scan_ms"]) / fused_ms, 3),
            "schedule": {k: sched[k] for k in ("segment_steps", "chain_steps", "slab_segments", "slabs", "last_slab_steps")},
            "fused_schedule": {k: fsched[k] for k in ("segment_steps", "chain_steps", "slab_segments", "slabs", "last_slab_steps",
                                                      "matrix_products")},
            "scan_matrix_products": mm, "scan_flop": flop, "scan_tflops": round(tf, 2),
            "frac_of_fp32_mfma_peak": round(tf / 157.3, 4),
            "two_level_frac_of_fp32_mfma_peak": round(
                ((T - 1 + 63) // 64 - 2) * 63 * B * 2 * H ** 3 / (two_level_ms * 1e-3) / 1e12 / 157.3, 4),
            "note": "scan_tflops counts the products the schedule executes; the serial chain removes products, "
                    "so compare scan_ms with two_level_scan_ms, not the rates",
            "scan_bytes_min": T * B * (4 * H * H + 4 * H), "jacobian_bytes": 4 * T * B * H * H}


def cnn_workload(bp, workloads, steps):
    """configs[4] (pruned VGG-11-style CNN, one 32x32x3 image): CSR builders, plan, sparse scan.

    Timing only: the layer inputs that decide the ReLU masks and pooling winners are seeded N(0,1)
    arrays of the right shapes (the parity tests use the real forward activations); the
    structure of the convolution and fully connected Jacobians does not depend on them."""
    import numpy as np
    import torch
    layers, _, _ = workloads.cnn_layers()
    rng = np.random.default_rng(1234 + 4)
    dev = "cuda"
    prepared = []
    for L in reversed(layers):                       # scan order: last layer first
        if L.kind == "conv":
            prepared.append((L, torch.from_numpy(L.weight).to(dev), torch.from_numpy(L.mask.astype(np.uint8)).to(dev)))
        elif L.kind == "fc":
            prepared.append((L, torch.from_numpy(L.weight).to(dev), torch.from_numpy(L.mask.astype(np.uint8)).to(dev)))
        else:
            a = rng.standard_normal(L.in_shape).astype(np.float32)
            prepared.append((L, torch.from_numpy(a).to(dev), None))

    def build():
        out = []
        for L, a, m in prepared:
            if L.kind == "conv":
                out.append(bp.csr_conv3x3(a, m, L.in_shape[1], L.in_shape[2]))
            elif L.kind == "fc":
                out.append(bp.csr_linear(a, m))
            elif L.kind == "relu":
                out.append(bp.csr_relu(a.reshape(-1)))
            else:
                out.append(bp.csr_maxpool2x2(a))
        return out

    build()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    jts = build()
    torch.cuda.synchronize()
    build_ms = (time.perf_counter() - t0) * 1e3      # includes the host reads of nnz (two-call pattern)
    nnz = sum(m.nnz for m in jts)
    rows = sum(m.rows for m in jts)
    seed = torch.from_numpy(rng.standard_normal(jts[0].cols).astype(np.float32)).to(dev)
    grads = [torch.empty((m.rows,), dtype=torch.float32, device=dev) for m in jts]
    arena = torch.empty((1 << 30,), dtype=torch.uint8, device=dev)
    res = {"workload": "pruned_vgg11_cnn_32x32x3 (configs[4])", "jacobians": len(jts), "nnz": nnz,
           "csr_bytes": 8 * nnz + 4 * (rows + len(jts)), "build_all_jacobians_ms": round(build_ms, 3)}
    reps = max(5, min(50, steps))
    for U in (0, 2):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        plan = bp.SpscanPlan(jts, U, arena)
        torch.cuda.synchronize()
        plan_ms = (time.perf_counter() - t0) * 1e3
        for _ in range(3):
            plan.run(jts, seed, grads)
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
        for a, z in evs:
            a.record()
            plan.run(jts, seed, grads)
            z.record()
        torch.cuda.synchronize()
        run_ms = statistics.mean(a.elapsed_time(z) for a, z in evs)
        mm, mv = plan.flops()
        res["up_levels_%d" % U] = {"plan_ms": round(plan_ms, 3), "run_ms": round(run_ms, 4),
                                   "products": plan.num_products(), "mm_flop": mm, "mv_flop": mv,
                                   "arena_bytes": plan.arena_used()}
        if U:
            # FLOP per tree level (the series of Section 5.3's static analysis) and the cost of a
            # plan whose symbolic phase comes from the cache
            series = {}
            for st in plan.steps():
                key = "%s%s_%s" % (st["phase"], "" if st["phase"] in ("linear", "tail") else st["level"], st["kind"])
                series[key] = series.get(key, 0) + st["flops"]
            res["up_levels_%d" % U]["flop_by_level"] = series
            cache = bp.SpscanCache()
            bp.SpscanPlan(jts, U, arena, cache=cache).close()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            again = bp.SpscanPlan(jts, U, arena, cache=cache)
            torch.cuda.synchronize()
            res["up_levels_%d" % U]["plan_cached_ms"] = round((time.perf_counter() - t0) * 1e3, 3)
            assert cache.stats()[:2] == (1, 1)
            again.close()
            cache.close()
        plan.close()
    b = res["csr_bytes"] + 4 * (rows + jts[0].cols)
    res["spmv_chain_gbps"] = round(b / (res["up_levels_0"]["run_ms"] * 1e-3) / 1e9, 2)
    return res


def train_workload(bp, workloads, T, B, reps, materialise=False):
    """One training iteration of the Section 4.1 task (bit-stream classification, H = 20, Adam,
    lr = 1e-5) at sequence length T and batch B: forward, head, backward as a scan, parameter
    gradients, update.  Batches are generated on the host beforehand and resident on the GPU."""
    import torch
    H, I, C = 20, 1, 10
    params = {k: torch.from_numpy(v) for k, v in workloads.rnn_parameters().items()}
    tr = bp.RnnTrainer(T, B, H, I, C, params, materialise=materialise)
    batches = []
    for k in range(2):
        x, labels = workloads.bitstream_batch(T, B, first_sample=k * B)
        batches.append((torch.from_numpy(x).cuda(), torch.from_numpy(labels).cuda()))
    for k in range(3):
        tr.step(*batches[k % 2])
    torch.cuda.synchronize()
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
    for k, (a, z) in enumerate(evs):
        a.record()
        tr.step(*batches[k % 2])
        z.record()
    torch.cuda.synchronize()
    total = statistics.median(a.elapsed_time(z) for a, z in evs)
    bp.check_scan(tr.workspace)
    assert math.isfinite(float(tr.loss.item()))

    # the same calls one by one, for the breakdown (forward pass / backward pass / the rest)
    x, labels = batches[0]
    w_ih, w_hh = tr.view(tr.params, "w_ih"), tr.view(tr.params, "w_hh")
    b_ih, b_hh = tr.view(tr.params, "b_ih"), tr.view(tr.params, "b_hh")
    w_out, b_out = tr.view(tr.params, "w_out"), tr.view(tr.params, "b_out")
    g = {k: tr.view(tr.grads, k) for k in bp.RNN_PARAM_ORDER}

    def timed(fn):
        for _ in range(2):
            fn()
        e = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
        for a, z in e:
            a.record()
            fn()
            z.record()
        torch.cuda.synchronize()
        return statistics.median(a.elapsed_time(z) for a, z in e)

    def backward():
        if materialise:
            bp.build_jacobians(bp.RNN_TANH, tr.h, w_hh=w_hh, Jt=tr.Jt)
            bp.scan(tr.Jt, tr.seed, tr.G, workspace=tr.workspace)
        else:
            bp.rnn_scan_fused(tr.h, w_hh, tr.seed, tr.G, workspace=tr.workspace)
        bp.param_grads(bp.RNN_TANH, tr.h, x, tr.G, out=(g["w_ih"], g["w_hh"], g["b_ih"], g["b_hh"]),
                       workspace=tr.workspace)

    fwd = timed(lambda: bp.forward(bp.RNN_TANH, x, w_ih, w_hh, b_ih, b_hh, tr.h))
    head = timed(lambda: bp.head_backward(tr.h[T], w_out, b_out, labels, tr.seed, tr.loss, g["w_out"], g["b_out"]))
    bwd = timed(backward)
    upd = timed(lambda: bp.adam_step(tr.params, tr.grads, tr.adam_m, tr.adam_v, 5))
    return {"T": T, "B": B, "iteration_ms": round(total, 4), "forward_ms": round(fwd, 4), "head_ms": round(head, 4),
            "backward_ms": round(bwd, 4), "update_ms": round(upd, 4),
            "samples_per_s": round(B / (total * 1e-3), 1)}


def train_sweeps(bp, workloads, reps):
    """Sequence-length and batch-size sweeps in the shape of Section 5.1's sensitivity analysis."""
    import torch
    out = {"task": "bitstream classification, 10 classes, Bernoulli(0.05 + 0.1 c), RNN H=20, Adam lr=1e-5",
           "jacobians": "generated inside the scan (bppsa_rnn_scan_fused)", "by_T_at_B16": [], "by_B_at_T1000": []}
    for T in (10, 30, 100, 300, 1000, 3000, 10000, 30000):
        out["by_T_at_B16"].append(train_workload(bp, workloads, T, 16, reps))
        torch.cuda.empty_cache()
    for B in (2, 4, 8, 16, 32, 64, 128, 256):
        out["by_B_at_T1000"].append(train_workload(bp, workloads, 1000, B, reps))
        torch.cuda.empty_cache()
    out["materialised_T1000_B16"] = train_workload(bp, workloads, 1000, 16, reps, materialise=True)
    return out


def cpu_baseline(w, budget_s=15.0):
    """The fp64 oracle's backward (chain + parameter sums) on the same workload, one thread."""
    import numpy as np
    from threadpoolctl import threadpool_limits
    from oracle import rnn as orn
    with threadpool_limits(limits=1):
        h = orn.forward(w["x"], w["w_ih"], w["w_hh"], w["b"])
        _, seed = orn.head(h[-1], w["w_out"], w["b_out"], w["labels"])
        times = []
        t_start = time.perf_counter()
        while len(times) < 20 and (time.perf_counter() - t_start) < budget_s:
            t0 = time.perf_counter()
            G, _ = orn.backward_chain(h, w["w_hh"], seed)
            orn.param_grads(h, w["x"], G)
            times.append((time.perf_counter() - t0) * 1e3)
    return statistics.median(times), len(times)


def host_cpu():
    model = "unknown"
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                model = line.split(":", 1)[1].strip()
                break
    except OSError:
        pass
    return {"nproc": os.cpu_count(), "model": model}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--no-long", action="store_true", help="skip the T=30000 scan figure")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--no-extra", action="store_true", help="skip the compact GRU (configs[3]) and CNN (configs[4]) figures")
    ap.add_argument("--no-fused", action="store_true",
                    help="skip the bppsa_rnn_scan_fused figures (profiling runs: keeps the kernel's launches uniform)")
    ap.add_argument("--long-only", action="store_true",
                    help="time only the T=30000 scan (for profiling); prints its JSON object")
    ap.add_argument("--gru", action="store_true",
                    help="time the three calls on configs[3] (GRU H=128, T=4096); prints its JSON object")
    ap.add_argument("--train", action="store_true",
                    help="whole training iterations of the Section 4.1 task over sequence lengths and batch sizes")
    ap.add_argument("--cnn", action="store_true",
                    help="time the sparse path on configs[4] (pruned CNN); prints its JSON object")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run only the known-size copy kernel (768 MB in, 768 MB out) that "
                         "hardware traffic counters are scaled against; prints its JSON object")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding, no collectives); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import workloads
    import paper_1907_10134_amd as bp

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)

    if args.long_only:
        print(json.dumps(long_scan(bp, workloads, args.steps, fused=not args.no_fused)))
        return
    if args.gru:
        print(json.dumps(gru_workload(bp, workloads, args.steps)))
        return
    if args.train:
        print(json.dumps(train_sweeps(bp, workloads, max(5, min(30, args.steps)))))
        return
    if args.cnn:
        print(json.dumps(cnn_workload(bp, workloads, args.steps)))
        return
    if args.copy_calibration:
        print(json.dumps(copy_calibration(bp, max(5, min(50, args.steps)))))
        return

    w = workloads.config_inputs(1)
    T, B, H = w["T"], w["B"], w["H"]
    bufs = prepare(bp, w)
    wall_ms, parts = time_steps(bp, bufs, args.steps, args.warmup)
    bp.check_scan(bufs["scan_ws"])      # the timed scans ended normally

    cold_ms = time_steps_cold(bp, bufs, max(5, min(30, args.steps)))
    fused_wall_ms, fused_scan_ms = (None, None) if args.no_fused else time_fused(bp, bufs, args.steps, args.warmup)
    scan_bytes = scan_algorithmic_bytes(T, B, H)
    scan_gbps = scan_bytes / (parts["scan_ms"] * 1e-3) / 1e9
    out = {
        "metric": "backward_pass_ms (build_jacobians + scan + param_grads), RNN H=20 B=16 T=1000",
        "value": round(wall_ms, 5),
        "unit": "ms",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(wall_ms, 5),
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": "rnn_tanh_H20_I1_T1000_B16 (configs[1])", "T": T, "B": B, "H": H,
                   "parallelism": "single-gpu"},
        "paper_context": "context, not the target: the paper reports a 16x backward-pass speedup for this workload "
                         "on an RTX 2070 and up to 108x over its sweeps on an RTX 2080 Ti (Section 5.1); "
                         "its Table 4 epoch times imply about 1.7 ms of BPPSA backward work per iteration at T=1000 "
                         "and 7.7 ms at T=30000 (figures that also contain the head's backward and the optimizer step)",
        "breakdown_ms": {k: round(v, 5) for k, v in parts.items()},
        "cold_cache_step_ms": round(cold_ms, 5),
        "fused_path": {"what": "bppsa_rnn_scan_fused + bppsa_param_grads (Jacobians generated inside the scan, "
                               "never stored); not the metric above", "step_ms": None if fused_wall_ms is None else round(fused_wall_ms, 5),
                       "scan_ms": None if fused_scan_ms is None else round(fused_scan_ms, 5)},
        "scan_gbps": round(scan_gbps, 2),
        "roofline": {"kernel": "scan_h20_kernel (all of bppsa_scan: clearing launch + main kernel)", "bound": "hbm", "achieved": round(scan_gbps, 2),
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(scan_gbps / HBM_PEAK_GBPS, 5),
                     "traffic": measured_traffic_bytes(T, B, H), "algorithmic_bytes": scan_bytes},
    }

    # scan work and look-back statistics of the headline workload, and one roofline entry per call
    hops1 = lookback_hops(bp, bufs)
    work1 = scan_h20_work(T, B, False, hops1["total"])
    out["scan_products"] = work1
    out["scan_gflops"] = round(work1["flop"] / (parts["scan_ms"] * 1e-3) / 1e9, 1)
    out["scan_lookback_hops"] = hops1
    I = w["I"]
    call_bytes = {
        "bppsa_build_jacobians": T * B * (4 * H * H + 4 * H) + 4 * H * H,          # tiles written, h and W_hh read
        "bppsa_scan": scan_bytes,
        "bppsa_param_grads": T * B * (2 * 4 * H + 4 * H + 4 * I) + 4 * H * (H + I + 1),   # G, h (twice: as h[t] and h[t-1]), x read
    }
    out["rooflines"] = []
    for call, key in (("bppsa_build_jacobians", "build_jacobians_ms"), ("bppsa_scan", "scan_ms"),
                      ("bppsa_param_grads", "param_grads_ms")):
        g = call_bytes[call] / (parts[key] * 1e-3) / 1e9
        out["rooflines"].append({"call": call, "bound": "hbm", "algorithmic_bytes": call_bytes[call],
                                 "ms": round(parts[key], 5), "achieved": round(g, 1), "peak": HBM_PEAK_GBPS,
                                 "unit": "GB/s", "frac": round(g / HBM_PEAK_GBPS, 5)})

    if not args.no_long:
        del bufs
        torch.cuda.empty_cache()
        out["long_scan"] = long_scan(bp, workloads, args.steps, fused=not args.no_fused)
        # the box's own streaming rate (768 MB read + 768 MB written), for context beside the 8 TB/s peak
        cal = copy_calibration(bp, 10)
        torch.cuda.empty_cache()
        out["measured_copy_gbps"] = cal["gbps_read_plus_write"]
        out["long_scan"]["frac_of_measured_copy"] = round(out["long_scan"]["gbps"] / cal["gbps_read_plus_write"], 5)

    if not args.no_extra:
        # the other two workloads, compact: GRU H=128 (scan bound by the fp32 matrix cores) and the
        # pruned CNN (sparse scan)
        torch.cuda.empty_cache()
        g = gru_workload(bp, workloads, 5)
        # scan_tflops counts the products the schedule executes (scan_matrix_products), which the
        # serial chain makes fewer: compare times, not this rate, across schedules
        out["gru"] = {k: g[k] for k in ("workload", "build_jacobians_ms", "scan_ms", "param_grads_ms",
                                        "fused_scan_ms", "two_level_scan_ms", "schedule", "scan_matrix_products",
                                        "scan_tflops", "frac_of_fp32_mfma_peak", "two_level_frac_of_fp32_mfma_peak",
                                        "note")}
        torch.cuda.empty_cache()
        c = cnn_workload(bp, workloads, 10)
        out["cnn"] = {"workload": c["workload"], "nnz": c["nnz"], "build_all_jacobians_ms": c["build_all_jacobians_ms"],
                      "up_levels_0": c["up_levels_0"], "up_levels_2": c["up_levels_2"],
                      "spmv_chain_gbps": c["spmv_chain_gbps"]}
        torch.cuda.empty_cache()
        # whole training iterations of the Section 4.1 task (forward + head + backward + Adam)
        out["train"] = [train_workload(bp, workloads, 1000, 16, 20), train_workload(bp, workloads, 30000, 16, 5)]
        torch.cuda.empty_cache()

    if not args.no_cpu:
        ms, reps = cpu_baseline(w)
        out["cpu_baseline"] = {"value": round(ms, 4), "unit": "ms", "cores": 1, "kind": "oracle", **host_cpu(),
                               "sample": "full configs[1] workload (T=1000, B=16): fp64 sequential chain + "
                                         "parameter sums, median of %d passes, numpy limited to one thread" % reps}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
