"""Seeded synthetic inputs for the five BPPSA workloads.

This module only draws random numbers and shapes them into input tensors.  It
holds none of the method's arithmetic (no forward pass, no Jacobians, no
gradients), so that the CPU oracle and the HIP path can both consume exactly
the same fp32 values without sharing any code that computes results.

All generators are counter based (numpy Philox keyed by the seed) and return
C-contiguous numpy arrays: float32 for values, int32/int64 for labels.

Workload shapes follow the paper's experiments: the vanilla tanh RNN with 20
hidden units on length-T sequences (Section 4.1), the GRU (Section 4.2) and
the pruned VGG-11-style CNN on one 32x32 image (Section 4.3).
"""
from __future__ import annotations

import math
from dataclasses import dataclass

import numpy as np

BASE_SEED = 1234

# (cell, T, B, H, I, classes) of the four recurrent configurations.
CONFIGS = {
    0: dict(cell="rnn", T=16, B=2, H=20, I=1, C=10),
    1: dict(cell="rnn", T=1000, B=16, H=20, I=1, C=10),
    2: dict(cell="rnn", T=30000, B=16, H=20, I=1, C=10),
    3: dict(cell="gru", T=4096, B=16, H=128, I=1, C=11),
}


def _rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=int(seed)))


def _uniform(rng, shape, bound):
    return rng.uniform(-bound, bound, size=shape).astype(np.float32)


def rnn_inputs(T, B, H=20, I=1, C=10, seed=BASE_SEED):
    """Vanilla tanh RNN workload (Section 4.1 shapes).

    x ~ N(0,1); every weight and bias ~ U(-1/sqrt(H), 1/sqrt(H)); uniform
    random integer labels for the C-way head applied to the last hidden state.
    """
    rng = _rng(seed)
    k = 1.0 / math.sqrt(H)
    return dict(
        cell="rnn", T=T, B=B, H=H, I=I, C=C,
        x=rng.standard_normal((T, B, I)).astype(np.float32),
        w_ih=_uniform(rng, (H, I), k),
        w_hh=_uniform(rng, (H, H), k),
        b=_uniform(rng, (H,), k),
        w_out=_uniform(rng, (C, H), k),
        b_out=_uniform(rng, (C,), k),
        labels=rng.integers(0, C, size=(B,)).astype(np.int32),
    )


def bitstream_batch(T, B, first_sample=0, seed=BASE_SEED + 7, classes=10):
    """A mini-batch of the synthetic bit-stream classification set of Section 4.1.

    Sample k (k = first_sample .. first_sample + B - 1 of the 32000 the paper synthesises) has a
    class c drawn uniformly from 0..classes-1 and a stream x[t] ~ Bernoulli(0.05 + 0.1 c), t = 0..T-1,
    both from a generator keyed on (seed, k), so a sample does not depend on the batch it is in.
    Returns x [T, B, 1] float32 in {0, 1} and labels [B] int32.
    """
    x = np.empty((T, B, 1), np.float32)
    labels = np.empty((B,), np.int32)
    for j in range(B):
        rng = np.random.Generator(np.random.Philox(key=[int(seed), int(first_sample + j)]))
        c = int(rng.integers(0, classes))
        labels[j] = c
        x[:, j, 0] = rng.random(T) < (0.05 + 0.1 * c)
    return x, labels


def rnn_parameters(H=20, I=1, C=10, seed=BASE_SEED + 8):
    """Initial parameters of the Section 4.1 model: every entry ~ U(-1/sqrt(H), 1/sqrt(H))."""
    rng = _rng(seed)
    k = 1.0 / math.sqrt(H)
    return dict(w_ih=_uniform(rng, (H, I), k), w_hh=_uniform(rng, (H, H), k), b_ih=_uniform(rng, (H,), k),
                b_hh=_uniform(rng, (H,), k), w_out=_uniform(rng, (C, H), k), b_out=_uniform(rng, (C,), k))


def rnn_inputs_norm_preserving(T, B, H=20, I=1, C=10, gain=1.05, seed=BASE_SEED):
    """Test-only variant whose recurrent matrix is gain * (random orthogonal).

    With the default initialisation the gradient shrinks by about one half per
    step, so dL/dh_t underflows fp32 some 125 steps before T and parity far from
    the end of the sequence would compare zeros with zeros.  A scaled orthogonal
    W_hh together with small inputs keeps |dL/dh_t| within a few orders of
    magnitude over thousands of steps, which makes every time step a real test.
    """
    rng = _rng(seed)
    inp = rnn_inputs(T, B, H, I, C, seed=seed + 7919)
    q, r = np.linalg.qr(rng.standard_normal((H, H)))
    q = q * np.sign(np.diag(r))[None, :]
    inp["w_hh"] = (gain * q).astype(np.float32)
    inp["x"] = (0.05 * inp["x"]).astype(np.float32)
    inp["w_ih"] = (0.2 * inp["w_ih"]).astype(np.float32)
    inp["b"] = (0.05 * inp["b"]).astype(np.float32)
    return inp


def gru_inputs(T, B, H=128, I=1, C=11, seed=BASE_SEED + 3, audio=True):
    """GRU workload (Section 4.2 cell, gate order r, z, n).

    The input is an audio-like stream standing in for the MFCC features of the
    paper's instrument-classification set: per sample and input channel, the sum
    of three sinusoids with frequencies ~ U(0, 0.5) cycles per step and phases
    ~ U(0, 2 pi), plus N(0, 0.1) noise.
    """
    rng = _rng(seed)
    k = 1.0 / math.sqrt(H)
    if audio:
        f = rng.uniform(0.0, 0.5, size=(3, B, I))
        ph = rng.uniform(0.0, 2.0 * math.pi, size=(3, B, I))
        t = np.arange(T, dtype=np.float64)[:, None, None]
        x = np.zeros((T, B, I))
        for j in range(3):
            x += np.sin(2.0 * math.pi * f[j][None] * t + ph[j][None])
        x += 0.1 * rng.standard_normal((T, B, I))
        x = x.astype(np.float32)
    else:
        x = rng.standard_normal((T, B, I)).astype(np.float32)
    return dict(
        cell="gru", T=T, B=B, H=H, I=I, C=C, x=x,
        w_ih=_uniform(rng, (3 * H, I), k),
        w_hh=_uniform(rng, (3 * H, H), k),
        b_ih=_uniform(rng, (3 * H,), k),
        b_hh=_uniform(rng, (3 * H,), k),
        w_out=_uniform(rng, (C, H), k),
        b_out=_uniform(rng, (C,), k),
        labels=rng.integers(0, C, size=(B,)).astype(np.int32),
    )


def config_inputs(index: int):
    """Inputs of recurrent configuration `index` (0..3) with its fixed seed."""
    c = CONFIGS[index]
    if c["cell"] == "rnn":
        return rnn_inputs(c["T"], c["B"], c["H"], c["I"], c["C"], seed=BASE_SEED + index)
    return gru_inputs(c["T"], c["B"], c["H"], c["I"], c["C"], seed=BASE_SEED + index)


def random_jacobian_chain(T, B, H, seed=0, scale=None, dtype=np.float32):
    """A chain of T random dense H x H matrices per sample plus a seed vector.

    Entries ~ N(0, scale^2) with scale = 1/sqrt(H) by default, so products keep
    roughly unit norm.  Used to exercise the scan on inputs that are not RNN
    Jacobians.
    """
    rng = _rng(seed)
    s = (1.0 / math.sqrt(H)) if scale is None else scale
    jt = (s * rng.standard_normal((T, B, H, H))).astype(dtype)
    seed_vec = rng.standard_normal((B, H)).astype(dtype)
    return jt, seed_vec


def reflection_jacobian_chain(T, B, H, seed=0, jitter=0.02, dtype=np.float32):
    """A chain of dense matrices c * (I - 2 v v^T / |v|^2) with c ~ U(1 - jitter, 1 + jitter).

    Each factor is a scaled Householder reflection, so products neither vanish
    nor overflow over tens of thousands of steps while every entry is non-zero.
    """
    rng = _rng(seed)
    v = rng.standard_normal((T, B, H))
    v /= np.linalg.norm(v, axis=-1, keepdims=True)
    c = rng.uniform(1.0 - jitter, 1.0 + jitter, size=(T, B, 1, 1))
    jt = c * (np.eye(H)[None, None] - 2.0 * v[..., :, None] * v[..., None, :])
    seed_vec = rng.standard_normal((B, H))
    return jt.astype(dtype), seed_vec.astype(dtype)


# --------------------------------------------------------------------------
# Pruned VGG-11-style CNN (Section 4.3 stand-in): layer list, weights, masks.
# --------------------------------------------------------------------------

VGG11_CONV_CHANNELS = (64, 128, 256, 256, 512, 512, 512, 512)
VGG11_POOL_AFTER = (1, 2, 4, 6, 8)          # 1-based conv indices followed by 2x2 max-pool
VGG11_FC = (512, 512, 10)


@dataclass
class Layer:
    kind: str                 # "conv", "relu", "pool", "fc"
    in_shape: tuple           # (c, h, w) or (d,)
    out_shape: tuple
    weight: np.ndarray | None = None   # conv: [co, ci, 3, 3]; fc: [out, in]; already masked
    mask: np.ndarray | None = None     # bool, same shape as weight (True = kept)
    bias: np.ndarray | None = None


def magnitude_mask(w: np.ndarray, keep_fraction: float) -> np.ndarray:
    """Boolean mask keeping the ceil(keep_fraction * size) entries of largest |w|.

    Ties are broken towards the lower flat index (stable sort on -|w|).
    """
    flat = np.abs(w.reshape(-1).astype(np.float64))
    keep = int(math.ceil(keep_fraction * flat.size))
    order = np.argsort(-flat, kind="stable")
    m = np.zeros(flat.size, dtype=bool)
    m[order[:keep]] = True
    return m.reshape(w.shape)


def cnn_layers(conv_channels=VGG11_CONV_CHANNELS, pool_after=VGG11_POOL_AFTER,
               fc=VGG11_FC, in_shape=(3, 32, 32), prune=0.9, seed=BASE_SEED + 4):
    """Layer list of the pruned VGG-11-style network with He-normal weights.

    Conv/FC weights ~ N(0, 2/fan_in), biases zero, then per layer the
    `prune` fraction of smallest-magnitude weights is masked out (set to 0 and
    recorded as structurally absent in `mask`).  Returns (layers, image).
    """
    rng = _rng(seed)
    layers = []
    c, h, w = in_shape
    for li, co in enumerate(conv_channels, start=1):
        fan_in = c * 9
        wt = (math.sqrt(2.0 / fan_in) * rng.standard_normal((co, c, 3, 3))).astype(np.float32)
        m = magnitude_mask(wt, 1.0 - prune)
        wt = np.where(m, wt, np.float32(0)).astype(np.float32)
        layers.append(Layer("conv", (c, h, w), (co, h, w), wt, m, np.zeros(co, np.float32)))
        layers.append(Layer("relu", (co, h, w), (co, h, w)))
        c = co
        if li in pool_after:
            layers.append(Layer("pool", (c, h, w), (c, h // 2, w // 2)))
            h, w = h // 2, w // 2
    d = c * h * w
    for fi, dout in enumerate(fc):
        wt = (math.sqrt(2.0 / d) * rng.standard_normal((dout, d))).astype(np.float32)
        m = magnitude_mask(wt, 1.0 - prune)
        wt = np.where(m, wt, np.float32(0)).astype(np.float32)
        layers.append(Layer("fc", (d,), (dout,), wt, m, np.zeros(dout, np.float32)))
        if fi != len(fc) - 1:
            layers.append(Layer("relu", (dout,), (dout,)))
        d = dout
    image = rng.standard_normal(in_shape).astype(np.float32)
    label = int(rng.integers(0, fc[-1]))
    return layers, image, label
