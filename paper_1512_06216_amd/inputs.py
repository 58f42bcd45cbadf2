"""Seeded synthetic inputs for the SACP gradient-synchronisation path.

This module only draws numbers and shapes them; it contains none of the method's
arithmetic (no packing, no reconstruction, no update, no cost rule).  Both the HIP
path's tests/benchmarks and the CPU oracle's tests consume these arrays, so the two
sides see identical bits.

Shapes follow the paper's workloads: AlexNet's parameter split (Table 3: conv 2.3 M,
FC 59 M weights), the fc6/fc7 example of Section 4.3.1 (4096 x 4096, batch 256), the
21 841-way ImageNet-22K classifier (Section 5.1.3), batch 256 per node on 8 nodes
(Section 5.1.2).  Values are synthetic stand-ins for real activations / errors:

  activations  a = max(0, N(0,1))          (about half exact zeros, like post-ReLU)
  errors       delta ~ N(0, std)           or (softmax(z) - onehot(y)) / B, z ~ N(0,1)
  weights      W ~ N(0, std 0.01), momentum buffer zero
  conv grads   G_p ~ N(0, std 1e-3), one dense copy per worker

Naming: M = layer inputs (length of a), N = layer outputs (length of delta), B = batch
per worker, P = workers, K = P*B stacked rows.  W and Mom are N x M row-major.
"""
from __future__ import annotations

import numpy as np

BASE_SEED = 151206216

# name -> FC layer workload (the four single-layer configurations)
FC_CONFIGS = {
    1: dict(name="tiny_fc_f32", M=256, N=128, B=32, P=4, factor_dtype="f32",
            delta_kind="gauss", delta_std=1e-2),
    2: dict(name="classifier_fc_f32", M=4096, N=1000, B=256, P=8, factor_dtype="f32",
            delta_kind="gauss", delta_std=1e-3),
    3: dict(name="fc6_bf16", M=9216, N=4096, B=256, P=8, factor_dtype="bf16",
            delta_kind="gauss", delta_std=1e-3),
    4: dict(name="cls22k_bf16", M=4096, N=21841, B=256, P=8, factor_dtype="bf16",
            delta_kind="softmax", delta_std=None),
}

# Full 8-layer CNN iteration (config 5): conv filter banks (out, in/group, kh, kw) and the
# three FC layers (M inputs -> N outputs), listed bottom-up.
CONV_SHAPES = [(96, 3, 11, 11), (256, 48, 5, 5), (384, 256, 3, 3), (384, 192, 3, 3),
               (256, 192, 3, 3)]
CONV_NAMES = ["conv1", "conv2", "conv3", "conv4", "conv5"]
FC_SHAPES = [(9216, 4096), (4096, 4096), (4096, 1000)]
FC_NAMES = ["fc6", "fc7", "fc8"]
CNN_B = 256
CNN_P = 8
CNN_S = 8

LR = 0.01
MU = 0.9


def conv_sizes():
    """Flattened parameter count of each conv layer of config 5."""
    return [int(np.prod(s)) for s in CONV_SHAPES]


def _rng(*key):
    return np.random.default_rng(np.random.SeedSequence([BASE_SEED, *[int(k) for k in key]]))


def relu_gauss(rng, shape):
    x = rng.standard_normal(shape, dtype=np.float32)
    np.maximum(x, 0.0, out=x)
    return x


def softmax_minus_onehot(rng, B, N):
    """(softmax(z) - onehot(y)) / B with z ~ N(0,1), y uniform; rows sum to ~0."""
    z = rng.standard_normal((B, N))
    z -= z.max(axis=1, keepdims=True)
    e = np.exp(z)
    e /= e.sum(axis=1, keepdims=True)
    y = rng.integers(0, N, size=B)
    e[np.arange(B), y] -= 1.0
    e /= B
    return e.astype(np.float32)


def fc_layer(M, N, B, P, seed, delta_kind="gauss", delta_std=1e-3, w_std=1e-2,
             mom_std=0.0):
    """Per-worker factor blocks and the layer state for one FC layer.

    Returns dict: act[p] (B x M), delta[p] (B x N), W (N x M), Mom (N x M), all float32
    C-contiguous.
    """
    act, delta = [], []
    for p in range(P):
        act.append(relu_gauss(_rng(seed, 1, p), (B, M)))
    for p in range(P):
        r = _rng(seed, 2, p)
        if delta_kind == "gauss":
            delta.append((r.standard_normal((B, N), dtype=np.float32)
                          * np.float32(delta_std)))
        elif delta_kind == "softmax":
            delta.append(softmax_minus_onehot(r, B, N))
        else:
            raise ValueError(delta_kind)
    W = _rng(seed, 3).standard_normal((N, M), dtype=np.float32) * np.float32(w_std)
    if mom_std:
        Mom = _rng(seed, 4).standard_normal((N, M), dtype=np.float32) * np.float32(mom_std)
    else:
        Mom = np.zeros((N, M), dtype=np.float32)
    return dict(M=M, N=N, B=B, P=P, act=act, delta=delta, W=W, Mom=Mom)


def fc_config(cfg_id, **override):
    c = dict(FC_CONFIGS[cfg_id])
    c.update(override)
    d = fc_layer(c["M"], c["N"], c["B"], c["P"], seed=cfg_id, delta_kind=c["delta_kind"],
                 delta_std=c["delta_std"])
    d["factor_dtype"] = c["factor_dtype"]
    d["name"] = c["name"]
    return d


def fc_layer_integer(M, N, B, P, seed, amax=3):
    """Small-integer factors and state: every partial sum stays below 2^24, so any
    summation order gives the same fp32 (and bf16-factor) result bit for bit.
    Pair with lr and mu that are powers of two."""
    r = _rng(seed, 5)
    act = [r.integers(0, amax + 1, size=(B, M)).astype(np.float32) for _ in range(P)]
    delta = [r.integers(-amax, amax + 1, size=(B, N)).astype(np.float32) for _ in range(P)]
    W = r.integers(-64, 65, size=(N, M)).astype(np.float32)
    Mom = r.integers(-8, 9, size=(N, M)).astype(np.float32)
    return dict(M=M, N=N, B=B, P=P, act=act, delta=delta, W=W, Mom=Mom)


def dense_layer(n, P, seed, g_std=1e-3, w_std=1e-2, mom_std=0.0):
    """P dense gradient copies of an n-parameter layer plus its state (flat float32)."""
    G = [_rng(seed, 6, p).standard_normal(n, dtype=np.float32) * np.float32(g_std)
         for p in range(P)]
    W = _rng(seed, 7).standard_normal(n, dtype=np.float32) * np.float32(w_std)
    if mom_std:
        Mom = _rng(seed, 8).standard_normal(n, dtype=np.float32) * np.float32(mom_std)
    else:
        Mom = np.zeros(n, dtype=np.float32)
    return dict(n=n, P=P, G=G, W=W, Mom=Mom)


def dense_layer_integer(n, P, seed, amax=7):
    r = _rng(seed, 9)
    G = [r.integers(-amax, amax + 1, size=n).astype(np.float32) for _ in range(P)]
    W = r.integers(-64, 65, size=n).astype(np.float32)
    Mom = r.integers(-8, 9, size=n).astype(np.float32)
    return dict(n=n, P=P, G=G, W=W, Mom=Mom)


def cnn_iteration(seed=5, B=CNN_B, P=CNN_P, scale=1):
    """Config 5: five conv layers (dense copies) and three FC layers (factors).

    `scale` > 1 divides every FC width and conv filter count for CPU-sized tests
    (the layer structure and ordering stay the same).  Layers are returned
    bottom-up; the path issues them top-down.
    """
    layers = []
    for i, (name, shp) in enumerate(zip(CONV_NAMES, CONV_SHAPES)):
        o, c, kh, kw = shp
        n = max(1, o // scale) * c * kh * kw
        d = dense_layer(n, P, seed * 100 + i)
        d.update(name=name, kind="conv")
        layers.append(d)
    for i, (name, (M, N)) in enumerate(zip(FC_NAMES, FC_SHAPES)):
        d = fc_layer(max(1, M // scale), max(1, N // scale), B, P, seed * 100 + 10 + i)
        d.update(name=name, kind="fc")
        layers.append(d)
    return layers
