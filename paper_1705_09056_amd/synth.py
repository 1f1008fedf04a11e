"""Seeded synthetic inputs for the D-PSGD hot path (numpy only).

This module serves both the CPU oracle's tests and the HIP path, so it holds
none of the method's arithmetic: it only draws the random numbers a workload
needs (initial point x_0 of Algorithm 1, the per-worker minibatches xi_{k,i} of
Algorithm 1 step 2, the teacher that labels them) and describes where each
layer's parameters sit inside a worker's flattened parameter vector.

The inputs stand in for the image-classification workloads of Section 5.1
(32x32x3 images, 10 classes): same shapes and class count, values ~ N(0,1),
labels from a random Gaussian teacher.
"""
from __future__ import annotations

from typing import List, NamedTuple, Tuple

import numpy as np

from .configs import (BASE_SEED, MODEL_LSQ, MODEL_MLP, MODEL_RESNET20,
                      MODEL_SOFTMAX, Workload)

# stream tags (third key word of the seed sequence)
_TAG_BATCH, _TAG_TEACHER, _TAG_XSTAR, _TAG_X0, _TAG_MISC = 11, 12, 13, 14, 15


def rng(cfg_index: int, tag: int, *key: int, seed: int = BASE_SEED) -> np.random.Generator:
    """Independent stream for (seed, config, tag, key...)."""
    return np.random.default_rng([seed, cfg_index, tag, *key])


# --------------------------------------------------------------------------- bf16
def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16 (ties to even); result stays float32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    u = (u + 0x7FFF + lsb) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(a.shape)


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """Upper 16 bits of float32 values that are already bf16-representable."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    assert not np.any(u & 0xFFFF), "value is not bf16-representable"
    return (u >> 16).astype(np.uint16).reshape(a.shape)


# ------------------------------------------------------------------ parameter layout
class Param(NamedTuple):
    name: str
    offset: int
    shape: Tuple[int, ...]
    fan_in: int        # 0 for biases
    size: int


def param_layout(model_kind: int, widths) -> List[Param]:
    """Order of the parameters inside one worker's vector: layer by layer,
    weight (out x in [x kh x kw], row-major) followed by its bias."""
    out: List[Param] = []
    off = 0

    def add(name, shape, fan_in):
        nonlocal off
        size = int(np.prod(shape))
        out.append(Param(name, off, tuple(shape), fan_in, size))
        off += size

    if model_kind == MODEL_LSQ:
        add("x", (widths[0],), 0)
    elif model_kind in (MODEL_SOFTMAX, MODEL_MLP):
        for l in range(len(widths) - 1):
            add(f"W{l}", (widths[l + 1], widths[l]), widths[l])
            add(f"b{l}", (widths[l + 1],), 0)
    elif model_kind == MODEL_RESNET20:
        cin, _h, _w, base, blocks, classes = widths
        add("stem.W", (base, cin, 3, 3), cin * 9)
        add("stem.b", (1,), 0)
        c_prev = base
        for s in range(3):
            c = base << s
            for j in range(blocks):
                add(f"s{s}b{j}.W1", (c, c_prev, 3, 3), c_prev * 9)
                add(f"s{s}b{j}.b1", (1,), 0)
                add(f"s{s}b{j}.W2", (c, c, 3, 3), c * 9)
                add(f"s{s}b{j}.b2", (1,), 0)
                c_prev = c
        add("fc.W", (classes, c_prev), c_prev)
        add("fc.b", (classes,), 0)
    else:
        raise ValueError(model_kind)
    return out


def model_dim(model_kind: int, widths) -> int:
    lay = param_layout(model_kind, widths)
    return lay[-1].offset + lay[-1].size


def padded_stride(d: int, multiple: int = 64) -> int:
    """Row stride (in floats) the harness allocates for the n x d replica matrix."""
    return (d + multiple - 1) // multiple * multiple


# ----------------------------------------------------------------------- draws
def make_x0(cfg: Workload) -> np.ndarray:
    """Common initial point x_0 (Algorithm 1, Require): zeros for the convex
    workloads, one Kaiming-normal draw N(0, 2/fan_in) with zero biases otherwise.
    In the CNN, which has no normalisation layers, the second conv of each of the
    R residual blocks is scaled by 1/sqrt(2R) so that the residual sums keep the
    activations at unit scale at x_0."""
    d = model_dim(cfg.model_kind, cfg.widths)
    x0 = np.zeros(d, dtype=np.float32)
    if cfg.model_kind in (MODEL_MLP, MODEL_RESNET20):
        g = rng(cfg.index, _TAG_X0)
        nblocks = 3 * cfg.widths[4] if cfg.model_kind == MODEL_RESNET20 else 0
        for p in param_layout(cfg.model_kind, cfg.widths):
            if p.fan_in:
                std = np.sqrt(2.0 / p.fan_in)
                if p.name.endswith(".W2"):
                    std /= np.sqrt(2.0 * nblocks)
                x0[p.offset:p.offset + p.size] = g.standard_normal(p.size, dtype=np.float32) * np.float32(std)
    return x0


def make_replicas(cfg: Workload, spread: float = 0.0, key: int = 0) -> np.ndarray:
    """n x d matrix whose rows are x_0 (+ an optional per-worker perturbation so that
    single-step tests see workers that disagree, as they do after the first iteration)."""
    x0 = make_x0(cfg)
    X = np.tile(x0, (cfg.n, 1))
    if spread:
        g = rng(cfg.index, _TAG_MISC, key)
        scale = np.float32(spread) * np.maximum(np.abs(x0), np.float32(0.05))
        X = X + g.standard_normal(X.shape, dtype=np.float32) * scale
    return np.ascontiguousarray(X, dtype=np.float32)


def teacher(cfg: Workload) -> np.ndarray:
    classes = cfg.widths[-1]
    return rng(cfg.index, _TAG_TEACHER).standard_normal((classes, cfg.features))


def x_star(cfg: Workload) -> np.ndarray:
    return rng(cfg.index, _TAG_XSTAR).standard_normal(cfg.features)


def make_batch(cfg: Workload, k: int, workers=None):
    """Minibatches xi_{k,i} of iteration k for the given workers (default: all).

    Returns (inputs float32 [m][B][features], targets) with targets float32
    [m][B] for least squares and int32 labels [m][B] otherwise.  With
    ``cfg.bf16`` the inputs are already rounded to bf16-representable values.
    """
    workers = range(cfg.n) if workers is None else workers
    B, F = cfg.batch, cfg.features
    xs, ts = [], []
    aux = x_star(cfg) if cfg.model_kind == MODEL_LSQ else teacher(cfg)
    for i in workers:
        g = rng(cfg.index, _TAG_BATCH, k, i)
        a = g.standard_normal((B, F), dtype=np.float32)
        if cfg.bf16:
            a = round_to_bf16(a)
        if cfg.model_kind == MODEL_LSQ:
            y = a.astype(np.float64) @ aux + 0.1 * g.standard_normal(B)
            ts.append(y.astype(np.float32))
        else:
            score = a.astype(np.float64) @ aux.T
            ts.append(np.argmax(score, axis=1).astype(np.int32))
        xs.append(a)
    return np.stack(xs), np.stack(ts)
