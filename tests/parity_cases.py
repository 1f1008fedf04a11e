"""Inputs of the bf16 gradient parity cases, built on the host from the seeded generators only (no arithmetic of
the method): shared by the GPU parity tests, by the CPU test that measures what the workload's operand rounding
alone does to the gradient, and by the script that writes that test's stored values."""
import numpy as np

from paper_1705_09056_amd import synth
from paper_1705_09056_amd.configs import CONFIGS, shrink

# (widths, minibatch, workers) of the MLP cases on 64-float-aligned row strides
MLP_ALIGNED = [
    ((3072, 1024, 10), 128, 2),        # configs[2] layer shapes
    ((3072, 256, 256, 10), 32, 3),     # configs[3] structure, narrower hidden layers
    ((512, 4096, 10), 32, 2),          # a full-width 4096 hidden layer
    ((256, 128, 10), 64, 2),           # the 64-row tiling
    ((256, 128, 64, 10), 130, 2),      # more than one row block
    ((64, 272, 7), 37, 3),             # class layer on the split-contraction kernel, ragged minibatch
    ((128, 256, 32), 33, 2),           # 32 outputs: the widest class layer that kernel takes
    ((128, 256, 33), 33, 2),           # 33 outputs: back on the general tile
]

# CNN cases: (widths, minibatch, workers, deep); deep = three blocks per stage
RESNET = [
    ((2, 6, 6, 2, 1, 3), 2, 2, False),
    ((3, 8, 8, 4, 1, 10), 3, 2, False),
    ((3, 7, 5, 2, 2, 4), 2, 3, False),       # odd image sizes, two blocks per stage
    ((3, 8, 8, 16, 2, 10), 4, 2, False),     # the benchmark's channel counts on small images
    ((3, 16, 16, 16, 1, 10), 5, 2, False),
    ((3, 32, 32, 16, 1, 10), 3, 2, False),   # full-size images, one block per stage
    ((3, 16, 16, 16, 3, 10), 8, 2, True),    # three blocks per stage
]


# Bars of the deep CNN cases (three blocks per stage, 19 convs, no normalisation), in units of the 2e-2 bar of the bf16
# workloads.  They come from a CPU experiment, tests/test_oracle_bf16_gap.py::test_sum_precision_alone_moves_the_deep_cnn:
# ONE implementation (PyTorch autograd with the workload's bf16 casts) run with fp32 sums and with fp64 sums on these
# very inputs ends 4e-4 ... 9e-3 apart on the whole gradient and up to 1.9e-2 on one layer (a sum that differs in its
# last bits now and then stores the neighbouring bf16 activation, which now and then flips a ReLU further down), while
# the one-block networks stay at 1e-6.  So: the whole gradient is held to the bar itself, one layer to twice the bar
# (the experiment's worst layer with a margin of two), and a scalar conv bias - one sum over all pixels, which can sit
# on a cancellation - to the bar in units of max(its own size, the rms of all scalar bias gradients).
DEEP_WHOLE_BAR = 1.0
DEEP_LAYER_BAR = 2.0


def scalar_bias_errors(g, ref, layout):
    """{name: |g - ref| / max(|ref|, rms of all scalar-bias entries of ref)} over the single-element blocks."""
    g, ref = np.asarray(g, np.float64), np.asarray(ref, np.float64)
    ones = [p for p in layout if p.size == 1]
    if not ones:
        return {}
    scale = np.sqrt(np.mean([np.mean(ref[..., p.offset] ** 2) for p in ones]))
    return {p.name: float(np.max(np.abs(g[..., p.offset] - ref[..., p.offset]) /
                                 np.maximum(np.abs(ref[..., p.offset]), scale))) for p in ones}


def mlp_cfg(widths, batch, n):
    return shrink(CONFIGS[2], widths=widths, batch=batch, n=n)


def mlp_inputs(cfg, k=0, spread=0.3, extra_bias=0.0):
    """(X [n][d] float32, inputs, targets) of an MLP / softmax-regression gradient case."""
    X = synth.make_replicas(cfg, spread=spread, key=k)
    if extra_bias:
        X = X + np.float32(extra_bias) * synth.rng(cfg.index, 98, k).standard_normal(X.shape).astype(np.float32)
    inp, tgt = synth.make_batch(cfg, k)
    return X, inp, tgt


def resnet_cfg(widths, batch, n):
    return shrink(CONFIGS[4], widths=widths, batch=batch, n=n)


def resnet_inputs(cfg, spread=0.3):
    """(X, inputs, targets) of a CNN gradient case; biases are non-zero so that every bias path is exercised."""
    X = synth.make_replicas(cfg, spread=spread)
    rb = synth.rng(cfg.index, 96)
    for p in synth.param_layout(cfg.model_kind, cfg.widths):
        if not p.fan_in:
            X[:, p.offset:p.offset + p.size] = 0.05 * rb.standard_normal((cfg.n, p.size)).astype(np.float32)
    inp, tgt = synth.make_batch(cfg, 0)
    return X, inp, tgt


def case_id(widths, batch, n):
    return "x".join(str(w) for w in widths) + f"_B{batch}_n{n}"
