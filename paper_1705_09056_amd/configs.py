"""The five synthetic workloads of the D-PSGD hot path, as data.

Each entry fixes the workload model, the number of simulated workers n, the
topology of the weight matrix W (Section 3: symmetric, doubly stochastic), the
per-worker minibatch, the step length gamma and the iteration count K of
Algorithm 1.  Nothing here computes anything; the seeded generators that turn a
config into arrays live in ``synth.py``.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Tuple

# model kinds (values match the C-ABI enum and, separately, the oracle's enum)
MODEL_LSQ = 0
MODEL_SOFTMAX = 1
MODEL_MLP = 2
MODEL_RESNET20 = 3

BASE_SEED = 170509056


@dataclass(frozen=True)
class Workload:
    index: int                 # position in the benchmark's config list
    name: str
    model_kind: int
    widths: Tuple[int, ...]    # LSQ: (features,); SOFTMAX/MLP: layer widths;
    #                            RESNET20: (in_ch, height, width, base_ch, blocks_per_stage, classes)
    n: int                     # simulated workers
    topology: str              # "ring" | "torus"
    torus_dims: Tuple[int, int] = (0, 0)
    batch: int = 32            # per-worker minibatch
    gamma: float = 0.1
    iters: int = 100           # K
    bf16: bool = False         # inputs rounded to bf16 and bf16 MFMA operands
    features: int = field(default=0)  # flattened input features per sample


def _mk(index, name, kind, widths, n, topo, batch, gamma, iters, bf16, dims=(0, 0)):
    if kind == MODEL_RESNET20:
        feat = widths[0] * widths[1] * widths[2]
    else:
        feat = widths[0]
    return Workload(index, name, kind, tuple(widths), n, topo, dims, batch, gamma, iters, bf16, feat)


CONFIGS = (
    _mk(0, "lsq_ring8", MODEL_LSQ, (64,), 8, "ring", 32, 0.01, 100, False),
    _mk(1, "softmax_ring16", MODEL_SOFTMAX, (3072, 10), 16, "ring", 128, 0.05, 200, False),
    _mk(2, "mlp2_ring32", MODEL_MLP, (3072, 1024, 10), 32, "ring", 128, 0.1, 100, True),
    _mk(3, "mlp3_ring64", MODEL_MLP, (3072, 4096, 4096, 10), 64, "ring", 32, 0.1, 50, True),
    _mk(4, "resnet20_ring112", MODEL_RESNET20, (3, 32, 32, 16, 3, 10), 112, "ring", 32, 0.1, 20, True),
)

# configs[3] is run on a ring and on an 8x8 torus; gamma is not given for it in the
# benchmark definition, so the value of its neighbours (0.1) is used.
CONFIG3_TORUS = _mk(3, "mlp3_torus8x8", MODEL_MLP, (3072, 4096, 4096, 10), 64, "torus", 32, 0.1, 50, True, (8, 8))


def by_name(name: str) -> Workload:
    for c in CONFIGS + (CONFIG3_TORUS,):
        if c.name == name:
            return c
    raise KeyError(name)


def shrink(cfg: Workload, **kw) -> Workload:
    """A copy of ``cfg`` with some fields replaced (tests use reduced sizes)."""
    d = dict(index=cfg.index, name=cfg.name, model_kind=cfg.model_kind, widths=cfg.widths, n=cfg.n,
             topology=cfg.topology, torus_dims=cfg.torus_dims, batch=cfg.batch, gamma=cfg.gamma,
             iters=cfg.iters, bf16=cfg.bf16, features=cfg.features)
    d.update(kw)
    w = d["widths"]
    d["features"] = w[0] * w[1] * w[2] if d["model_kind"] == MODEL_RESNET20 else w[0]
    return Workload(**d)
