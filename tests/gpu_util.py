"""Helpers of the GPU parity tests: host <-> device marshalling only."""
import numpy as np
import torch

from paper_1705_09056_amd import binding as B
from paper_1705_09056_amd import synth

PAD = 777.0


def to_dev(a: np.ndarray, ld: int = 0) -> torch.Tensor:
    """[n][d] float array -> CUDA float32 [n][ld]; padding columns hold a sentinel."""
    a = np.asarray(a, dtype=np.float32)
    n, d = a.shape
    ld = ld or d
    t = torch.full((n, ld), PAD, dtype=torch.float32)
    t[:, :d] = torch.from_numpy(a)
    return t.cuda()


def from_dev(t: torch.Tensor, d: int) -> np.ndarray:
    h = t.cpu().numpy()
    if h.shape[1] > d:
        assert np.all(h[:, d:] == PAD), "padding columns were written"
    return h[:, :d].astype(np.float64)


def bf16_dev(a: np.ndarray) -> torch.Tensor:
    """float32 values already bf16-representable -> CUDA bfloat16 tensor of the same shape."""
    bits = synth.bf16_bits(a).astype(np.int16)
    return torch.from_numpy(bits).view(torch.bfloat16).cuda()


def topo_for(cfg):
    if cfg.topology == "ring":
        return B.Topology.ring()
    if cfg.topology == "torus":
        return B.Topology.torus(*cfg.torus_dims)
    if cfg.topology == "ring_chord":
        return B.Topology.ring_chord()
    raise ValueError(cfg.topology)


def oracle_topo_for(cfg):
    import oracle
    if cfg.topology == "ring":
        t = oracle.ring(cfg.n)
    elif cfg.topology == "torus":
        t = oracle.torus(*cfg.torus_dims)
    else:
        t = oracle.ring_chord(cfg.n)
    return t.with_fp32_values()
