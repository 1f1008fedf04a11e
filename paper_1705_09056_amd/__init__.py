"""MI355X-native hot path of decentralized parallel SGD (D-PSGD).

``configs`` and ``synth`` describe and generate the synthetic workloads; ``binding`` is the thin
ctypes layer over the C-ABI library built from ``csrc/`` (imported on first use so that the
input generators stay importable on machines without the built library).
"""
from . import configs, synth  # noqa: F401

__all__ = ["configs", "synth"]
