"""Writes tests/golden/bf16_rounding_gap.txt: for every bf16 gradient parity case, the relative Frobenius distance
between the oracle's gradient with the workload's bf16 operand roundings and the oracle's plain fp64 gradient, on
the inputs the GPU tests use.  Calls the oracle and the seeded generators only.

    python tests/golden/make_bf16_rounding_gap.py
"""
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))
sys.path.insert(0, os.path.dirname(HERE))

import oracle  # noqa: E402
from conftest import rel_err  # noqa: E402
from parity_cases import MLP_ALIGNED, RESNET, case_id, mlp_cfg, mlp_inputs, resnet_cfg, resnet_inputs  # noqa: E402


def gap(cfg, X, inp, tgt):
    g_round, l_round = oracle.grad_all(cfg.model_kind, cfg.widths, X, inp, tgt, bf16_operands=True)
    g_plain, l_plain = oracle.grad_all(cfg.model_kind, cfg.widths, X, inp, tgt)
    return rel_err(g_round, g_plain), rel_err(l_round, l_plain)


def rows():
    for widths, batch, n in MLP_ALIGNED:
        cfg = mlp_cfg(widths, batch, n)
        yield "mlp_" + case_id(widths, batch, n), gap(cfg, *mlp_inputs(cfg))
    for widths, batch, n, _deep in RESNET:
        cfg = resnet_cfg(widths, batch, n)
        yield "resnet_" + case_id(widths, batch, n), gap(cfg, *resnet_inputs(cfg))


if __name__ == "__main__":
    out = os.path.join(HERE, "bf16_rounding_gap.txt")
    with open(out, "w") as f:
        f.write("# distance of the gradient with bf16 operand roundings from the plain fp64 gradient (relative Frobenius),\n"
                "# and the same for the per-worker losses; both from the CPU oracle alone (make_bf16_rounding_gap.py).\n"
                "# The roundings are the benchmark's \"bf16 compute\" (configs[2]-[4]); the paper trains in fp32 (Section 5.1).\n")
        for name, (g, l) in rows():
            f.write(f"{name} {g:.6e} {l:.6e}\n")
            print(name, f"{g:.3e} {l:.3e}", flush=True)
