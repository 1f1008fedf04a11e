"""GPU parity of dpsgd_grad with bf16 MFMA operands (softmax regression / ReLU MLP) against the
CPU oracle in its bf16-operand mode (operands of every contraction rounded to bf16, fp64 sums), so
that ReLU decisions are taken on the same rounded values on both sides.  Bar: 2e-2 relative
Frobenius; the kernels are expected to sit far below it (fp32 vs fp64 accumulation only), which
TIGHT checks.  The distance to the un-rounded fp64 gradient is printed as the cost of bf16."""
import numpy as np
import pytest
import torch

import oracle
from paper_1705_09056_amd import binding as B
from paper_1705_09056_amd import synth
from paper_1705_09056_amd.configs import CONFIGS, CONFIG3_TORUS, MODEL_MLP, MODEL_SOFTMAX, shrink

from conftest import rel_err
from gpu_util import bf16_dev, from_dev, oracle_topo_for, to_dev, topo_for

pytestmark = pytest.mark.gpu
TOL = 2e-2
TIGHT = 2e-3


def grad_case(cfg, ld, k=0, spread=0.3, bf16_inputs=True, extra_bias=0.0):
    d = synth.model_dim(cfg.model_kind, cfg.widths)
    X = synth.make_replicas(cfg, spread=spread, key=k)
    if extra_bias:
        X = X + np.float32(extra_bias) * synth.rng(cfg.index, 98, k).standard_normal(X.shape).astype(np.float32)
    inp, tgt = synth.make_batch(cfg, k)
    Gref, lref = oracle.grad_all(cfg.model_kind, cfg.widths, X, inp, tgt, bf16_operands=True)
    Gplain, _ = oracle.grad_all(cfg.model_kind, cfg.widths, X, inp, tgt)
    Xd = to_dev(X, ld)
    Gd = torch.full_like(Xd, 777.0)
    loss = torch.zeros(cfg.n, device="cuda")
    inp_d = bf16_dev(inp) if bf16_inputs else torch.from_numpy(inp).cuda()
    tgt_d = torch.from_numpy(tgt).cuda()
    model = B.Model(cfg.model_kind, cfg.widths, compute_bf16=True)
    print(f"grad bf16 {cfg.name} widths={cfg.widths} n={cfg.n} B={cfg.batch} ld={ld} bf16_in={bf16_inputs}", flush=True)
    with B.Dpsgd(cfg.n, d, topo_for(cfg), cfg.gamma, ld=ld) as ctx:
        ctx.grad(model, Xd, inp_d, tgt_d, cfg.batch, Gd, loss, input_is_bf16=bf16_inputs)
        ctx.grad(model, Xd, inp_d, tgt_d, cfg.batch, Gd, loss, input_is_bf16=bf16_inputs)   # workspace reuse
        torch.cuda.synchronize()
    G = from_dev(Gd, d)
    e_all = rel_err(G, Gref)
    lay = synth.param_layout(cfg.model_kind, cfg.widths)
    per = {p.name: rel_err(G[:, p.offset:p.offset + p.size], Gref[:, p.offset:p.offset + p.size]) for p in lay}
    print("  rel err G %.3e  loss %.3e  per-layer %s" % (e_all, rel_err(loss.cpu().numpy(), lref),
                                                        {k_: "%.2e" % v for k_, v in per.items()}), flush=True)
    print("  distance to the un-rounded fp64 gradient: %.3e" % rel_err(G, Gplain), flush=True)
    assert e_all < TIGHT
    assert all(v < TIGHT for v in per.values())
    assert rel_err(loss.cpu().numpy(), lref) < TIGHT


@pytest.mark.parametrize("widths,batch,n", [
    ((3072, 1024, 10), 128, 2),        # configs[2] layer shapes
    ((3072, 256, 256, 10), 32, 3),     # configs[3] structure, narrower hidden layers
    ((512, 4096, 10), 32, 2),          # a full-width 4096 hidden layer
    ((256, 128, 10), 64, 2),           # the 64-row tiling
    ((256, 128, 64, 10), 130, 2),      # more than one row block
    ((64, 272, 7), 37, 3),             # class layer on the split-contraction kernel, ragged minibatch
    ((128, 256, 32), 33, 2),           # 32 outputs: the widest class layer that kernel takes
    ((128, 256, 33), 33, 2),           # 33 outputs: back on the general tile
])
def test_mlp_bf16_aligned(widths, batch, n):
    cfg = shrink(CONFIGS[2], widths=widths, batch=batch, n=n)
    d = synth.model_dim(MODEL_MLP, widths)
    grad_case(cfg, synth.padded_stride(d))


@pytest.mark.parametrize("widths,batch,n", [((100, 70, 33, 5), 37, 4), ((96, 50, 10), 24, 3), ((33, 7, 3), 1, 2),
                                             ((130, 260, 9), 70, 2),
                                             ((200, 150, 70, 10), 20, 8),    # 8 workers: tiles renumbered per XCD
                                             ((136, 72, 10), 64, 16)])
def test_mlp_bf16_ragged(widths, batch, n):
    cfg = shrink(CONFIGS[2], widths=widths, batch=batch, n=n)
    d = synth.model_dim(MODEL_MLP, widths)
    grad_case(cfg, synth.padded_stride(d))
    grad_case(cfg, d + 1, bf16_inputs=False)     # odd row stride, fp32 inputs converted on the device


def test_softmax_regression_bf16():
    cfg = shrink(CONFIGS[1], widths=(3072, 10), batch=128, n=3, bf16=True)
    d = synth.model_dim(MODEL_SOFTMAX, cfg.widths)
    grad_case(cfg, synth.padded_stride(d), extra_bias=0.05)


def sampled_full_size(cfg, sample):
    """Full-size launch (all n workers, the shape bench.py times); the oracle checks `sample` workers."""
    d = synth.model_dim(cfg.model_kind, cfg.widths)
    ld = synth.padded_stride(d)
    x0 = synth.make_x0(cfg)
    rng = synth.rng(cfg.index, 97)
    Xd = torch.zeros(cfg.n, ld, device="cuda")
    Xd[:, :d] = torch.from_numpy(x0).cuda()
    rows = {}
    for i in sample:
        xi = x0 + np.float32(0.3) * np.maximum(np.abs(x0), np.float32(0.02)) * rng.standard_normal(d, dtype=np.float32)
        rows[i] = xi
        Xd[i, :d] = torch.from_numpy(xi).cuda()
    inp, tgt = synth.make_batch(cfg, 0)
    Gd = torch.zeros_like(Xd)
    loss = torch.zeros(cfg.n, device="cuda")
    model = B.Model(cfg.model_kind, cfg.widths, compute_bf16=True)
    print(f"full-size grad {cfg.name}: n={cfg.n} d={d} B={cfg.batch}; oracle on workers {sample}", flush=True)
    with B.Dpsgd(cfg.n, d, topo_for(cfg), cfg.gamma, ld=ld) as ctx:
        ctx.grad(model, Xd, bf16_dev(inp), torch.from_numpy(tgt).cuda(), cfg.batch, Gd, loss, input_is_bf16=True)
        torch.cuda.synchronize()
    for i in sample:
        l, g = oracle.loss_grad(cfg.model_kind, cfg.widths, rows[i], inp[i], tgt[i], bf16_operands=True)
        e = rel_err(Gd[i, :d].cpu().numpy(), g)
        print(f"  worker {i}: rel err G {e:.3e}, loss {float(loss[i]):.5f} vs {l:.5f}", flush=True)
        assert e < TIGHT
        assert abs(float(loss[i]) - l) < TIGHT * abs(l)
    del Xd, Gd
    torch.cuda.empty_cache()


def test_config2_full_size_sampled_workers():
    sampled_full_size(CONFIGS[2], [0, 17, 31])


def test_config3_full_size_sampled_workers():
    sampled_full_size(CONFIGS[3], [5, 63])


def test_config2_short_trajectory_single_step_gate():
    """Reduced configs[2] (hidden width 128): every iteration one GPU step from the oracle's iterate."""
    cfg = shrink(CONFIGS[2], widths=(3072, 128, 10), n=4, iters=6)
    d = synth.model_dim(cfg.model_kind, cfg.widths)
    ld = synth.padded_stride(d)
    topo_o = oracle_topo_for(cfg)
    model = B.Model(cfg.model_kind, cfg.widths, compute_bf16=True)
    Xo = synth.make_replicas(cfg).astype(np.float64)
    Xfree = to_dev(Xo, ld)
    Gd = torch.full_like(Xfree, 777.0)
    with B.Dpsgd(cfg.n, d, topo_for(cfg), cfg.gamma, ld=ld) as ctx:
        for k in range(cfg.iters):
            inp, tgt = synth.make_batch(cfg, k)
            inp_d, tgt_d = bf16_dev(inp), torch.from_numpy(tgt).cuda()
            Xn, Gref, _ = oracle.iteration(cfg.model_kind, cfg.widths, topo_o, np.float32(cfg.gamma), Xo, inp, tgt,
                                           bf16_operands=True)
            Xs = to_dev(Xo, ld)
            ctx.grad(model, Xs, inp_d, tgt_d, cfg.batch, Gd, input_is_bf16=True)
            assert rel_err(from_dev(Gd, d), Gref) < TOL
            ctx.mix_step(Xs, Gd, Xs)
            step_err = rel_err(from_dev(Xs, d), Xn)
            ctx.grad(model, Xfree, inp_d, tgt_d, cfg.batch, Gd, input_is_bf16=True)
            ctx.mix_step(Xfree, Gd, Xfree)
            traj_err = rel_err(from_dev(Xfree, d), Xn)
            print(f"  k={k}: single-step {step_err:.3e}  trajectory {traj_err:.3e}", flush=True)
            assert step_err < TOL and traj_err < TOL
            Xo = Xn
