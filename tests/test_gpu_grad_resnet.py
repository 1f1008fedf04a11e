"""GPU parity of dpsgd_grad for the BN-free ResNet-20-style CNN against the CPU oracle in its
bf16-operand mode (image, conv weights, stored activations and deltas rounded to bf16; fp64 sums).

Bar: 2e-2 relative Frobenius on the whole gradient.  Networks with at most two blocks per stage
must agree to TIGHT (only fp32-vs-fp64 summation differs).  With three blocks per stage (19 convs,
no normalisation) a 1e-7 summation difference now and then moves a stored activation to the
neighbouring bf16 value, and such a perturbation now and then flips a ReLU further down; one
flipped unit among N changes that layer's delta by sqrt(1/N), so deep cases sit around 1e-2 and
are held to the bar only."""
import numpy as np
import pytest
import torch

import oracle
from paper_1705_09056_amd import binding as B
from paper_1705_09056_amd import synth
from paper_1705_09056_amd.configs import CONFIGS, MODEL_RESNET20, shrink

from conftest import rel_err
from gpu_util import bf16_dev, from_dev, oracle_topo_for, to_dev, topo_for

pytestmark = pytest.mark.gpu
TOL = 2e-2
TIGHT = 3e-3


def grad_case(cfg, ld, spread=0.3, bf16_inputs=True, plain=True, deep=False):
    d = synth.model_dim(cfg.model_kind, cfg.widths)
    X = synth.make_replicas(cfg, spread=spread)
    # non-zero biases so that every bias path is exercised
    lay = synth.param_layout(cfg.model_kind, cfg.widths)
    rb = synth.rng(cfg.index, 96)
    for p in lay:
        if not p.fan_in:
            X[:, p.offset:p.offset + p.size] = 0.05 * rb.standard_normal((cfg.n, p.size)).astype(np.float32)
    inp, tgt = synth.make_batch(cfg, 0)
    Gref, lref = oracle.grad_all(cfg.model_kind, cfg.widths, X, inp, tgt, bf16_operands=True)
    Xd = to_dev(X, ld)
    Gd = torch.full_like(Xd, 777.0)
    loss = torch.zeros(cfg.n, device="cuda")
    inp_d = bf16_dev(inp) if bf16_inputs else torch.from_numpy(inp).cuda()
    tgt_d = torch.from_numpy(tgt).cuda()
    model = B.Model(cfg.model_kind, cfg.widths, compute_bf16=True)
    print(f"grad resnet widths={cfg.widths} n={cfg.n} B={cfg.batch} ld={ld} bf16_in={bf16_inputs}", flush=True)
    with B.Dpsgd(cfg.n, d, topo_for(cfg), cfg.gamma, ld=ld) as ctx:
        ctx.grad(model, Xd, inp_d, tgt_d, cfg.batch, Gd, loss, input_is_bf16=bf16_inputs)
        torch.cuda.synchronize()
    G = from_dev(Gd, d)
    per = {p.name: rel_err(G[:, p.offset:p.offset + p.size], Gref[:, p.offset:p.offset + p.size]) for p in lay}
    worst = max(per, key=per.get)
    print("  rel err G %.3e  loss %.3e  worst layer %s %.3e" % (rel_err(G, Gref), rel_err(loss.cpu().numpy(), lref),
                                                               worst, per[worst]), flush=True)
    if plain:
        Gp, _ = oracle.grad_all(cfg.model_kind, cfg.widths, X, inp, tgt)
        print("  distance to the un-rounded fp64 gradient: %.3e" % rel_err(G, Gp), flush=True)
    assert rel_err(loss.cpu().numpy(), lref) < TIGHT
    if deep:
        assert rel_err(G, Gref) < TOL
        assert all(v < 3 * TOL for v in per.values()), per
        return
    assert rel_err(G, Gref) < TIGHT
    # single scalars (conv biases) can sit on a cancellation; bound them by the bar, the rest tightly
    for p in lay:
        assert per[p.name] < (TOL if p.size == 1 else 4 * TIGHT), (p.name, per[p.name])


@pytest.mark.parametrize("widths,batch,n", [
    ((2, 6, 6, 2, 1, 3), 2, 2),
    ((3, 8, 8, 4, 1, 10), 3, 2),
    ((3, 7, 5, 2, 2, 4), 2, 3),        # odd image sizes, two blocks per stage
    ((3, 8, 8, 16, 2, 10), 4, 2),      # the benchmark's channel counts on small images
    ((3, 16, 16, 16, 1, 10), 5, 2),
    ((3, 32, 32, 16, 1, 10), 3, 2),    # full-size images, one block per stage
])
def test_resnet_small(widths, batch, n):
    cfg = shrink(CONFIGS[4], widths=widths, batch=batch, n=n)
    d = synth.model_dim(MODEL_RESNET20, widths)
    grad_case(cfg, synth.padded_stride(d))


def test_resnet_three_blocks_per_stage():
    cfg = shrink(CONFIGS[4], widths=(3, 16, 16, 16, 3, 10), batch=8, n=2)
    d = synth.model_dim(MODEL_RESNET20, cfg.widths)
    grad_case(cfg, synth.padded_stride(d), deep=True)


def test_resnet_fp32_inputs_and_odd_stride():
    cfg = shrink(CONFIGS[4], widths=(3, 8, 8, 4, 1, 10), batch=3, n=2)
    d = synth.model_dim(MODEL_RESNET20, cfg.widths)
    grad_case(cfg, d + 3, bf16_inputs=False)


def test_resnet_fp32_inputs_on_the_mfma_path():
    cfg = shrink(CONFIGS[4], widths=(3, 16, 16, 16, 1, 10), batch=9, n=2)
    d = synth.model_dim(MODEL_RESNET20, cfg.widths)
    grad_case(cfg, synth.padded_stride(d), bf16_inputs=False)


def test_resnet_config4_shape_two_workers():
    cfg = shrink(CONFIGS[4], n=3)
    d = synth.model_dim(MODEL_RESNET20, cfg.widths)
    grad_case(cfg, synth.padded_stride(d), plain=False, deep=True)


def test_config4_full_size_sampled_workers():
    """All 112 workers in the launch shape bench.py times; the oracle checks two of them."""
    cfg = CONFIGS[4]
    d = synth.model_dim(cfg.model_kind, cfg.widths)
    ld = synth.padded_stride(d)
    X = synth.make_replicas(cfg, spread=0.3)
    inp, tgt = synth.make_batch(cfg, 0)
    Xd = to_dev(X, ld)
    Gd = torch.full_like(Xd, 777.0)
    loss = torch.zeros(cfg.n, device="cuda")
    model = B.Model(cfg.model_kind, cfg.widths, compute_bf16=True)
    print(f"full-size grad {cfg.name}: n={cfg.n} d={d} B={cfg.batch}", flush=True)
    with B.Dpsgd(cfg.n, d, topo_for(cfg), cfg.gamma, ld=ld) as ctx:
        ctx.grad(model, Xd, bf16_dev(inp), torch.from_numpy(tgt).cuda(), cfg.batch, Gd, loss, input_is_bf16=True)
        torch.cuda.synchronize()
    G = from_dev(Gd, d)
    for i in (3, 111):
        l, g = oracle.loss_grad(cfg.model_kind, cfg.widths, X[i], inp[i], tgt[i], bf16_operands=True)
        e = rel_err(G[i], g)
        print(f"  worker {i}: rel err G {e:.3e}, loss {float(loss[i]):.5f} vs {l:.5f}", flush=True)
        assert e < TOL
        assert abs(float(loss[i]) - l) < TIGHT * abs(l)


def test_config4_short_trajectory():
    """Reduced configs[4] (8x8 images, 4 workers): single-step and free-running gates over 5 iterations."""
    cfg = shrink(CONFIGS[4], widths=(3, 8, 8, 16, 3, 10), n=4, batch=8, iters=5)
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
            ctx.mix_step(Xs, Gd, Xs)
            step_err = rel_err(from_dev(Xs, d), Xn)
            ctx.grad(model, Xfree, inp_d, tgt_d, cfg.batch, Gd, input_is_bf16=True)
            ctx.mix_step(Xfree, Gd, Xfree)
            traj_err = rel_err(from_dev(Xfree, d), Xn)
            print(f"  k={k}: single-step {step_err:.3e}  trajectory {traj_err:.3e}", flush=True)
            assert step_err < TOL          # strict gate: one step from the oracle's iterate
            assert traj_err < 10 * TOL     # free-running non-convex trajectory: reported, loosely bounded
            Xo = Xn
