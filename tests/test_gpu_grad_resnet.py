"""GPU parity of dpsgd_grad for the BN-free ResNet-20-style CNN against the CPU oracle.

The oracle in its bf16-operand mode (image, conv weights, stored activations and deltas rounded to bf16; fp64
sums) is the tight check.  Networks with at most two blocks per stage must agree to TIGHT (only fp32-vs-fp64
summation differs), whole gradient and per layer, Frobenius and element-wise.  With three blocks per stage (19
convs, no normalisation) a 1e-7 summation difference now and then moves a stored activation to the neighbouring
bf16 value, and such a perturbation now and then flips a ReLU further down (tests/test_oracle_bf16_gap.py shows
the same with fp32 against fp64 sums on the CPU alone, and the bars of the deep cases come from it): the whole
gradient is held to the 2e-2 bar of the bf16 workloads, one layer to twice that, a scalar conv bias to the bar in
units of the typical scalar-bias gradient (tests/parity_cases.py).
The plain fp64 oracle (no rounding inside) binds the loss at 2e-2, and the gradient through
dist(GPU, plain) == dist(bf16-operand oracle, plain) to two digits: the distance is the workload's operand
rounding, and the kernels add nothing to it."""
import numpy as np
import pytest
import torch

import oracle
from paper_1705_09056_amd import binding as B
from paper_1705_09056_amd import synth
from paper_1705_09056_amd.configs import CONFIGS, MODEL_RESNET20, shrink

from conftest import check_close, max_err, rel_err
from gpu_util import bf16_dev, from_dev, oracle_topo_for, to_dev, topo_for
from parity_cases import DEEP_LAYER_BAR, DEEP_WHOLE_BAR, RESNET, resnet_inputs, scalar_bias_errors

pytestmark = pytest.mark.gpu
TOL = 2e-2
TIGHT = 3e-3


def grad_case(cfg, ld, spread=0.3, bf16_inputs=True, plain=True, deep=False):
    d = synth.model_dim(cfg.model_kind, cfg.widths)
    X, inp, tgt = resnet_inputs(cfg, spread)
    lay = synth.param_layout(cfg.model_kind, cfg.widths)
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
    print("  rel err G %.3e (max element %.3e rms)  loss %.3e  worst layer %s %.3e" % (
        rel_err(G, Gref), max_err(G, Gref), rel_err(loss.cpu().numpy(), lref), worst, per[worst]), flush=True)
    assert rel_err(loss.cpu().numpy(), lref) < TIGHT
    if plain:
        Gp, lp = oracle.grad_all(cfg.model_kind, cfg.widths, X, inp, tgt)
        gap_gpu, gap_rounding = rel_err(G, Gp), rel_err(Gref, Gp)
        print("  distance to the un-rounded fp64 gradient: GPU %.3e, bf16-operand oracle %.3e" % (gap_gpu, gap_rounding),
              flush=True)
        assert rel_err(loss.cpu().numpy(), lp) < TOL
        assert abs(gap_gpu - gap_rounding) <= (0.1 if deep else 0.02) * gap_rounding + 2e-5
    whole, layer = (DEEP_WHOLE_BAR * TOL, DEEP_LAYER_BAR * TOL) if deep else (TIGHT, TIGHT)
    check_close(G, Gref, whole, "G vs bf16-operand oracle", flips=True)
    for p in lay:
        if p.size > 1:
            check_close(G[:, p.offset:p.offset + p.size], Gref[:, p.offset:p.offset + p.size], layer, p.name,
                        flips=True)
    sb = scalar_bias_errors(G, Gref, lay)
    print("  worst scalar conv bias: %.3e" % max(sb.values()), flush=True)
    assert max(sb.values()) < (TOL if deep else TIGHT), sb


@pytest.mark.parametrize("widths,batch,n,deep", RESNET)
def test_resnet(widths, batch, n, deep):
    cfg = shrink(CONFIGS[4], widths=widths, batch=batch, n=n)
    d = synth.model_dim(MODEL_RESNET20, widths)
    grad_case(cfg, synth.padded_stride(d), deep=deep)


def test_resnet_fp32_inputs_and_odd_stride():
    cfg = shrink(CONFIGS[4], widths=(3, 8, 8, 4, 1, 10), batch=3, n=2)
    d = synth.model_dim(MODEL_RESNET20, cfg.widths)
    grad_case(cfg, d + 3, bf16_inputs=False)


def test_resnet_fp32_inputs_on_the_mfma_path():
    cfg = shrink(CONFIGS[4], widths=(3, 16, 16, 16, 1, 10), batch=9, n=2)
    d = synth.model_dim(MODEL_RESNET20, cfg.widths)
    grad_case(cfg, synth.padded_stride(d), bf16_inputs=False)


@pytest.mark.parametrize("widths,batch", [((3, 32, 16, 16, 1, 10), 3), ((3, 16, 32, 16, 1, 10), 2), ((3, 48, 32, 16, 1, 10), 2)])
def test_resnet_rectangular_images(widths, batch):
    """Heights and widths that differ, and a height (48) that 16 divides but 32 does not: the 16-row workgroup tiles of
    the convolutions and the 16-row bands of the weight gradient at stage 2 see 32 x 16, 16 x 32 and 48 x 32 pixels
    (stage 2: half of that, stage 3: a quarter, where 8-row tiles take over)."""
    cfg = shrink(CONFIGS[4], widths=widths, batch=batch, n=2)
    d = synth.model_dim(MODEL_RESNET20, widths)
    grad_case(cfg, synth.padded_stride(d), plain=False)


def test_resnet_config4_shape_two_workers():
    cfg = shrink(CONFIGS[4], n=3)
    d = synth.model_dim(MODEL_RESNET20, cfg.widths)
    grad_case(cfg, synth.padded_stride(d), deep=True)


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
        lp, gp = oracle.loss_grad(cfg.model_kind, cfg.widths, X[i], inp[i], tgt[i])
        e, m = check_close(G[i], g, TOL, f"worker {i}", flips=True)
        gap_gpu, gap_rounding = rel_err(G[i], gp), rel_err(g, gp)
        print(f"  worker {i}: rel err G {e:.3e} (max element {m:.3e} rms), loss {float(loss[i]):.5f} vs {l:.5f} "
              f"(plain fp64 {lp:.5f}); distance to the un-rounded gradient: GPU {gap_gpu:.3e}, oracle {gap_rounding:.3e}",
              flush=True)
        assert abs(float(loss[i]) - l) < TIGHT * abs(l)
        assert abs(float(loss[i]) - lp) < TOL * abs(lp)
        assert abs(gap_gpu - gap_rounding) <= 0.1 * gap_rounding


@pytest.mark.parametrize("widths,batch,n", [((3, 32, 32, 16, 1, 10), 3, 2), ((3, 32, 32, 16, 3, 10), 4, 8),
                                            ((3, 16, 16, 16, 2, 10), 6, 3), ((3, 8, 8, 16, 1, 10), 5, 2)])
def test_workgroup_tile_height_changes_no_bit(widths, batch, n):
    """The convolutions with 8 or 16 output rows of an image per workgroup ("conv_band_rows"; the default picks per
    convolution): which rows share a workgroup changes no sum, so gradient and loss are identical bit for bit (the
    default's result is the one the oracle checks above)."""
    cfg = shrink(CONFIGS[4], widths=widths, batch=batch, n=n)
    d = synth.model_dim(MODEL_RESNET20, widths)
    ld = synth.padded_stride(d)
    X, inp, tgt = resnet_inputs(cfg, 0.3)
    Xd, inp_d, tgt_d = to_dev(X, ld), bf16_dev(inp), torch.from_numpy(tgt).cuda()
    model = B.Model(cfg.model_kind, cfg.widths, compute_bf16=True)
    got = {}
    for rows in (0, 8, 16):
        Gd = torch.full_like(Xd, 777.0)
        loss = torch.zeros(cfg.n, device="cuda")
        print(f"conv_band_rows={rows} widths={widths} n={n} B={batch}", flush=True)
        with B.Dpsgd(cfg.n, d, topo_for(cfg), cfg.gamma, ld=ld) as ctx:
            ctx.set_option("conv_band_rows", rows)
            ctx.grad(model, Xd, inp_d, tgt_d, cfg.batch, Gd, loss, input_is_bf16=True)
            torch.cuda.synchronize()
        got[rows] = (from_dev(Gd, d), loss.cpu().numpy())
    for rows in (8, 16):
        assert np.array_equal(got[rows][0], got[0][0]), f"gradient differs with {rows} rows per workgroup"
        assert np.array_equal(got[rows][1], got[0][1])


@pytest.mark.parametrize("widths,batch,n", [((3, 32, 32, 16, 3, 10), 2, 2),    # the benchmark's network: 16, 32 and 64 channels
                                             ((3, 48, 32, 16, 2, 10), 2, 8),    # six bands per image; 8 workers: one XCD per worker
                                             ((3, 8, 32, 16, 2, 10), 3, 2),     # 16 channels, one band per image: both halo rows lie outside it
                                             ((3, 32, 16, 16, 1, 10), 1, 3)])   # 16 pixels wide: a pair of MFMA tiles spans two rows
def test_residual_block_in_one_launch_changes_no_bit(widths, batch, n):
    """Both forward convolutions of a resolution-keeping residual block in one launch (the intermediate activation
    stays in LDS for the second one) against the two launches ("conv_block" 0): the same matrix instructions on the
    same operands, so gradient and loss are bit for bit the same."""
    cfg = shrink(CONFIGS[4], widths=widths, batch=batch, n=n)
    d = synth.model_dim(MODEL_RESNET20, widths)
    ld = synth.padded_stride(d)
    X, inp, tgt = resnet_inputs(cfg, 0.3)
    model = B.Model(cfg.model_kind, cfg.widths, compute_bf16=True)
    out = []
    for setting in (1, 0):
        Xd = to_dev(X, ld)
        Gd = torch.full_like(Xd, 777.0)
        loss = torch.zeros(cfg.n, device="cuda")
        print(f"conv_block={setting} widths={widths} n={n} B={batch}", flush=True)
        with B.Dpsgd(cfg.n, d, topo_for(cfg), cfg.gamma, ld=ld) as ctx:
            ctx.set_option("conv_block", setting)
            ctx.grad(model, Xd, bf16_dev(inp), torch.from_numpy(tgt).cuda(), cfg.batch, Gd, loss, input_is_bf16=True)
            torch.cuda.synchronize()
        out.append((Gd.clone(), loss.clone()))
    assert torch.equal(out[0][1], out[1][1]), "loss differs"
    assert torch.equal(out[0][0], out[1][0]), "gradient differs"
