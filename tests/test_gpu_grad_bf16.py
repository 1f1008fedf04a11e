"""GPU parity of dpsgd_grad with bf16 MFMA operands (softmax regression / ReLU MLP) against the CPU oracle.

Two oracles judge every case.  The plain fp64 oracle (no rounding inside) binds the loss at the 2e-2 bar of
the bf16 workloads, and the gradient through the identity  dist(GPU, plain) == dist(oracle with bf16 operands,
plain)  to two digits: the operand rounding the workload prescribes moves the gradient by 0.2-4e-2 of its norm
whoever computes it (tests/test_oracle_bf16_gap.py shows that on the CPU with two independent implementations),
and the kernel must add nothing to that.  The oracle in its bf16-operand mode (the same operand roundings, fp64
sums; ReLU decisions taken on the same rounded values) is the tight check of the kernel itself: TIGHT on the
whole gradient and per layer, Frobenius and element-wise."""
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest
import torch

import oracle
from paper_1705_09056_amd import binding as B
from paper_1705_09056_amd import synth
from paper_1705_09056_amd.configs import CONFIGS, CONFIG3_TORUS, MODEL_MLP, MODEL_SOFTMAX, shrink

from conftest import check_close, max_err, rel_err
from gpu_util import bf16_dev, from_dev, oracle_topo_for, to_dev, topo_for
from parity_cases import MLP_ALIGNED, mlp_inputs

pytestmark = pytest.mark.gpu
TOL = 2e-2
TIGHT = 2e-3


def grad_case(cfg, ld, k=0, spread=0.3, bf16_inputs=True, extra_bias=0.0):
    d = synth.model_dim(cfg.model_kind, cfg.widths)
    X, inp, tgt = mlp_inputs(cfg, k, spread, extra_bias)
    Gref, lref = oracle.grad_all(cfg.model_kind, cfg.widths, X, inp, tgt, bf16_operands=True)
    Gplain, lplain = oracle.grad_all(cfg.model_kind, cfg.widths, X, inp, tgt)
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
    lay = synth.param_layout(cfg.model_kind, cfg.widths)
    e_all, m_all = check_close(G, Gref, TIGHT, "G vs bf16-operand oracle", flips=True)
    per = {p.name: check_close(G[:, p.offset:p.offset + p.size], Gref[:, p.offset:p.offset + p.size], TIGHT, p.name,
                               flips=True)
           for p in lay}
    print("  rel err G %.3e (max element %.3e rms)  loss %.3e  per-layer %s" % (
        e_all, m_all, rel_err(loss.cpu().numpy(), lref), {k_: "%.2e/%.2e" % v for k_, v in per.items()}), flush=True)
    assert rel_err(loss.cpu().numpy(), lref) < TIGHT
    # against the plain fp64 oracle: the loss meets the bar of the bf16 workloads, and the gradient is as far from
    # the un-rounded one as the operand rounding alone puts it (the CPU oracle with the same roundings), no further
    assert rel_err(loss.cpu().numpy(), lplain) < TOL
    gap_gpu, gap_rounding = rel_err(G, Gplain), rel_err(Gref, Gplain)
    print("  distance to the un-rounded fp64 gradient: GPU %.3e, bf16-operand oracle %.3e" % (gap_gpu, gap_rounding),
          flush=True)
    assert abs(gap_gpu - gap_rounding) <= 0.02 * gap_rounding + 2e-5
    return gap_gpu


@pytest.mark.parametrize("widths,batch,n", MLP_ALIGNED)
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
    # one oracle call is one worker on one thread: the sampled workers and both rounding modes run side by side
    with ThreadPoolExecutor(max_workers=2 * len(sample)) as pool:
        jobs = {(i, mode): pool.submit(oracle.loss_grad, cfg.model_kind, cfg.widths, rows[i], inp[i], tgt[i],
                                       bf16_operands=mode) for i in sample for mode in (True, False)}
        done = {key: job.result() for key, job in jobs.items()}
    for i in sample:
        l, g = done[(i, True)]
        lp, gp = done[(i, False)]
        got = Gd[i, :d].cpu().numpy()
        e, m = check_close(got, g, TIGHT, f"worker {i}", flips=True)
        gap_gpu, gap_rounding = rel_err(got, gp), rel_err(g, gp)
        print(f"  worker {i}: rel err G {e:.3e} (max element {m:.3e} rms), loss {float(loss[i]):.5f} vs {l:.5f} "
              f"(plain fp64 {lp:.5f}); distance to the un-rounded gradient: GPU {gap_gpu:.3e}, oracle {gap_rounding:.3e}",
              flush=True)
        assert abs(float(loss[i]) - l) < TIGHT * abs(l)
        assert abs(float(loss[i]) - lp) < TOL * abs(lp)
        assert abs(gap_gpu - gap_rounding) <= 0.02 * gap_rounding + 2e-5
    del Xd, Gd
    torch.cuda.empty_cache()


def test_config2_full_size_sampled_workers():
    sampled_full_size(CONFIGS[2], [0, 17, 31])


def test_config3_full_size_sampled_workers():
    sampled_full_size(CONFIGS[3], [5, 63])


@pytest.mark.parametrize("widths,batch,n", [((3072, 1024, 10), 128, 3), ((200, 150, 70, 10), 20, 4), ((96, 50, 16), 33, 2)])
def test_class_layer_backward_in_one_launch_agrees_with_the_tiled_kernels(widths, batch, n):
    """The class layer's backward (weight, bias and data gradient, bias gradient of the layer below) as one launch
    against the three launches of the tiled kernels it replaces ("class_bwd" 0): the same products, summed in another
    order, so the gradients agree far inside the bar to the oracle."""
    cfg = shrink(CONFIGS[2], widths=widths, batch=batch, n=n)
    d = synth.model_dim(MODEL_MLP, widths)
    ld = synth.padded_stride(d)
    X, inp, tgt = mlp_inputs(cfg, 0, 0.3, 0.0)
    model = B.Model(cfg.model_kind, cfg.widths, compute_bf16=True)
    out = []
    for setting in (1, 0):
        Xd = to_dev(X, ld)
        Gd = torch.full_like(Xd, 777.0)
        loss = torch.zeros(cfg.n, device="cuda")
        print(f"class_bwd={setting} widths={widths} n={n} B={batch}", flush=True)
        with B.Dpsgd(cfg.n, d, topo_for(cfg), cfg.gamma, ld=ld) as ctx:
            ctx.set_option("class_bwd", setting)
            ctx.grad(model, Xd, bf16_dev(inp), torch.from_numpy(tgt).cuda(), cfg.batch, Gd, loss, input_is_bf16=True)
            torch.cuda.synchronize()
        out.append(from_dev(Gd, d))
    for p in synth.param_layout(cfg.model_kind, cfg.widths):
        sl = slice(p.offset, p.offset + p.size)
        e = rel_err(out[0][:, sl], out[1][:, sl])
        print(f"  {p.name}: one launch vs tiled kernels {e:.3e}", flush=True)
        assert e < 5e-4
