"""Algorithm 1 run for K' iterations at the FULL layer widths of the non-convex bf16 workloads, on the smallest ring
the ring kernels take (n = 3), fresh minibatches every iteration, for both device paths:

  * two calls     dpsgd_grad + in-place dpsgd_mix_step
  * one call      dpsgd_step (weight gradients of the large MLP layers formed inside the mix kernel)

Two gates per iteration k, as for the convex workloads:
  (i)  single step: the device is handed the oracle's X_k (rounded to fp32) and its X_{k+1} is compared; strict;
  (ii) trajectory: the device runs on its own iterates and they are compared with the oracle's X_{k+1}: reported per
       iteration together with the first iteration over the bar (if any), and asserted, because they do stay under it.

Both oracles run the recursion: the one with the workload's bf16 operand roundings (tight bars) and the plain fp64
one (the 2e-2 bar of the bf16 workloads on X, the node average, the loss and the consensus distance).  K' is what
about two minutes of oracle time allow: the oracle is plain scalar C."""
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest
import torch

import oracle
from paper_1705_09056_amd import binding as B
from paper_1705_09056_amd import synth
from paper_1705_09056_amd.configs import CONFIGS, shrink

from conftest import check_close, max_err, rel_err
from gpu_util import bf16_dev, from_dev, oracle_topo_for, to_dev, topo_for

pytestmark = pytest.mark.gpu
TOL = 2e-2      # bar of the bf16 workloads
TIGHT = 3e-3    # one step against the oracle with the same operand roundings


def run_trajectory(cfg, iters):
    d = synth.model_dim(cfg.model_kind, cfg.widths)
    ld = synth.padded_stride(d, 256)
    topo_o = oracle_topo_for(cfg)
    model = B.Model(cfg.model_kind, cfg.widths, compute_bf16=True)
    gamma = np.float32(cfg.gamma)
    X0 = synth.make_replicas(cfg).astype(np.float64)      # x_{0,i} = x_0 for every worker (Algorithm 1, Require)
    Xr, Xp = X0, X0                                       # oracle trajectories: bf16 operands / plain fp64
    free = {"two-call": to_dev(X0, ld), "dpsgd_step": to_dev(X0, ld)}
    G = torch.full((cfg.n, ld), 777.0, device="cuda")
    loss = torch.zeros(cfg.n, device="cuda")
    cons = torch.zeros(1, device="cuda")
    xbar = torch.zeros(d, device="cuda")
    first_over = {name: None for name in free}
    worst = {name: 0.0 for name in free}
    pool = ThreadPoolExecutor(max_workers=2)
    print(f"trajectory {cfg.name}: widths={cfg.widths} n={cfg.n} B={cfg.batch} gamma={cfg.gamma} iterations={iters} "
          f"of K={CONFIGS[cfg.index].iters}", flush=True)
    print("   k | single step, update vs rounding oracle (two-call, dpsgd_step) | own trajectory, X vs rounding oracle "
          "| displacement X - X_0 | X vs plain fp64 oracle | loss vs plain | consensus distance vs rounding / plain oracle",
          flush=True)

    def advance(ctx, name, X, inp_d, tgt_d):
        if name == "two-call":
            ctx.grad(model, X, inp_d, tgt_d, cfg.batch, G, loss, input_is_bf16=True)
            ctx.mix_step(X, G, X, cons)
        else:
            ctx.step(model, X, inp_d, tgt_d, cfg.batch, G, loss, cons, input_is_bf16=True)

    with B.Dpsgd(cfg.n, d, topo_for(cfg), cfg.gamma, ld=ld) as ctx:
        for k in range(iters):
            inp, tgt = synth.make_batch(cfg, k)
            inp_d, tgt_d = bf16_dev(inp), torch.from_numpy(tgt).cuda()
            fr = pool.submit(oracle.iteration, cfg.model_kind, cfg.widths, topo_o, gamma, Xr, inp, tgt, True)
            fp = pool.submit(oracle.iteration, cfg.model_kind, cfg.widths, topo_o, gamma, Xp, inp, tgt, False)
            Xr_next, _, loss_r = fr.result()
            Xp_next, _, loss_p = fp.result()
            line = [f"{k:4d}"]
            # (i) one step from the oracle's iterate
            for name in free:
                Xs = to_dev(Xr, ld)
                advance(ctx, name, Xs, inp_d, tgt_d)
                start = Xr.astype(np.float32).astype(np.float64)
                e, m = check_close(from_dev(Xs, d) - start, Xr_next - start, TIGHT, f"k={k} {name} single-step update",
                                   flips=True)
                assert rel_err(loss.cpu().numpy(), loss_r) < TIGHT
                line.append(f"{e:.2e}/{m:.2e}")
            # (ii) the device's own trajectory
            for name, X in free.items():
                advance(ctx, name, X, inp_d, tgt_d)
                ctx.mean(X, xbar)
                got = from_dev(X, d)
                e_r = rel_err(got, Xr_next)
                e_disp = rel_err(got - X0, Xr_next - X0)
                e_p = rel_err(got, Xp_next)
                e_loss = rel_err(loss.cpu().numpy(), loss_p)
                line.append(f"{name}: {e_r:.2e} | {e_disp:.2e} | {e_p:.2e} (max element {max_err(got, Xp_next):.2e} rms) "
                            f"| {e_loss:.2e}")
                worst[name] = max(worst[name], e_r, e_p)
                if first_over[name] is None and max(e_r, e_p) >= TOL:
                    first_over[name] = k
                check_close(got, Xr_next, TOL, f"k={k} {name} X vs rounding oracle")
                # against the plain oracle the iterate is held in the Frobenius norm only.  Element by element the
                # rounding of the workload shows in the parameters that move fastest (the 10-class layer, the
                # biases, which start at zero): they drift from the un-rounded trajectory by 2-4 % of their own
                # displacement per step, which after some iterations is a large multiple of the rms of the whole
                # matrix, although it stays a few percent of those parameters themselves.
                assert e_p < TOL, f"k={k} {name} X vs plain oracle: {e_p:.3e}"
                assert e_loss < TOL
                assert rel_err(xbar.cpu().numpy(), oracle.mean(Xp_next)) < TOL
                # the consensus distance is made of differences of gradients only (all workers started from one
                # x_0), so it feels the operand rounding twice as much as X does: reported against both oracles,
                # held to the bar against the one with the same roundings
                c_r, c_p = oracle.consensus(Xr_next), oracle.consensus(Xp_next)
                line.append(f"M {abs(float(cons) - c_r) / c_r:.2e} / {abs(float(cons) - c_p) / c_p:.2e}")
                assert float(cons) == pytest.approx(c_r, rel=TOL)
            print("  " + "  ".join(line), flush=True)
            Xr, Xp = Xr_next, Xp_next
    pool.shutdown()
    for name in free:
        print(f"  {name}: worst relative error of X over {iters} iterations {worst[name]:.3e}; first iteration over "
              f"{TOL:g}: {first_over[name]}", flush=True)
    # the two device paths stay together too
    a, b = from_dev(free["two-call"], d), from_dev(free["dpsgd_step"], d)
    print(f"  two-call vs dpsgd_step after {iters} iterations: {rel_err(a, b):.3e} (max element {max_err(a, b):.3e} rms)",
          flush=True)
    assert rel_err(a, b) < TOL


@pytest.mark.timeout(400)
def test_config2_trajectory_full_widths():
    run_trajectory(shrink(CONFIGS[2], n=3), iters=40)


@pytest.mark.timeout(400)
def test_config3_trajectory_full_widths():
    run_trajectory(shrink(CONFIGS[3], n=3), iters=8)


@pytest.mark.timeout(400)
def test_config4_trajectory_full_size_images():
    run_trajectory(shrink(CONFIGS[4], n=3), iters=CONFIGS[4].iters)
