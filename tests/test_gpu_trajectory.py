"""Algorithm 1 run for K' iterations at the FULL layer widths of the non-convex bf16 workloads, on the smallest ring
the ring kernels take (n = 3), fresh minibatches every iteration, for both device paths:

  * two calls     dpsgd_grad + in-place dpsgd_mix_step
  * one call      dpsgd_step (weight gradients of the large MLP layers formed inside the mix kernel)

Two gates per iteration k, as for the convex workloads:
  (i)  single step: the device is handed the oracle's X_k (rounded to fp32) and its X_{k+1} is compared; strict;
  (ii) trajectory: the device runs on its own iterates and they are compared with the oracles' X_{k+1}.  Every quantity
       (iterate, its displacement from x_0, node average, per-worker loss, consensus distance) is reported per iteration
       with the first iteration at which it goes over the 2e-2 bar, if it does.  The iterate and the node average are
       asserted under the bar against both oracles for the first 10 iterations; beyond that a free-running non-convex
       trajectory is reported, not asserted: at configs[2] the loss drifts over the bar against the un-rounded oracle
       after ~15 iterations and the iterate itself after ~24 (different ReLU decisions, then growing drift).

Both oracles run the recursion: the one with the workload's bf16 operand roundings and the plain fp64 one.  K' is what
one to two minutes of oracle time allow: the oracle is plain scalar C.  Each iteration's line goes to the terminal as
it is computed (past pytest's capture), so a run of these minutes-long tests shows its progress."""
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
HORIZON = 10    # iterations over which a free-running trajectory must stay under the bar


def run_trajectory(cfg, iters, capsys):
    def say(text):
        with capsys.disabled():
            print(text, flush=True)

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
    first_over = {name: {} for name in free}
    worst = {name: {} for name in free}
    pool = ThreadPoolExecutor(max_workers=2)
    say(f"\ntrajectory {cfg.name}: widths={cfg.widths} n={cfg.n} B={cfg.batch} gamma={cfg.gamma} iterations={iters} "
        f"of K={CONFIGS[cfg.index].iters}")
    say("   k | single step, update vs rounding oracle: Frobenius/largest element (two-call, dpsgd_step) | own trajectory of "
        "each path")

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
            # (ii) the device's own trajectory: every quantity is recorded with the first iteration it goes over the
            # bar; the iterate and the node average are also asserted (they stay under it), the loss and the consensus
            # distance of a free-running non-convex trajectory are reported
            for name, X in free.items():
                advance(ctx, name, X, inp_d, tgt_d)
                ctx.mean(X, xbar)
                got = from_dev(X, d)
                c_r, c_p = oracle.consensus(Xr_next), oracle.consensus(Xp_next)
                q = {"X vs rounding oracle": rel_err(got, Xr_next),
                     "displacement X - X_0 vs rounding oracle": rel_err(got - X0, Xr_next - X0),
                     "X vs plain oracle": rel_err(got, Xp_next),
                     "xbar vs plain oracle": rel_err(xbar.cpu().numpy(), oracle.mean(Xp_next)),
                     "loss vs rounding oracle": rel_err(loss.cpu().numpy(), loss_r),
                     "loss vs plain oracle": rel_err(loss.cpu().numpy(), loss_p),
                     "consensus vs rounding oracle": abs(float(cons) - c_r) / c_r,
                     "consensus vs plain oracle": abs(float(cons) - c_p) / c_p}
                line.append(f"{name}: X {q['X vs rounding oracle']:.2e} | disp {q['displacement X - X_0 vs rounding oracle']:.2e} "
                            f"| X/plain {q['X vs plain oracle']:.2e} (max element {max_err(got, Xp_next):.2e} rms) "
                            f"| loss {q['loss vs rounding oracle']:.2e} / plain {q['loss vs plain oracle']:.2e} "
                            f"| M {q['consensus vs rounding oracle']:.2e} / plain {q['consensus vs plain oracle']:.2e}")
                for key, val in q.items():
                    worst[name][key] = max(worst[name].get(key, 0.0), val)
                    if val >= TOL and key not in first_over[name]:
                        first_over[name][key] = k
                # A free-running trajectory of a non-convex model is REPORTED: two trajectories that differ in the last
                # bits of a sum take different ReLU decisions sooner or later and then drift apart at a growing rate
                # (the paper gives no guidance here; its theory bounds averages over iterations, not iterates).  What
                # is asserted: the iterate and the node average stay under the bar against both oracles for the first
                # HORIZON iterations, in the Frobenius norm (the element-wise bars belong to gate (i): element by
                # element the drift shows first in the parameters that move fastest - the 10-class layer, the biases,
                # which start at zero - as a large multiple of the rms of the whole matrix).
                if k < HORIZON:
                    assert q["X vs rounding oracle"] < TOL, f"k={k} {name} X vs rounding oracle: {q['X vs rounding oracle']:.3e}"
                    assert q["X vs plain oracle"] < TOL, f"k={k} {name} X vs plain oracle: {q['X vs plain oracle']:.3e}"
                    assert q["xbar vs plain oracle"] < TOL
            say("  " + "  ".join(line))
            Xr, Xp = Xr_next, Xp_next
    pool.shutdown()
    for name in free:
        say(f"  {name}, worst over {iters} iterations: " + "; ".join(f"{k_} {v:.2e}" for k_, v in worst[name].items()))
        say(f"  {name}, first iteration over {TOL:g}: " + ("; ".join(f"{k_}: k={v}" for k_, v in first_over[name].items()) or "none"))
    # the two device paths against each other
    a, b = from_dev(free["two-call"], d), from_dev(free["dpsgd_step"], d)
    say(f"  two-call vs dpsgd_step after {iters} iterations: {rel_err(a, b):.3e} (max element {max_err(a, b):.3e} rms)")


@pytest.mark.timeout(400)
def test_config2_trajectory_full_widths(capsys):
    run_trajectory(shrink(CONFIGS[2], n=3), 32, capsys)


@pytest.mark.timeout(400)
def test_config3_trajectory_full_widths(capsys):
    run_trajectory(shrink(CONFIGS[3], n=3), 4, capsys)


@pytest.mark.timeout(400)
def test_config4_trajectory_full_size_images(capsys):
    run_trajectory(shrink(CONFIGS[4], n=3), 12, capsys)
