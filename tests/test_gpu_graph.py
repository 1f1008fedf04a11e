"""dpsgd_step recorded into a HIP graph: after one eager call has sized the workspace the call only enqueues
kernels, so a caller may capture several iterations and replay them.  Every replay is checked against the same
iterations run eagerly, with eager work and synchronisations between the replays."""
import numpy as np
import pytest
import torch

from paper_1705_09056_amd import binding as B
from paper_1705_09056_amd import synth
from paper_1705_09056_amd.configs import CONFIGS, CONFIG3_TORUS, shrink

from gpu_util import bf16_dev, to_dev, topo_for

pytestmark = pytest.mark.gpu

ITERS = 3      # iterations recorded in one graph
REPLAYS = 3


def graph_case(cfg, bf16, options=()):
    d = synth.model_dim(cfg.model_kind, cfg.widths)
    ld = synth.padded_stride(d)
    model = B.Model(cfg.model_kind, cfg.widths, compute_bf16=bf16)
    batches = []
    for k in range(ITERS):
        inp, tgt = synth.make_batch(cfg, k)
        batches.append((bf16_dev(inp) if bf16 else torch.from_numpy(inp).cuda(), torch.from_numpy(tgt).cuda()))
    X0 = to_dev(synth.make_replicas(cfg), ld)
    print(f"graph {cfg.name} widths={cfg.widths} n={cfg.n} B={cfg.batch} topo={cfg.topology}", flush=True)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        Xe, Xg = X0.clone(), X0.clone()
        G = torch.zeros_like(X0)
        loss_e, loss_g = torch.zeros(ITERS, cfg.n, device="cuda"), torch.zeros(ITERS, cfg.n, device="cuda")
        cons_e, cons_g = torch.zeros(ITERS, device="cuda"), torch.zeros(ITERS, device="cuda")
        ctx = B.Dpsgd(cfg.n, d, topo_for(cfg), cfg.gamma, ld=ld, stream=side)
        for key, value in options:
            ctx.set_option(key, value)

        def iterations(X, loss, cons):
            for k, (inp_d, tgt_d) in enumerate(batches):
                ctx.step(model, X, inp_d, tgt_d, cfg.batch, G, loss[k], cons[k:k + 1], input_is_bf16=bf16)

        scratch = X0.clone()
        iterations(scratch, loss_e, cons_e)     # eager once: the workspace is sized here, outside the capture
        side.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            iterations(Xg, loss_g, cons_g)
        for rep in range(REPLAYS):
            # eager reference of this replay, from the state the graph is about to start from
            Xe.copy_(Xg)
            loss_e.zero_()
            cons_e.zero_()
            iterations(Xe, loss_e, cons_e)
            side.synchronize()
            loss_g.fill_(-1.0)
            cons_g.fill_(-1.0)
            graph.replay()
            side.synchronize()
            same = bool(torch.equal(Xe, Xg))
            diff = float(torch.linalg.vector_norm(Xe[:, :d] - Xg[:, :d]) / torch.linalg.vector_norm(Xe[:, :d]))
            print(f"  replay {rep}: X bit-identical {same}, rel diff {diff:.2e}, consensus {cons_g.tolist()}", flush=True)
            assert diff < 1e-6
            assert torch.allclose(loss_e, loss_g, rtol=1e-5, atol=1e-7)
            assert torch.allclose(cons_e, cons_g, rtol=1e-5, atol=0.0)
            assert bool(torch.all(Xg[:, d:] == X0[:, d:]))     # padding columns untouched
        ctx.close()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()


def test_graph_of_fused_ring_steps():
    graph_case(shrink(CONFIGS[2], widths=(1024, 1024, 10), batch=32, n=6), bf16=True)


def test_graph_with_the_bf16_shadow_option():
    """Recorded calls neither read nor write the bf16 weight copy (its contents at replay time are unknown); the
    eager calls between the replays do.  Both must agree bit for bit."""
    graph_case(shrink(CONFIGS[3], widths=(1024, 1024, 1024, 10), batch=32, n=5), bf16=True,
               options=(("bf16_shadow", 1),))


def test_graph_of_fused_torus_steps():
    graph_case(shrink(CONFIG3_TORUS, widths=(1024, 1024, 10), batch=32, n=12, torus_dims=(3, 4)), bf16=True)


def test_graph_of_fused_steps_on_the_ring_with_a_far_link():
    """The kernel that holds every worker's tile in LDS (a W without a walk kernel), with minibatches of 128 rows:
    the class layer's one-launch backward with its samples split over groups, softmax in the forward launch."""
    graph_case(shrink(CONFIGS[2], widths=(1024, 1024, 10), batch=128, n=10, topology="ring_chord"), bf16=True)


def test_graph_of_fp32_softmax_and_lsq_steps():
    graph_case(shrink(CONFIGS[1], widths=(300, 10), batch=16, n=6), bf16=False)
    graph_case(shrink(CONFIGS[0], widths=(64,), batch=32, n=8), bf16=False)


def test_graph_of_small_cnn_steps():
    graph_case(shrink(CONFIGS[4], batch=4, n=4), bf16=True)
