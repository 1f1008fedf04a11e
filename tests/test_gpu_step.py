"""GPU parity of dpsgd_step (one whole iteration of Algorithm 1 in place; weight gradients of large MLP
layers formed inside the mix kernel) against the CPU oracle's iteration and against the two-call
sequence dpsgd_grad + dpsgd_mix_step on the same device data."""
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest
import torch

import oracle
from paper_1705_09056_amd import binding as B
from paper_1705_09056_amd import synth
from paper_1705_09056_amd.configs import CONFIGS, CONFIG3_TORUS, shrink

from conftest import check_close, max_err, rel_err
from gpu_util import bf16_dev, from_dev, oracle_topo_for, to_dev, topo_for

pytestmark = pytest.mark.gpu
TOL = 2e-2
TIGHT = 2e-3


def step_case(cfg, bf16=True, spread=0.3, options=(), ld=0, expect_fused=None, topos=None):
    d = synth.model_dim(cfg.model_kind, cfg.widths)
    ld = ld or synth.padded_stride(d)
    X = synth.make_replicas(cfg, spread=spread)
    inp, tgt = synth.make_batch(cfg, 0)
    # topos: (W for the library, the same W for the oracle) where the workload's topology name does not say it
    topo_o = topos[1] if topos else oracle_topo_for(cfg)
    Xn, Gref, lref = oracle.iteration(cfg.model_kind, cfg.widths, topo_o, np.float32(cfg.gamma), X, inp, tgt,
                                      bf16_operands=bf16)
    # the plain fp64 oracle (no rounding inside) binds the iterate-level outputs at the bar of the bf16 workloads
    Xp, _, lplain = (oracle.iteration(cfg.model_kind, cfg.widths, topo_o, np.float32(cfg.gamma), X, inp, tgt)
                     if bf16 else (Xn, Gref, lref))
    model = B.Model(cfg.model_kind, cfg.widths, compute_bf16=bf16)
    inp_d = bf16_dev(inp) if bf16 else torch.from_numpy(inp).cuda()
    tgt_d = torch.from_numpy(tgt).cuda()
    Xa, Xb = to_dev(X, ld), to_dev(X, ld)
    Ga, Gb = torch.full_like(Xa, 777.0), torch.full_like(Xa, 777.0)
    la, lb = torch.zeros(cfg.n, device="cuda"), torch.zeros(cfg.n, device="cuda")
    ca, cb = torch.zeros(1, device="cuda"), torch.zeros(1, device="cuda")
    xbar = torch.zeros(d, device="cuda")
    print(f"step {cfg.name} widths={cfg.widths} n={cfg.n} B={cfg.batch} topo={cfg.topology}", flush=True)
    with B.Dpsgd(cfg.n, d, topos[0] if topos else topo_for(cfg), cfg.gamma, ld=ld) as ctx:
        for key, value in options:
            ctx.set_option(key, value)
        ctx.step(model, Xa, inp_d, tgt_d, cfg.batch, Ga, la, ca, input_is_bf16=bf16)
        ctx.grad(model, Xb, inp_d, tgt_d, cfg.batch, Gb, lb, input_is_bf16=bf16)
        ctx.mix_step(Xb, Gb, Xb, cb)
        ctx.mean(Xa, xbar)
        torch.cuda.synchronize()
    A, Bm = from_dev(Xa, d), from_dev(Xb, d)
    if expect_fused is not None:
        # the scratch gradient of a fused layer's weights is never written: the sentinel is still there
        for p in synth.param_layout(cfg.model_kind, cfg.widths):
            if p.size >= (1 << 20):
                untouched = bool((Ga[:, p.offset:p.offset + p.size] == 777.0).all())
                assert untouched == expect_fused, f"{p.name}: fused={untouched}, expected {expect_fused}"
    X64 = X.astype(np.float64)
    tight, bar = (TIGHT, TOL) if bf16 else (1e-4, 1e-5)
    # the update itself (X_next - X) is what the gradient kernels produce; compare it, not just X_next: over the
    # whole matrix and over every parameter block, Frobenius and element-wise
    e_oracle, m_oracle = check_close(A - X64, Xn - X64, tight, "update vs oracle", flips=bf16)
    for p in synth.param_layout(cfg.model_kind, cfg.widths):
        sl = slice(p.offset, p.offset + p.size)
        check_close((A - X64)[:, sl], (Xn - X64)[:, sl], tight, f"update of {p.name} vs oracle", flips=bf16)
        check_close((A - X64)[:, sl], (Bm - X64)[:, sl], 1e-4, f"update of {p.name}: one call vs two calls")
    e_twocall = rel_err(A, Bm)
    print("  update vs oracle %.3e (max element %.3e rms), X_next vs oracle %.3e, vs plain fp64 oracle %.3e, fused vs "
          "two-call %.3e, consensus %.6g / %.6g / %.6g (plain %.6g)" % (
              e_oracle, m_oracle, rel_err(A, Xn), rel_err(A, Xp), e_twocall, float(ca), float(cb),
              oracle.consensus(Xn), oracle.consensus(Xp)), flush=True)
    check_close(A, Xn, bar, "X_next vs oracle")
    assert e_twocall < 1e-5
    assert rel_err(la.cpu().numpy(), lref) < TIGHT
    assert float(ca) == pytest.approx(oracle.consensus(Xn), rel=1e-3)
    assert float(ca) == pytest.approx(float(cb), rel=1e-4)
    # spec gate of the bf16 workloads against the un-rounded oracle: iterate, node average, loss, consensus
    check_close(A, Xp, bar, "X_next vs plain oracle")
    check_close(xbar.cpu().numpy(), oracle.mean(Xp), bar, "xbar vs plain oracle")
    assert rel_err(la.cpu().numpy(), lplain) < bar
    assert float(ca) == pytest.approx(oracle.consensus(Xp), rel=TOL)


@pytest.mark.parametrize("widths,batch,n", [
    ((1024, 1024, 10), 32, 5),          # one fused layer, the rest through the range mix
    ((1024, 1024, 1024, 10), 32, 4),    # two fused layers
    ((1024, 1024, 96, 10), 48, 3),      # a layer too small to fuse between fused ones; 64-row tiling
    ((2048, 512, 10), 128, 3),          # minibatch 128
    ((1024, 1024, 10), 200, 3),         # minibatch padded to 224: beyond what the LDS operand buffer of the fused kernel holds
    ((100, 70, 33, 5), 37, 4),          # nothing fusable: plain ranges only
])
def test_step_mlp_bf16_ring(widths, batch, n):
    step_case(shrink(CONFIGS[2], widths=widths, batch=batch, n=n))


@pytest.mark.parametrize("dims,widths,batch", [
    ((3, 8), (1024, 1024, 10), 32),          # smallest number of grid rows
    ((8, 8), (1024, 1024, 1024, 10), 32),    # the benchmark's 8 x 8 grid, two fused layers
    ((5, 8), (2048, 512, 10), 96),           # odd number of grid rows, three 32-sample steps
    ((3, 3), (1024, 1024, 10), 32),          # smallest grid: every neighbour is also a wrap-around
    ((4, 5), (1056, 1024, 10), 40),          # 5 columns; inputs a multiple of 32 but not of 64; ragged minibatch
    ((6, 4), (1024, 1056, 64, 10), 32),      # 4 columns, 33 output tiles
    ((3, 7), (2048, 544, 10), 64),           # 7 columns
    ((3, 12), (1024, 1024, 10), 32),         # 12 columns: one group of 12 waves per workgroup
    ((5, 16), (1024, 1024, 10), 32),         # 16 columns, 80 workers: 1024 threads per workgroup
])
def test_step_mlp_bf16_torus(dims, widths, batch):
    """Weight gradient formed inside the torus mix kernel: one wave per grid column, grid rows walked with three
    rows of tiles in registers, row neighbours exchanged through LDS."""
    step_case(shrink(CONFIG3_TORUS, widths=widths, batch=batch, n=dims[0] * dims[1], torus_dims=dims), expect_fused=True)


@pytest.mark.parametrize("topology,n,dims,widths,batch,options", [
    ("ring_chord", 8, None, (1024, 1024, 10), 32, ()),                 # the supplement's ring with a far link: [16][128] tiles
    ("ring_chord", 16, None, (1024, 1024, 1024, 10), 32, ()),          # its 16 workers, two fused layers
    ("ring_chord", 40, None, (1024, 1024, 10), 48, ()),                # 40 workers: [16][32] tiles; two operand steps
    ("ring_chord", 6, None, (1056, 1024, 10), 32, ()),                 # fewer workers than waves; 33 column groups: no wider tile divides
    ("torus", 27, (3, 9), (1024, 1024, 10), 32, (("fused_slab", 2),)),  # 9 grid columns, instead of the torus walk: [16][32] tiles
    ("torus", 16, (2, 8), (1024, 1024, 10), 32, ()),                   # 2 grid rows: neighbours coincide, weights differ per entry
    ("torus", 16, (4, 4), (1024, 1024, 10), 32, (("fused_slab", 2),)),  # instead of the torus walk
    ("torus", 64, (8, 8), (1024, 1024, 10), 32, (("fused_slab", 2),)),  # 64 workers fill the 128 KB
])
def test_step_mlp_bf16_any_topology_through_lds(topology, n, dims, widths, batch, options):
    """Weight gradient formed inside the mix for a W without a walk kernel: every worker's tile in LDS, rows combined
    in CSR order."""
    base = CONFIG3_TORUS if topology == "torus" else CONFIGS[2]
    kw = dict(torus_dims=dims) if topology == "torus" else dict(topology=topology)
    step_case(shrink(base, widths=widths, batch=batch, n=n, **kw), options=options, expect_fused=True)


def test_step_mlp_bf16_csr_topologies_through_lds():
    """General sparse W handed over as CSR: a hypercube (degree 4), the complete graph (every row combines all
    tiles) and a random symmetric doubly stochastic matrix with unequal weights."""
    from test_gpu_mix import hypercube_csr, random_symmetric_ds
    rowptr, col, val = hypercube_csr(4)
    cfg = shrink(CONFIGS[2], widths=(1024, 1024, 10), batch=32, n=16)
    step_case(cfg, expect_fused=True,
              topos=(B.Topology.csr(rowptr, col, val), oracle.Topology(16, rowptr, col, val.astype(np.float64))))
    cfg = shrink(CONFIGS[2], widths=(1024, 1024, 10), batch=32, n=12)
    step_case(cfg, expect_fused=True, topos=(B.Topology.complete(), oracle.complete(12).with_fp32_values()))
    rowptr, col, val = random_symmetric_ds(20, np.random.default_rng(20))
    cfg = shrink(CONFIGS[2], widths=(1024, 1024, 10), batch=64, n=20)
    step_case(cfg, expect_fused=True,
              topos=(B.Topology.csr(rowptr, col, val), oracle.Topology(20, rowptr, col, val.astype(np.float64))))


def test_launch_options_reject_unknown_keys_and_values():
    """dpsgd_set_option: every documented key is accepted with its documented values, anything else is DPSGD_EINVAL and
    leaves the context usable."""
    with B.Dpsgd(8, 64, B.Topology.ring(), 0.1) as ctx:
        for key, good, bad in (("fused_slab", (0, 1, 2), (3, -1)), ("class_bwd", (0, 1), ()), ("fused_lds", (0, 1), ()),
                               ("ring_rows", (0, 1), ()), ("ring_chunks", (0, 1), ()), ("mix_vec", (0, 1, 2, 4), (3, 8)),
                               ("mix_bands", (0, 16), (17, -1)), ("conv_band_rows", (0, 8, 16), (4, 32))):
            for v in good:
                ctx.set_option(key, v)
            for v in bad:
                with pytest.raises(B.DpsgdError) as e:
                    ctx.set_option(key, v)
                assert e.value.status == B.EINVAL
        with pytest.raises(B.DpsgdError) as e:
            ctx.set_option("no_such_option", 1)
        assert e.value.status == B.EINVAL
        ctx.set_option("fused_slab", 1)


def test_step_falls_back_on_other_topologies_and_fp32():
    step_case(shrink(CONFIG3_TORUS, widths=(1024, 1000, 10), batch=32, n=24, torus_dims=(3, 8)),
              expect_fused=False)   # 1000 outputs: tiles do not divide
    step_case(shrink(CONFIGS[2], widths=(1024, 1024, 10), batch=32, n=8, topology="ring_chord"),
              options=(("fused_slab", 0),), expect_fused=False)   # switched off: the two calls
    step_case(shrink(CONFIGS[2], widths=(1024, 1024, 10), batch=32, n=66, topology="ring_chord"),
              expect_fused=False)   # more workers than 128 KB of LDS hold tiles for
    step_case(shrink(CONFIGS[1], widths=(300, 10), batch=16, n=6), bf16=False)
    step_case(shrink(CONFIGS[0], widths=(64,), batch=32, n=8), bf16=False, spread=1.0)


def test_step_with_odd_row_stride():
    """Row stride d + 1: rows are only 4-byte aligned.  The ring kernel still fuses (4-byte accesses); the torus
    kernel needs 8-byte aligned rows and hands over to the two calls."""
    for cfg in (shrink(CONFIGS[2], widths=(1024, 1024, 10), batch=32, n=5),
                shrink(CONFIG3_TORUS, widths=(1024, 1024, 10), batch=32, n=12, torus_dims=(3, 4))):
        step_case(cfg, ld=synth.model_dim(cfg.model_kind, cfg.widths) + 1)


@pytest.mark.parametrize("topology", ["ring", "torus"])
def test_step_config3_full_size_one_worker(topology):
    """The launch shape bench.py times.  The oracle forms one worker's next iterate from its own gradient and the
    rows of its neighbours (ring: worker 7 and workers 6, 8; 8 x 8 torus: worker 27 = (3, 3) and workers 19, 26,
    28, 35); the two-call sequence on the GPU checks every element."""
    cfg = CONFIGS[3] if topology == "ring" else CONFIG3_TORUS
    me, nbrs = (7, (6, 8)) if topology == "ring" else (27, (19, 26, 28, 35))
    d = synth.model_dim(cfg.model_kind, cfg.widths)
    ld = B.recommended_ld(d, topo_for(cfg))     # as bench.py lays X out
    x0 = synth.make_x0(cfg)
    rng = synth.rng(cfg.index, 95)
    Xa = torch.zeros(cfg.n, ld, device="cuda")
    Xa[:, :d] = torch.from_numpy(x0).cuda()
    rows = {}
    for i in (me,) + nbrs:
        xi = x0 + np.float32(0.3) * np.maximum(np.abs(x0), np.float32(0.02)) * rng.standard_normal(d, dtype=np.float32)
        rows[i] = xi
        Xa[i, :d] = torch.from_numpy(xi).cuda()
    Xb = Xa.clone()
    inp, tgt = synth.make_batch(cfg, 0)
    inp_d, tgt_d = bf16_dev(inp), torch.from_numpy(tgt).cuda()
    G = torch.zeros_like(Xa)
    model = B.Model(cfg.model_kind, cfg.widths, compute_bf16=True)
    ca, cb = torch.zeros(1, device="cuda"), torch.zeros(1, device="cuda")
    with B.Dpsgd(cfg.n, d, topo_for(cfg), cfg.gamma, ld=ld) as ctx:
        ctx.step(model, Xa, inp_d, tgt_d, cfg.batch, G, None, ca, input_is_bf16=True)
        ctx.grad(model, Xb, inp_d, tgt_d, cfg.batch, G, None, input_is_bf16=True)
        ctx.mix_step(Xb, G, Xb, cb)
        torch.cuda.synchronize()
    diff = float(torch.linalg.vector_norm((Xa - Xb)[:, :d]) / torch.linalg.vector_norm(Xb[:, :d]))
    print(f"  fused vs two-call over all {cfg.n} x {d} elements: {diff:.3e}; consensus {float(ca):.6g} / {float(cb):.6g}",
          flush=True)
    assert diff < 1e-5
    assert float(ca) == pytest.approx(float(cb), rel=1e-4)
    with ThreadPoolExecutor(max_workers=2) as pool:   # both rounding modes of the oracle side by side
        jobs = [pool.submit(oracle.loss_grad, cfg.model_kind, cfg.widths, rows[me], inp[me], tgt[me], bf16_operands=mode)
                for mode in (True, False)]
        (_, gme), (_, gplain) = [job.result() for job in jobs]
    w = np.float64(np.float32(1.0 / (1 + len(nbrs))))
    want = w * sum(rows[i].astype(np.float64) for i in (me,) + nbrs) - np.float64(np.float32(cfg.gamma)) * gme
    got = Xa[me, :d].cpu().numpy().astype(np.float64)
    e, m = check_close(got - rows[me], want - rows[me], TIGHT, f"worker {me} update vs oracle", flips=True)
    print(f"  worker {me} update vs oracle: {e:.3e} (max element {m:.3e} rms)", flush=True)
    # the un-rounded fp64 oracle binds the iterate itself at the bar of the bf16 workloads
    want_plain = w * sum(rows[i].astype(np.float64) for i in (me,) + nbrs) - np.float64(np.float32(cfg.gamma)) * gplain
    check_close(got, want_plain, TOL, f"worker {me} X_next vs plain oracle")
    # every element of the fused result against the two-call one, not only the norm
    worst = float((Xa - Xb)[:, :d].abs().max() / Xb[:, :d].pow(2).mean().sqrt())
    print(f"  largest element difference fused vs two-call: {worst:.3e} rms", flush=True)
    assert worst < 16 * 1e-5


def test_step_short_trajectory_with_gamma_schedule():
    """Ten iterations of dpsgd_step on its own trajectory, fresh minibatches, gamma lowered half way
    (dpsgd_set_gamma): strict single-step gate from the oracle's X_k at every iteration, loose gate on the
    free-running iterates, and the node-average recursion of the proof of Theorem 1 on the device data."""
    cfg = shrink(CONFIGS[2], widths=(1024, 1024, 10), batch=32, n=6, iters=10)
    d = synth.model_dim(cfg.model_kind, cfg.widths)
    ld = synth.padded_stride(d)
    topo_o = oracle_topo_for(cfg)
    model = B.Model(cfg.model_kind, cfg.widths, compute_bf16=True)
    Xo = synth.make_replicas(cfg).astype(np.float64)
    Xfree = to_dev(Xo, ld)
    G = torch.full_like(Xfree, 777.0)
    loss = torch.zeros(cfg.n, device="cuda")
    with B.Dpsgd(cfg.n, d, topo_for(cfg), cfg.gamma, ld=ld) as ctx:
        for k in range(cfg.iters):
            gamma = cfg.gamma if k < 5 else cfg.gamma / 10
            ctx.set_gamma(gamma)
            inp, tgt = synth.make_batch(cfg, k)
            inp_d, tgt_d = bf16_dev(inp), torch.from_numpy(tgt).cuda()
            Xn, Gref, _ = oracle.iteration(cfg.model_kind, cfg.widths, topo_o, np.float32(gamma), Xo, inp, tgt,
                                           bf16_operands=True)
            # single step from the oracle's X_k (rounded to fp32, as the device holds it)
            Xs = to_dev(Xo, ld)
            ctx.step(model, Xs, inp_d, tgt_d, cfg.batch, G, loss, None, input_is_bf16=True)
            # free-running
            before = from_dev(Xfree, d)
            ctx.step(model, Xfree, inp_d, tgt_d, cfg.batch, G, loss, None, input_is_bf16=True)
            torch.cuda.synchronize()
            e1, _ = check_close(from_dev(Xs, d) - Xo, Xn - Xo, TIGHT, f"k={k} single-step update", flips=True)
            after = from_dev(Xfree, d)
            ef, _ = check_close(after, Xn, TOL, f"k={k} free-running X")
            print(f"  k={k} gamma={gamma:g}: single-step update {e1:.3e}, free-running X {ef:.3e}", flush=True)
            assert e1 < TIGHT
            assert ef < TOL
            # the step moved the node average by -gamma * (mean gradient): |mean(after) - mean(before)| is O(gamma)
            drift = np.abs(after.mean(0) - before.mean(0)).max()
            assert drift < 50 * gamma
            Xo = Xn


def test_two_contexts_on_two_streams_do_not_share_state():
    """Two contexts (different topologies, own workspaces) enqueue interleaved on two streams; each result equals
    the one the same context gives alone."""
    cfg_a = shrink(CONFIGS[2], widths=(1024, 1024, 10), batch=32, n=6)
    cfg_b = shrink(CONFIG3_TORUS, widths=(1024, 1024, 10), batch=64, n=12, torus_dims=(3, 4))
    results = {}
    for interleaved in (False, True):
        streams = [torch.cuda.Stream(), torch.cuda.Stream()]
        state = []
        for cfg, st in zip((cfg_a, cfg_b), streams):
            d = synth.model_dim(cfg.model_kind, cfg.widths)
            ld = synth.padded_stride(d)
            inp, tgt = synth.make_batch(cfg, 0)
            with torch.cuda.stream(st):
                X = to_dev(synth.make_replicas(cfg), ld)
                G = torch.zeros_like(X)
                cons = torch.zeros(1, device="cuda")
                inp_d, tgt_d = bf16_dev(inp), torch.from_numpy(tgt).cuda()
                ctx = B.Dpsgd(cfg.n, d, topo_for(cfg), cfg.gamma, ld=ld, stream=st)
            state.append((cfg, st, X, G, cons, inp_d, tgt_d, ctx, d))
        torch.cuda.synchronize()
        model = B.Model(cfg_a.model_kind, cfg_a.widths, compute_bf16=True)
        order = [0, 1, 0, 1, 0, 1] if interleaved else [0, 0, 0, 1, 1, 1]
        for which in order:
            cfg, st, X, G, cons, inp_d, tgt_d, ctx, d = state[which]
            ctx.step(model, X, inp_d, tgt_d, cfg.batch, G, None, cons, input_is_bf16=True)
            if not interleaved:
                st.synchronize()
        torch.cuda.synchronize()
        results[interleaved] = [(from_dev(s[2], s[8]), float(s[4])) for s in state]
        for s in state:
            s[7].close()
    for (xa, ca), (xb, cb) in zip(results[False], results[True]):
        assert np.array_equal(xa, xb)
        assert ca == cb


@pytest.mark.parametrize("widths,batch,n", [
    ((1024, 1024, 10), 32, 5),        # 4 x 64 workgroups per layer, odd ring
    ((2048, 512, 4096, 10), 20, 3),   # ragged minibatch (padded to 32), the smallest ring, K = 2048 and 512
    ((1280, 2080, 10), 32, 4),        # 65 row groups of 32 and 5 column blocks
])
def test_row_layout_ring_kernel_agrees_with_the_tile_layout_one(widths, batch, n):
    """Minibatches of at most 32 rows take the [16 rows][1 KB] kernel where K % 256 == 0; "ring_rows" 0 forces the
    32 x 32 one.  The two sum the minibatch in a different order inside the MFMA (4 samples at a time against 16),
    so they agree to fp32 rounding of the gradient, not bit for bit."""
    cfg = shrink(CONFIGS[3], widths=widths, batch=batch, n=n, iters=2)
    d = synth.model_dim(cfg.model_kind, cfg.widths)
    ld = synth.padded_stride(d)
    model = B.Model(cfg.model_kind, cfg.widths, compute_bf16=True)
    X0 = to_dev(synth.make_replicas(cfg), ld)
    runs = []
    for rows in (0, 1):
        X = X0.clone()
        G = torch.zeros_like(X)
        loss = torch.zeros(cfg.iters, cfg.n, device="cuda")
        cons = torch.zeros(cfg.iters, device="cuda")
        with B.Dpsgd(cfg.n, d, topo_for(cfg), cfg.gamma, ld=ld) as ctx:
            ctx.set_option("ring_rows", rows)
            for k in range(cfg.iters):
                inp, tgt = synth.make_batch(cfg, k)
                ctx.step(model, X, bf16_dev(inp), torch.from_numpy(tgt).cuda(), cfg.batch, G, loss[k], cons[k:k + 1],
                         input_is_bf16=True)
            torch.cuda.synchronize()
        runs.append((X, loss, cons))
    (Xa, la, ca), (Xb, lb, cb) = runs
    print(f"rows vs tiles {widths} B={batch} n={n}: max |dX| {float((Xa - Xb).abs().max()):.3e}, "
          f"bit-identical {bool(torch.equal(Xa, Xb))}, consensus {ca.tolist()} {cb.tolist()}", flush=True)
    assert not torch.equal(Xa, X0)
    # one step moves an element by gamma * g; the two gradients differ by a few ulp of their own size
    step = float((Xa - X0).abs().max())
    assert float((Xa - Xb).abs().max()) <= 1e-5 * step + 1e-7
    assert torch.allclose(la, lb, rtol=1e-5, atol=1e-6)
    assert torch.allclose(ca, cb, rtol=1e-5, atol=0.0)
    assert bool(torch.all(Xb[:, d:] == X0[:, d:]))     # padding columns untouched


@pytest.mark.parametrize("widths,batch,n,shadow", [
    ((4096, 256, 10), 32, 3, 0),           # K = 4096: a wave's 512-byte pieces two rows apart (16 row groups)
    ((4096, 288, 10), 20, 4, 0),           # 18 row groups, ragged minibatch
    ((8192, 128, 10), 32, 3, 0),           # K = 8192: one row apart
    ((1024, 4096, 1024, 10), 32, 3, 1),    # hidden layer with K = 4096 and its bf16 copy, written by one step and read by the next
    ((3072, 512, 10), 32, 3, 0),           # K = 3072 (12 KB rows): a wave's 1 KB pieces eight rows apart, 16 rows of a block of 32 per workgroup
    ((1024, 1056, 2048, 10), 20, 4, 0),    # K = 1024 and K = 1056 (no map: not a multiple of 1024); 33 blocks of 32 rows
    ((2048, 512, 10), 32, 5, 0),           # K = 2048
])
def test_chunked_wave_map_of_the_row_kernel_changes_no_bit(widths, batch, n, shadow):
    """The [16 rows][1 KB] kernel: which wave owns which rows ("ring_chunks" 1, the default: pieces a multiple of 32 KB
    apart where the row length allows it - K = 4096 or 8192: 512-byte pieces; other multiples of 1024: 1 KB pieces
    eight rows apart; 0: four consecutive rows per wave) changes no sum: iterates, losses and consensus distances are
    identical bit for bit over three iterations, with and without the bf16 weight copy."""
    cfg = shrink(CONFIGS[3], widths=widths, batch=batch, n=n, iters=3)
    d = synth.model_dim(cfg.model_kind, cfg.widths)
    ld = synth.padded_stride(d)
    model = B.Model(cfg.model_kind, cfg.widths, compute_bf16=True)
    X0 = to_dev(synth.make_replicas(cfg), ld)
    runs = []
    for chunks in (1, 0):
        X = X0.clone()
        G = torch.zeros_like(X)
        loss = torch.zeros(cfg.iters, cfg.n, device="cuda")
        cons = torch.zeros(cfg.iters, device="cuda")
        print(f"ring_chunks={chunks} widths={widths} B={batch} n={n} shadow={shadow}", flush=True)
        with B.Dpsgd(cfg.n, d, topo_for(cfg), cfg.gamma, ld=ld) as ctx:
            ctx.set_option("bf16_shadow", shadow)
            ctx.set_option("ring_chunks", chunks)
            for k in range(cfg.iters):
                inp, tgt = synth.make_batch(cfg, k)
                ctx.step(model, X, bf16_dev(inp), torch.from_numpy(tgt).cuda(), cfg.batch, G, loss[k], cons[k:k + 1],
                         input_is_bf16=True)
            torch.cuda.synchronize()
        runs.append((X, loss, cons))
    (Xa, la, ca), (Xb, lb, cb) = runs
    assert not torch.equal(Xa, X0)
    assert torch.equal(Xa, Xb), f"max |dX| {float((Xa - Xb).abs().max()):.3e}"
    assert torch.equal(la, lb) and torch.equal(ca, cb)


@pytest.mark.parametrize("widths,batch,n", [
    ((3072, 1024, 10), 128, 4),       # configs[2]'s layer: 8 operand steps per worker, 40 KB of LDS per workgroup
    ((1024, 1024, 10), 64, 5),        # 4 steps, odd ring
    ((1280, 2080, 10), 90, 3),        # ragged minibatch padded to 96 (6 steps: two waves fetch two steps of dZ^T, two one)
    ((512, 1024, 10), 150, 3),        # padded to 160: 10 steps
])
def test_operands_through_lds_change_no_bit(widths, batch, n):
    """Minibatches of more than 32 rows on the ring: the fused kernel whose operands travel from L2 into LDS
    asynchronously ("fused_lds" 1, the default) and the one that fetches them into registers ("fused_lds" 0) issue the
    same matrix instructions on the same operands in the same order: iterates, losses and consensus distances are
    identical bit for bit over three iterations."""
    cfg = shrink(CONFIGS[2], widths=widths, batch=batch, n=n, iters=3)
    d = synth.model_dim(cfg.model_kind, cfg.widths)
    ld = synth.padded_stride(d)
    model = B.Model(cfg.model_kind, cfg.widths, compute_bf16=True)
    X0 = to_dev(synth.make_replicas(cfg), ld)
    runs = []
    for lds in (1, 0):
        X = X0.clone()
        G = torch.zeros_like(X)
        loss = torch.zeros(cfg.iters, cfg.n, device="cuda")
        cons = torch.zeros(cfg.iters, device="cuda")
        print(f"fused_lds={lds} widths={widths} B={batch} n={n}", flush=True)
        with B.Dpsgd(cfg.n, d, topo_for(cfg), cfg.gamma, ld=ld) as ctx:
            ctx.set_option("fused_lds", lds)
            for k in range(cfg.iters):
                inp, tgt = synth.make_batch(cfg, k)
                ctx.step(model, X, bf16_dev(inp), torch.from_numpy(tgt).cuda(), cfg.batch, G, loss[k], cons[k:k + 1],
                         input_is_bf16=True)
            torch.cuda.synchronize()
        runs.append((X, loss, cons))
    (Xa, la, ca), (Xb, lb, cb) = runs
    assert not torch.equal(Xa, X0)
    assert torch.equal(Xa, Xb), f"max |dX| {float((Xa - Xb).abs().max()):.3e}"
    assert torch.equal(la, lb) and torch.equal(ca, cb)


@pytest.mark.parametrize("widths,batch", [
    ((1024, 1024, 1024, 10), 32),     # one hidden layer with a copy, read by the forward and the data gradient
    ((1024, 1024, 1152, 1024, 10), 32),   # two of them, 36 and 32 output tiles
    ((1024, 1024, 1120, 10), 32),     # 35 output tiles: written, but the readers want multiples of 64 and use fp32
    ((1024, 1024, 1024, 10), 64),     # minibatch 64: the forward of that tiling reads fp32, the data gradient the copy
])
@pytest.mark.parametrize("ring_rows", [1, 0])
def test_bf16_shadow_option_on_other_shapes(widths, batch, ring_rows):
    cfg = shrink(CONFIGS[3], widths=widths, batch=batch, n=4, iters=3)
    d = synth.model_dim(cfg.model_kind, cfg.widths)
    ld = synth.padded_stride(d)
    model = B.Model(cfg.model_kind, cfg.widths, compute_bf16=True)
    X0 = to_dev(synth.make_replicas(cfg), ld)
    runs = []
    for shadow in (0, 1):
        X = X0.clone()
        G = torch.zeros_like(X)
        loss = torch.zeros(cfg.iters, cfg.n, device="cuda")
        with B.Dpsgd(cfg.n, d, topo_for(cfg), cfg.gamma, ld=ld) as ctx:
            ctx.set_option("bf16_shadow", shadow)
            ctx.set_option("ring_rows", ring_rows)     # which fused kernel writes the copy, hence its layout
            for k in range(cfg.iters):
                inp, tgt = synth.make_batch(cfg, k)
                ctx.step(model, X, bf16_dev(inp), torch.from_numpy(tgt).cuda(), cfg.batch, G, loss[k], None,
                         input_is_bf16=True)
            torch.cuda.synchronize()
        runs.append((X, loss))
    assert torch.equal(runs[0][0], runs[1][0])
    assert torch.equal(runs[0][1], runs[1][1])


@pytest.mark.parametrize("ring_rows", [1, 0])
def test_bf16_shadow_option_gives_the_same_trajectory_and_is_dropped_when_x_changes(ring_rows):
    """With "bf16_shadow" the fused kernel leaves the bf16 rounding of the new hidden-layer weights for the next
    call's forward and data gradient: the same values, so every iterate must be bit-identical to the run without
    the option.  A dpsgd_mix_step in between (X changes behind the copy's back), a second matrix X and a smaller
    minibatch must all be handled."""
    cfg = shrink(CONFIGS[3], widths=(1024, 1024, 1024, 10), batch=32, n=5, iters=6)
    d = synth.model_dim(cfg.model_kind, cfg.widths)
    ld = synth.padded_stride(d)
    model = B.Model(cfg.model_kind, cfg.widths, compute_bf16=True)
    X0 = to_dev(synth.make_replicas(cfg), ld)
    batches = []
    for k in range(cfg.iters):
        inp, tgt = synth.make_batch(cfg, k)
        batches.append((bf16_dev(inp), torch.from_numpy(tgt).cuda()))

    def run(shadow):
        Xa, Xb = X0.clone(), (X0 * 1.01).contiguous()
        G = torch.zeros_like(Xa)
        loss = torch.zeros(cfg.iters + 4, cfg.n, device="cuda")
        cons = torch.zeros(cfg.iters + 4, device="cuda")
        snaps = []
        with B.Dpsgd(cfg.n, d, topo_for(cfg), cfg.gamma, ld=ld) as ctx:
            ctx.set_option("bf16_shadow", 1 if shadow else 0)
            ctx.set_option("ring_rows", ring_rows)     # which fused kernel writes the copy, hence its layout
            for k, (inp_d, tgt_d) in enumerate(batches):
                ctx.step(model, Xa, inp_d, tgt_d, cfg.batch, G, loss[k], cons[k:k + 1], input_is_bf16=True)
                snaps.append(Xa.clone())
                if k == 2:      # X changes through another entry point: the copy must not be used afterwards
                    G.copy_(Xa).mul_(1e-2)
                    ctx.mix_step(Xa, G, Xa, None)
                if k == 3:      # another matrix in between, then back
                    ctx.step(model, Xb, inp_d, tgt_d, cfg.batch, G, loss[cfg.iters], cons[cfg.iters:cfg.iters + 1],
                             input_is_bf16=True)
                    snaps.append(Xb.clone())
                if k == 4:      # the caller edits X itself and says so by switching the option off and on
                    Xa[:, :100] += 1e-3
                    ctx.set_option("bf16_shadow", 1 if shadow else 0)
            # a smaller minibatch (other workspace layout) on the same X
            inp_d, tgt_d = batches[0]
            half = cfg.batch // 2
            inp_h = inp_d.view(cfg.n, cfg.batch, -1)[:, :half].contiguous()
            tgt_h = tgt_d.view(cfg.n, cfg.batch)[:, :half].contiguous()
            ctx.step(model, Xa, inp_h, tgt_h, half, G, loss[cfg.iters + 1], cons[cfg.iters + 1:cfg.iters + 2], input_is_bf16=True)
            snaps.append(Xa.clone())
            # a larger one: other kernels read the copy the call above left (its layout goes by the writer), and the
            # copy they leave is read by the minibatch of 32 again
            inp_2 = inp_d.view(cfg.n, cfg.batch, -1).repeat(1, 2, 1).contiguous()
            tgt_2 = tgt_d.view(cfg.n, cfg.batch).repeat(1, 2).contiguous()
            ctx.step(model, Xa, inp_2, tgt_2, 2 * cfg.batch, G, loss[cfg.iters + 2], cons[cfg.iters + 2:cfg.iters + 3], input_is_bf16=True)
            snaps.append(Xa.clone())
            ctx.step(model, Xa, inp_d, tgt_d, cfg.batch, G, loss[cfg.iters + 3], cons[cfg.iters + 3:cfg.iters + 4], input_is_bf16=True)
            snaps.append(Xa.clone())
            torch.cuda.synchronize()
        return snaps, loss.clone(), cons.clone()

    plain, loss_p, cons_p = run(False)
    shadow, loss_s, cons_s = run(True)
    assert len(plain) == len(shadow)
    for k, (a, b) in enumerate(zip(plain, shadow)):
        assert torch.equal(a, b), f"snapshot {k} differs"
    assert torch.equal(loss_p, loss_s)
    assert torch.equal(cons_p, cons_s)


def test_bf16_shadow_is_dropped_by_a_step_that_does_not_fuse():
    """dpsgd_step calls that run the two calls internally (fp32 arithmetic; the generic CSR kernel forced by an
    option) change X behind the bf16 copy's back: the next fused step must read the fp32 weights again.  Every iterate
    of the run with the copy equals the run without it bit for bit, and the last step matches the oracle."""
    cfg = shrink(CONFIGS[3], widths=(1024, 1024, 1024, 10), batch=32, n=5, iters=5)
    d = synth.model_dim(cfg.model_kind, cfg.widths)
    ld = synth.padded_stride(d)
    bf16_model = B.Model(cfg.model_kind, cfg.widths, compute_bf16=True)
    fp32_model = B.Model(cfg.model_kind, cfg.widths, compute_bf16=False)
    X0 = to_dev(synth.make_replicas(cfg), ld)
    batches = [synth.make_batch(cfg, k) for k in range(cfg.iters)]

    def run(shadow):
        X = X0.clone()
        G = torch.zeros_like(X)
        loss = torch.zeros(cfg.n, device="cuda")
        snaps = []
        with B.Dpsgd(cfg.n, d, topo_for(cfg), cfg.gamma, ld=ld) as ctx:
            ctx.set_option("bf16_shadow", shadow)
            for k, (inp, tgt) in enumerate(batches):
                tgt_d = torch.from_numpy(tgt).cuda()
                if k == 1:       # fp32 arithmetic: no fused kernel, X is updated by the plain mix
                    ctx.step(fp32_model, X, torch.from_numpy(inp).cuda(), tgt_d, cfg.batch, G, loss, None)
                else:
                    if k == 3:   # the generic CSR kernel for the ring: again no fused kernel
                        ctx.set_option("mix_force_csr", 1)
                    if k == 4:
                        ctx.set_option("mix_force_csr", 0)
                    ctx.step(bf16_model, X, bf16_dev(inp), tgt_d, cfg.batch, G, loss, None, input_is_bf16=True)
                snaps.append(X.clone())
            torch.cuda.synchronize()
        return snaps

    plain, shadow = run(0), run(1)
    for k, (a, b) in enumerate(zip(plain, shadow)):
        assert torch.equal(a, b), f"iterate {k + 1} differs with the bf16 copy on"
    # and the iterate after the fp32 step, stepped once more by the fused kernels, is what the oracle gets from it
    inp, tgt = batches[2]
    before = from_dev(shadow[1], d)
    want, _, _ = oracle.iteration(cfg.model_kind, cfg.widths, oracle_topo_for(cfg), np.float32(cfg.gamma), before, inp, tgt,
                                  bf16_operands=True)
    check_close(from_dev(shadow[2], d) - before, want - before, TIGHT, "fused step after an fp32 step", flips=True)
