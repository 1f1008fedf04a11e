"""GPU parity of dpsgd_mix_step / dpsgd_mix_step_swapped / dpsgd_mean against the CPU oracle
(Algorithm 1 steps 4, 5, 7; consensus distance of eq. 10/13).  fp32: 1e-5 relative Frobenius."""
import numpy as np
import pytest
import torch

import oracle
from paper_1705_09056_amd import binding as B

from conftest import check_close, rel_err
from gpu_util import from_dev, to_dev

pytestmark = pytest.mark.gpu
TOL = 1e-5


def random_state(n, d, seed, spread=0.05):
    rng = np.random.default_rng(seed)
    base = rng.standard_normal(d).astype(np.float32)
    X = (base + spread * rng.standard_normal((n, d))).astype(np.float32)
    G = rng.standard_normal((n, d)).astype(np.float32)
    return X, G


def random_symmetric_ds(n, rng, terms=3):
    """Symmetric doubly stochastic W with fp32-exact dyadic weights: mean of (P + P^T)/2 over 4 perms."""
    W = np.zeros((n, n))
    for _ in range(4):
        P = np.eye(n)[rng.permutation(n)]
        W += (P + P.T) / 8.0
    rowptr, col, val = [0], [], []
    for i in range(n):
        for j in np.nonzero(W[i])[0]:
            col.append(int(j)); val.append(W[i, j])
        rowptr.append(len(col))
    return np.array(rowptr, np.int32), np.array(col, np.int32), np.array(val, np.float32)


def run_mix(n, d, ld, topo_b, topo_o, seed, inplace, cons, swapped=False, options=(), gamma=0.05):
    X, G = random_state(n, d, seed)
    ref = oracle.mix_step(topo_o, X, G, np.float32(gamma), swapped=swapped)
    Xd, Gd = to_dev(X, ld), to_dev(G, ld)
    out = Xd if inplace else torch.full_like(Xd, 777.0)
    cd = torch.zeros(1, device="cuda") if cons else None
    with B.Dpsgd(n, d, topo_b, gamma, ld=ld) as ctx:
        for k, v in options:
            ctx.set_option(k, v)
        print(f"mix n={n} d={d} ld={ld} inplace={inplace} cons={cons} swapped={swapped} opts={options}", flush=True)
        ctx.mix_step(Xd, Gd, out, cd, swapped=swapped)
        torch.cuda.synchronize()
    got = from_dev(out, d)
    check_close(got, ref, TOL, "X_next")
    if not inplace:
        assert np.array_equal(from_dev(Xd, d), X.astype(np.float64))     # input untouched
    assert np.array_equal(from_dev(Gd, d), G.astype(np.float64))
    if cons:
        want = oracle.consensus(ref)
        assert float(cd.item()) == pytest.approx(want, rel=1e-4)


@pytest.mark.parametrize("n", [3, 8, 16, 33, 112])
@pytest.mark.parametrize("d,ld", [(1, 1), (5, 5), (64, 64), (1003, 1003), (1003, 1024), (30730, 30784), (70001, 70002)])
@pytest.mark.parametrize("inplace", [False, True])
def test_ring(n, d, ld, inplace):
    run_mix(n, d, ld, B.Topology.ring(), oracle.ring(n).with_fp32_values(), n * 1000 + d, inplace, cons=True)


@pytest.mark.parametrize("bands", [1, 2, 4, 8, 16])
@pytest.mark.parametrize("vec", [1, 2, 4])
def test_ring_launch_shapes(bands, vec):
    n, d, ld = 37, 5000, 5056
    run_mix(n, d, ld, B.Topology.ring(), oracle.ring(n).with_fp32_values(), 99, True, True,
            options=(("mix_bands", bands), ("mix_vec", vec)))


@pytest.mark.parametrize("n", [1, 2])
def test_degenerate_rings(n):
    run_mix(n, 300, 320, B.Topology.ring(), oracle.ring(n).with_fp32_values(), 5, True, True)


@pytest.mark.parametrize("dims", [(8, 8), (3, 5), (2, 4), (4, 16), (7, 16)])
@pytest.mark.parametrize("inplace", [False, True])
def test_torus(dims, inplace):
    n = dims[0] * dims[1]
    for d, ld in [(7, 7), (4100, 4160), (30730, 30784)]:
        run_mix(n, d, ld, B.Topology.torus(*dims), oracle.torus(*dims).with_fp32_values(), n + d, inplace, True)


@pytest.mark.parametrize("inplace", [False, True])
def test_wide_matrices_through_the_slab_kernel(inplace):
    """Wide matrices: the LDS-slab kernel deals whole super-blocks of columns to its workgroups as 512-byte chunks
    32 KB apart (two float4 per lane while 64 workers' rows fit 128 KB of LDS, one beyond that), the remaining columns
    consecutively, the last d % 4 one by one."""
    d, ld = 33 * 16384 + 1000 + 3, 33 * 16384 + 1024
    run_mix(12, d, ld, B.Topology.torus(3, 4), oracle.torus(3, 4).with_fp32_values(), 21, inplace, True)
    run_mix(8, d, ld, B.Topology.ring_chord(), oracle.ring_chord(8).with_fp32_values(), 22, inplace, True)
    run_mix(6, d, ld, B.Topology.ring(), oracle.ring(6).with_fp32_values(), 23, inplace, True, swapped=True)
    run_mix(72, d, ld, B.Topology.torus(8, 9), oracle.torus(8, 9).with_fp32_values(), 24, inplace, True)   # one float4 per lane


@pytest.mark.parametrize("extra", [0, 3, 4 * 64 + 1])
def test_wide_ring_whose_columns_end_at_or_just_past_whole_super_blocks(extra):
    """64 super-blocks of 131 072 columns exactly, plus nothing, plus three columns (no whole float4 left: the fat-lane
    kernel, then the tail alone), plus one column group and one column (the tail rides in the remainder's launch)."""
    d = 64 * 131072 + extra
    ld = (d + 3) // 4 * 4
    run_mix(3, d, ld, B.Topology.ring(), oracle.ring(3).with_fp32_values(), 40 + extra, True, True)


@pytest.mark.parametrize("dims", [(3, 3), (8, 8), (5, 4), (3, 8), (9, 7)])
@pytest.mark.parametrize("inplace", [False, True])
def test_wide_torus(dims, inplace):
    """Tori of several shapes with more than a million columns (chunked column ownership of the slab kernel, its
    consecutive remainder and the tail columns), with and without the consensus distance."""
    n = dims[0] * dims[1]
    d = 16 * 65536 + 16384 + 1000 + 2
    run_mix(n, d, d + 2, B.Topology.torus(*dims), oracle.torus(*dims).with_fp32_values(), 30 + n, inplace, True)
    if dims == (5, 4):
        run_mix(n, d, d + 2, B.Topology.torus(*dims), oracle.torus(*dims).with_fp32_values(), 31 + n, inplace, False)


def test_ring_tag_through_the_csr_kernel_matches():
    run_mix(16, 9000, 9024, B.Topology.ring(), oracle.ring(16).with_fp32_values(), 3, True, True,
            options=(("mix_force_csr", 1),))


@pytest.mark.parametrize("n", [5, 40, 130, 300])
def test_complete_and_random_csr(n):
    rng = np.random.default_rng(n)
    run_mix(n, 2500, 2560, B.Topology.complete(), oracle.complete(n).with_fp32_values(), n, n <= 256, True)
    rowptr, col, val = random_symmetric_ds(n, rng)
    to = oracle.Topology(n, rowptr, col, val.astype(np.float64))
    assert to.check(1e-12) == 0
    run_mix(n, 2500, 2560, B.Topology.csr(rowptr, col, val), to, n + 1, n <= 256, True)


def hypercube_csr(k):
    """n = 2^k workers, neighbours differ in one bit; itself and its k neighbours at 1/(k+1)."""
    n = 1 << k
    rowptr, col, val = [0], [], []
    for i in range(n):
        for j in sorted([i] + [i ^ (1 << b) for b in range(k)]):
            col.append(j); val.append(1.0 / (k + 1))
        rowptr.append(len(col))
    return np.array(rowptr, np.int32), np.array(col, np.int32), np.array(val, np.float32)


@pytest.mark.parametrize("n", [4, 16, 112])
@pytest.mark.parametrize("inplace", [False, True])
def test_ring_with_far_link(n, inplace):
    """The 16-machine topology of the supplement's scalability experiment, through the CSR slab kernel."""
    run_mix(n, 5003, 5056, B.Topology.ring_chord(), oracle.ring_chord(n).with_fp32_values(), 40 + n, inplace, True)


@pytest.mark.parametrize("k", [3, 4, 6])
def test_hypercube_csr(k):
    rowptr, col, val = hypercube_csr(k)
    to = oracle.Topology(1 << k, rowptr, col, val.astype(np.float64))
    assert to.check(1e-6) == 0
    run_mix(1 << k, 4100, 4160, B.Topology.csr(rowptr, col, val), to, 50 + k, True, True)
    run_mix(1 << k, 4100, 4160, B.Topology.csr(rowptr, col, val), to, 60 + k, False, True, swapped=True)


def test_inplace_without_slab_is_refused():
    n, d = 300, 100
    X, G = random_state(n, d, 1)
    Xd, Gd = to_dev(X), to_dev(G)
    with B.Dpsgd(n, d, B.Topology.complete(), 0.1) as ctx:
        with pytest.raises(B.DpsgdError) as e:
            ctx.mix_step(Xd, Gd, Xd)
        assert e.value.status == B.EUNSUPPORTED


@pytest.mark.parametrize("topo", ["ring", "torus"])
def test_swapped_order(topo):
    if topo == "ring":
        tb, to, n = B.Topology.ring(), oracle.ring(12).with_fp32_values(), 12
    else:
        tb, to, n = B.Topology.torus(3, 4), oracle.torus(3, 4).with_fp32_values(), 12
    run_mix(n, 3000, 3008, tb, to, 17, True, True, swapped=True)
    run_mix(n, 3001, 3001, tb, to, 18, False, False, swapped=True)


def test_exported_topology_is_bit_exact():
    with B.Dpsgd(64, 10, B.Topology.torus(8, 8), 0.1) as ctx:
        rowptr, col, val = ctx.topology_export()
    t = oracle.torus(8, 8)
    assert np.array_equal(rowptr, t.rowptr) and np.array_equal(col, t.col)
    assert np.all(val == np.float32(0.2))


@pytest.mark.parametrize("n,d,ld", [(1, 10, 10), (8, 64, 64), (16, 30730, 30784), (112, 5001, 5001), (64, 100000, 100032)])
def test_mean(n, d, ld):
    X, _ = random_state(n, d, n + d, spread=1.0)
    Xd = to_dev(X, ld)
    out = torch.zeros(d, device="cuda")
    with B.Dpsgd(n, d, B.Topology.ring(), 0.1, ld=ld) as ctx:
        ctx.mean(Xd, out)
        torch.cuda.synchronize()
    check_close(out.cpu().numpy(), oracle.mean(X), TOL, "xbar")


@pytest.mark.parametrize("n", [1, 2, 5])
def test_mean_of_a_wide_matrix_takes_the_fat_lane_kernel(n):
    """64 whole super-blocks of 65 536 columns and a ragged rest: the fat-lane mean kernel, the ordinary one on the
    rest, against the oracle; and bit for bit against the ordinary kernel alone ("mix_narrow")."""
    d = 64 * 65536 + 3 * 256 + 3
    ld = d + 5 - (d + 5) % 4 + 4
    X, _ = random_state(n, d, 7 + n, spread=1.0)
    Xd = to_dev(X, ld)
    out, ref = torch.zeros(d, device="cuda"), torch.zeros(d, device="cuda")
    with B.Dpsgd(n, d, B.Topology.ring(), 0.1, ld=ld) as ctx:
        ctx.mean(Xd, out)
        ctx.set_option("mix_narrow", 1)
        ctx.mean(Xd, ref)
        torch.cuda.synchronize()
    check_close(out.cpu().numpy(), oracle.mean(X), TOL, "xbar")
    assert torch.equal(out, ref)


def test_multi_step_invariants_on_device():
    """Node-average recursion (proof of Theorem 1) and consensus decay hold for the GPU iterates."""
    n, d, ld, gamma = 16, 4099, 4160, 0.1
    X, _ = random_state(n, d, 42, spread=1.0)
    Xd = to_dev(X, ld)
    Z = to_dev(np.zeros((n, d), np.float32), ld)
    cd = torch.zeros(1, device="cuda")
    mean0 = X.astype(np.float64).mean(0)
    prev = oracle.consensus(X)
    with B.Dpsgd(n, d, B.Topology.ring(), gamma, ld=ld) as ctx:
        for k in range(20):
            ctx.mix_step(Xd, Z, Xd, cd)
            cur = float(cd.item())
            assert cur <= prev * (1 + 1e-5)
            prev = cur
    got = from_dev(Xd, d)
    assert rel_err(got.mean(0), mean0) < 1e-5
    lam2 = (1 + 2 * np.cos(2 * np.pi / n)) / 3
    assert prev <= oracle.consensus(X) * lam2 ** (2 * 20) * (1 + 1e-3)


def _full_size_mix(n, d, topo_b, topo_o, gamma=0.1):
    """The launch shape bench.py times (in place, consensus on); the oracle checks sampled columns, and the
    consensus distance chunk by chunk."""
    ld = (d + 63) // 64 * 64
    gen = torch.Generator(device="cuda")
    gen.manual_seed(170509056)
    base = torch.randn(ld, device="cuda", generator=gen)
    Xd = base + 0.05 * torch.randn(n, ld, device="cuda", generator=gen)
    Gd = torch.randn(n, ld, device="cuda", generator=gen)
    rng = np.random.default_rng(3)
    cols = np.unique(np.concatenate([rng.integers(0, d, 4000), np.arange(0, 300), np.arange(d - 300, d)]))
    cols_d = torch.from_numpy(cols).cuda()
    Xs = Xd[:, cols_d].cpu().numpy()
    Gs = Gd[:, cols_d].cpu().numpy()
    ref = oracle.mix_step(topo_o, Xs, Gs, np.float32(gamma))
    cons = torch.zeros(1, device="cuda")
    print(f"full-size mix n={n} d={d}", flush=True)
    with B.Dpsgd(n, d, topo_b, gamma, ld=ld) as ctx:
        ctx.mix_step(Xd, Gd, Xd, cons)
        torch.cuda.synchronize()
    got = Xd[:, cols_d].cpu().numpy()
    check_close(got, ref, TOL, "sampled columns of X_next")
    # consensus of the whole output, accumulated by the oracle over column chunks
    total = 0.0
    step = 2_000_000
    for c0 in range(0, d, step):
        chunk = Xd[:, c0:min(d, c0 + step)].cpu().numpy()
        total += oracle.consensus(chunk)
    assert float(cons.item()) == pytest.approx(total, rel=1e-5)


def test_full_size_config3_ring():
    _full_size_mix(64, 29409290, B.Topology.ring(), oracle.ring(64).with_fp32_values())


def test_full_size_config3_torus():
    _full_size_mix(64, 29409290, B.Topology.torus(8, 8), oracle.torus(8, 8).with_fp32_values())


def test_full_size_config4_ring():
    _full_size_mix(112, 268365, B.Topology.ring(), oracle.ring(112).with_fp32_values())


@pytest.mark.parametrize("n", [5, 8])
@pytest.mark.parametrize("with_consensus", [True, False])
def test_fat_lane_ring_kernel_matches_the_narrow_one_bitwise(n, with_consensus):
    """Wide matrices (at least 8192 groups of 2048 columns) take the kernel with eight float4 per lane; same
    arithmetic in the same order as the one-float4 kernel, so the outputs must be identical.  d leaves a remainder of
    1341 columns for the narrow kernel and the scalar tail; n = 5 leaves a row for the remainder loop of the variant
    with two rows in flight."""
    d = 8192 * 2048 + 1341
    ld = (d + 63) // 64 * 64
    gen = torch.Generator(device="cuda")
    gen.manual_seed(170509056 + n)
    Xd = torch.randn(ld, device="cuda", generator=gen) + 0.05 * torch.randn(n, ld, device="cuda", generator=gen)
    Gd = torch.randn(n, ld, device="cuda", generator=gen)
    outs, conss = [], []
    for narrow in (0, 1):
        out = torch.full_like(Xd, 777.0)
        cons = torch.zeros(1, device="cuda") if with_consensus else None
        with B.Dpsgd(n, d, B.Topology.ring(), 0.1, ld=ld) as ctx:
            ctx.set_option("mix_narrow", narrow)
            ctx.mix_step(Xd, Gd, out, cons)
            torch.cuda.synchronize()
        outs.append(out)
        conss.append(None if cons is None else float(cons.item()))
    assert torch.equal(outs[0], outs[1])
    assert bool(torch.all(outs[0][:, d:] == 777.0))
    if with_consensus:
        assert conss[0] == pytest.approx(conss[1], rel=1e-5)
    # in place gives the same as out of place
    Xi = Xd.clone()
    with B.Dpsgd(n, d, B.Topology.ring(), 0.1, ld=ld) as ctx:
        ctx.mix_step(Xi, Gd, Xi, None)
        torch.cuda.synchronize()
    assert torch.equal(Xi[:, :d], outs[0][:, :d])


# ------------------------------------------------------------------ momentum variant (dpsgd_mix_step_momentum)
def run_momentum(n, d, ld, topo_b, topo_o, seed, inplace, mu=0.9, gamma=0.05, steps=3, options=()):
    rng = np.random.default_rng(seed)
    X, _ = random_state(n, d, seed)
    V = np.zeros((n, d), np.float32)
    Xo, Vo = X.astype(np.float64), V.astype(np.float64)
    Xd, Vd = to_dev(X, ld), to_dev(V, ld)
    cd = torch.zeros(1, device="cuda")
    print(f"momentum n={n} d={d} ld={ld} inplace={inplace} mu={mu}", flush=True)
    with B.Dpsgd(n, d, topo_b, gamma, ld=ld) as ctx:
        for k, v in options:
            ctx.set_option(k, v)
        for k in range(steps):
            G = rng.standard_normal((n, d)).astype(np.float32)
            Xo, Vo = oracle.mix_step_momentum(topo_o, Xo, G, Vo, np.float32(gamma), np.float32(mu))
            Gd = to_dev(G, ld)
            out = Xd if inplace else torch.full_like(Xd, 777.0)
            ctx.mix_step_momentum(Xd, Gd, Vd, mu, out, cd)
            torch.cuda.synchronize()
            Xd = out
            check_close(from_dev(Xd, d), Xo, TOL, "X_next")
            check_close(from_dev(Vd, d), Vo, TOL, "V_next")
            assert np.array_equal(from_dev(Gd, d), G.astype(np.float64))
            assert float(cd.item()) == pytest.approx(oracle.consensus(Xo), rel=1e-4)


@pytest.mark.parametrize("n,d,ld", [(8, 1003, 1024), (16, 30730, 30784), (5, 70001, 70002), (33, 5, 5)])
@pytest.mark.parametrize("inplace", [False, True])
def test_momentum_ring(n, d, ld, inplace):
    run_momentum(n, d, ld, B.Topology.ring(), oracle.ring(n).with_fp32_values(), 70 + n, inplace)


def test_momentum_torus_ring_chord_and_gather():
    run_momentum(12, 3001, 3008, B.Topology.torus(3, 4), oracle.torus(3, 4).with_fp32_values(), 81, True)
    run_momentum(16, 3001, 3001, B.Topology.ring_chord(), oracle.ring_chord(16).with_fp32_values(), 82, True, mu=0.5)
    run_momentum(300, 700, 704, B.Topology.complete(), oracle.complete(300).with_fp32_values(), 83, False)
    # wide: the slab kernel's chunked column ownership, with the velocity riding along
    run_momentum(12, 33 * 16384 + 77, 33 * 16384 + 128, B.Topology.torus(3, 4), oracle.torus(3, 4).with_fp32_values(), 84, True,
                 steps=2)


def test_momentum_on_a_wide_ring_takes_the_fat_lane_kernel():
    """64 super-blocks of 131072 columns and a remainder: the fat-lane ring kernel carries the velocity too."""
    d = 64 * 131072 + 2048 + 5
    run_momentum(3, d, d + 3, B.Topology.ring(), oracle.ring(3).with_fp32_values(), 85, True, steps=2)
    run_momentum(3, d, d + 59, B.Topology.ring(), oracle.ring(3).with_fp32_values(), 86, False, steps=1)


@pytest.mark.parametrize("n,d,ld", [(16, 9000, 9024), (3, 64 * 131072 + 300, 64 * 131072 + 512)])
def test_momentum_zero_equals_plain_step_bitwise(n, d, ld):
    X, G = random_state(n, d, 91)
    Xd, Gd = to_dev(X, ld), to_dev(G, ld)
    Vd = to_dev(np.ones((n, d), np.float32), ld)
    a, b = torch.full_like(Xd, 777.0), torch.full_like(Xd, 777.0)
    with B.Dpsgd(n, d, B.Topology.ring(), 0.05, ld=ld) as ctx:
        ctx.mix_step(Xd, Gd, a)
        ctx.mix_step_momentum(Xd, Gd, Vd, 0.0, b)
        torch.cuda.synchronize()
    assert torch.equal(a, b)
    assert np.array_equal(from_dev(Vd, d), G.astype(np.float64))


def test_momentum_rejects_bad_arguments():
    n, d = 8, 100
    X, G = random_state(n, d, 92)
    Xd, Gd, Vd = to_dev(X), to_dev(G), to_dev(np.zeros((n, d), np.float32))
    with B.Dpsgd(n, d, B.Topology.ring(), 0.05) as ctx:
        for mu in (1.0, -0.1, float("nan")):
            with pytest.raises(B.DpsgdError) as e:
                ctx.mix_step_momentum(Xd, Gd, Vd, mu, Xd)
            assert e.value.status == B.EINVAL
        with pytest.raises(B.DpsgdError) as e:
            ctx.mix_step_momentum(Xd, Gd, Gd, 0.9, Xd)      # V aliases G
        assert e.value.status == B.EINVAL


def test_step_in_place_without_slab_is_refused_and_leaves_x_alone():
    """dpsgd_step is in place, so a W that is not Theorem 3's ring with n > 256 workers has no kernel: the status says
    so, and X still holds the iterate it held (the gradient has been written to the scratch matrix)."""
    n, feat = 300, 20
    rng = np.random.default_rng(8)
    X = rng.standard_normal((n, feat)).astype(np.float32)
    Xd, Gd = to_dev(X), to_dev(np.zeros_like(X))
    inp = torch.from_numpy(rng.standard_normal((n, 4, feat)).astype(np.float32)).cuda()
    tgt = torch.from_numpy(rng.standard_normal((n, 4)).astype(np.float32)).cuda()
    with B.Dpsgd(n, feat, B.Topology.complete(), 0.1) as ctx:
        with pytest.raises(B.DpsgdError) as e:
            ctx.step(B.Model(B.MODEL_LSQ, [feat]), Xd, inp, tgt, 4, Gd)
        assert e.value.status == B.EUNSUPPORTED
        torch.cuda.synchronize()
    assert np.array_equal(from_dev(Xd, feat), X.astype(np.float64))


@pytest.mark.parametrize("topo", ["ring", "torus"])
def test_averaging_on_a_second_stream_then_update_equals_mix_step(topo):
    """Footnote [b]: Algorithm 1's steps 3 and 4 do not depend on each other.  The composition bench.py --overlap
    times - the averaging W X on a second stream (a context with gamma = 0) while the first stream is busy, then
    X_next = (W X) - gamma G as a mix with the identity for W - gives dpsgd_mix_step's result and the oracle's."""
    n, dims = (12, None) if topo == "ring" else (12, (3, 4))
    d, ld, gamma = 20011, 20032, 0.07
    tb = B.Topology.ring() if topo == "ring" else B.Topology.torus(*dims)
    to = (oracle.ring(n) if topo == "ring" else oracle.torus(*dims)).with_fp32_values()
    X, G = random_state(n, d, 77)
    ref = oracle.mix_step(to, X, G, np.float32(gamma))
    Xd, Gd = to_dev(X, ld), to_dev(G, ld)
    direct, avg, out = torch.full_like(Xd, 777.0), torch.full_like(Xd, 777.0), torch.full_like(Xd, 777.0)
    c_direct, c_out = torch.zeros(1, device="cuda"), torch.zeros(1, device="cuda")
    main, side = torch.cuda.current_stream(), torch.cuda.Stream()
    ident = B.Topology.csr(np.arange(n + 1, dtype=np.int32), np.arange(n, dtype=np.int32), np.ones(n, dtype=np.float32))
    with B.Dpsgd(n, d, tb, gamma, ld=ld) as ctx, B.Dpsgd(n, d, tb, 0.0, ld=ld, stream=side) as ctx_avg, \
            B.Dpsgd(n, d, ident, gamma, ld=ld) as ctx_upd:
        ctx.mix_step(Xd, Gd, direct, c_direct)
        side.wait_stream(main)
        with torch.cuda.stream(side):
            ctx_avg.mix_step(Xd, Xd, avg, None)        # gamma = 0: the "gradient" operand contributes nothing
        busy = torch.randn(1 << 20, device="cuda").sum()    # the first stream does something else meanwhile
        main.wait_stream(side)
        ctx_upd.mix_step(avg, Gd, out, c_out)
        torch.cuda.synchronize()
    del busy
    check_close(from_dev(out, d), ref, TOL, "overlapped composition vs oracle")
    check_close(from_dev(out, d), from_dev(direct, d), TOL, "overlapped composition vs dpsgd_mix_step")
    assert float(c_out) == pytest.approx(float(c_direct), rel=1e-5)
