"""Host-side tests of the C-ABI: the library loads, exports what include/dpsgd.h declares,
and rejects bad arguments and bad weight matrices before touching a device."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import oracle
from paper_1705_09056_amd import binding as B
from paper_1705_09056_amd import synth
from paper_1705_09056_amd.configs import CONFIGS

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "dpsgd.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dpsgd_[a-z0-9_]+)\s*\(", text)))


def test_library_loads_and_exports_every_declared_symbol():
    L = B.load()
    names = declared_functions()
    assert set(names) == set(B.EXPORTS)
    for name in names:
        assert getattr(L, name) is not None


def test_strerror_is_total():
    for s in range(0, 8):
        assert isinstance(B.strerror(s), str) and B.strerror(s)


@pytest.mark.parametrize("n", [1, 2, 3, 8, 16, 64, 112])
def test_ring_topology_indices_bit_exact_vs_oracle(n):
    rowptr, col, val = B.topology_build(n, B.Topology.ring())
    t = oracle.ring(n)
    assert np.array_equal(rowptr, t.rowptr) and rowptr.dtype == np.int32
    assert np.array_equal(col, t.col) and col.dtype == np.int32
    assert np.array_equal(val, t.val.astype(np.float32))          # (float)(1/3), duplicates accumulated
    if n >= 3:
        assert np.all(val == np.float32(1.0 / 3.0))


@pytest.mark.parametrize("dims", [(8, 8), (3, 5), (2, 4), (1, 6), (4, 16)])
def test_torus_topology_indices_bit_exact_vs_oracle(dims):
    n = dims[0] * dims[1]
    rowptr, col, val = B.topology_build(n, B.Topology.torus(*dims))
    t = oracle.torus(*dims)
    assert np.array_equal(rowptr, t.rowptr)
    assert np.array_equal(col, t.col)
    np.testing.assert_allclose(val, t.val, rtol=3e-7)
    if min(dims) >= 3:
        assert np.all(val == np.float32(0.2))


@pytest.mark.parametrize("n", [4, 6, 16, 112])
def test_ring_with_far_link_indices_bit_exact_vs_oracle(n):
    rowptr, col, val = B.topology_build(n, B.Topology.ring_chord())
    t = oracle.ring_chord(n)
    assert np.array_equal(rowptr, t.rowptr)
    assert np.array_equal(col, t.col)
    assert np.array_equal(val, t.val.astype(np.float32))
    if n > 4:
        assert np.all(val == np.float32(0.25))


def test_ring_with_far_link_rejects_odd_or_tiny_rings():
    for n in (2, 3, 5, 15):
        with pytest.raises(B.DpsgdError) as e:
            B.topology_build(n, B.Topology.ring_chord())
        assert e.value.status == B.EINVAL


def test_complete_and_csr_roundtrip():
    rowptr, col, val = B.topology_build(5, B.Topology.complete())
    t = oracle.complete(5)
    assert np.array_equal(rowptr, t.rowptr) and np.array_equal(col, t.col)
    assert np.all(val == np.float32(0.2))
    r2, c2, v2 = B.topology_build(5, B.Topology.csr(rowptr, col, val))
    assert np.array_equal(r2, rowptr) and np.array_equal(c2, col) and np.array_equal(v2, val)


def _status(fn):
    with pytest.raises(B.DpsgdError) as e:
        fn()
    return e.value.status


def test_invalid_topologies_are_rejected():
    t = oracle.ring(6)
    v = t.val.astype(np.float32)
    bad = v.copy(); bad[0] = 0.5
    assert _status(lambda: B.topology_build(6, B.Topology.csr(t.rowptr, t.col, bad))) == B.ETOPOLOGY
    # not symmetric (directed 3-cycle with self loops)
    assert _status(lambda: B.topology_build(3, B.Topology.csr([0, 2, 4, 6], [0, 1, 1, 2, 0, 2], [0.5] * 6))) == B.ETOPOLOGY
    # column out of range / unsorted / negative weight / rowptr not starting at 0 / decreasing
    assert _status(lambda: B.topology_build(2, B.Topology.csr([0, 2, 4], [0, 2, 0, 1], [0.5] * 4))) == B.ETOPOLOGY
    assert _status(lambda: B.topology_build(2, B.Topology.csr([0, 2, 4], [1, 0, 0, 1], [0.5] * 4))) == B.ETOPOLOGY
    assert _status(lambda: B.topology_build(2, B.Topology.csr([0, 2, 4], [0, 1, 0, 1], [1.5, -0.5, -0.5, 1.5]))) == B.ETOPOLOGY
    assert _status(lambda: B.topology_build(2, B.Topology.csr([1, 2, 4], [0, 1, 0, 1], [0.5] * 4))) == B.ETOPOLOGY
    assert _status(lambda: B.topology_build(2, B.Topology.csr([0, 3, 2], [0, 1, 0, 1], [0.5] * 4))) == B.ETOPOLOGY
    # NaN weight
    assert _status(lambda: B.topology_build(2, B.Topology.csr([0, 2, 4], [0, 1, 0, 1], [np.nan, 0.5, 0.5, 0.5]))) == B.ETOPOLOGY
    # torus whose dims do not multiply to n, missing CSR arrays, n < 1, unknown kind
    assert _status(lambda: B.topology_build(10, B.Topology.torus(3, 3))) == B.EINVAL
    assert _status(lambda: B.topology_build(4, B.Topology(B.TOPO_CSR))) == B.EINVAL
    assert _status(lambda: B.topology_build(0, B.Topology.ring())) == B.EINVAL
    assert _status(lambda: B.topology_build(4, B.Topology(17))) == B.EINVAL


def test_model_dim():
    for cfg in CONFIGS:
        assert B.Model(cfg.model_kind, cfg.widths).dim == synth.model_dim(cfg.model_kind, cfg.widths)
    assert B.Model(B.MODEL_MLP, [3072, 4096, 4096, 10]).dim == 29409290
    assert B.Model(B.MODEL_RESNET20, [3, 32, 32, 16, 3, 10]).dim == 268365
    assert B.Model(B.MODEL_LSQ, [4, 4]).dim == -1
    assert B.Model(B.MODEL_SOFTMAX, [4]).dim == -1
    assert B.Model(B.MODEL_MLP, [4, 0, 3]).dim == -1
    assert B.Model(9, [4]).dim == -1


def test_recommended_row_stride():
    ring, torus = B.Topology.ring(), B.Topology.torus(8, 8)
    assert B.recommended_ld(29409290, ring) == 29409536          # 256 x 114881: rows 1 KB-aligned
    assert B.recommended_ld(29409290, torus) == 29409344         # 64 x 459521, 64 beyond a multiple of 256
    assert B.recommended_ld(256, ring) == 256 and B.recommended_ld(257, ring) == 512
    assert B.recommended_ld(256, torus) == 320 and B.recommended_ld(193, torus) == 320 and B.recommended_ld(192, torus) == 192
    for d in (1, 63, 64, 65, 1000, 30730, 268365):
        for topo in (ring, torus, B.Topology.complete(), B.Topology.ring_chord()):
            ld = B.recommended_ld(d, topo)
            assert d <= ld < d + 320 and ld % 64 == 0
            assert (ld % 256 != 0) if topo is torus else (ld % 256 == 0)
    with pytest.raises(B.DpsgdError):
        B.recommended_ld(0, ring)


def test_create_rejects_bad_arguments_before_any_device_call():
    L = B.load()
    h = C.c_void_p(None)
    ring = B.Topology.ring()._c()

    def create(n, d, ld, topo, gamma):
        return L.dpsgd_create(C.byref(h), n, d, ld, C.byref(topo) if topo is not None else None, gamma, None)

    assert create(0, 8, 0, ring, 0.1) == B.EINVAL
    assert create(4, 0, 0, ring, 0.1) == B.EINVAL
    assert create(4, 8, 4, ring, 0.1) == B.EINVAL           # ld < d
    assert create(4, 8, 0, None, 0.1) == B.EINVAL
    assert create(4, 8, 0, ring, float("nan")) == B.EINVAL
    assert create(4, 8, 0, ring, float("inf")) == B.EINVAL
    bad = B.Topology.csr([0, 2, 4, 6], [0, 1, 1, 2, 0, 2], [0.5] * 6)
    assert create(3, 8, 0, bad._c(), 0.1) == B.ETOPOLOGY
    assert h.value is None
    assert L.dpsgd_create(None, 4, 8, 0, C.byref(ring), 0.1, None) == B.EINVAL
    # null contexts
    assert L.dpsgd_destroy(None) == B.OK
    assert L.dpsgd_set_gamma(None, 0.1) == B.EINVAL
    assert L.dpsgd_mix_step(None, None, None, None, None) == B.EINVAL
    assert L.dpsgd_mean(None, None, None) == B.EINVAL
    assert L.dpsgd_grad(None, None, None, None, None, None) == B.EINVAL


def test_static_mix_step_rejects_what_its_fixed_array_cannot_hold_before_any_device_call():
    """dpsgd_mix_step_static: argument errors and sizes beyond its fixed device array are decided on the host, so
    the statuses come back on a machine without a GPU."""
    L = B.load()
    fake = C.c_void_p(0x1000)                      # never dereferenced: every case below is refused first

    def call(n, d, ld, topo, x_in=fake, g=C.c_void_p(0x40000000), x_out=fake, gamma=0.1):
        t = topo._c()
        return L.dpsgd_mix_step_static(n, d, ld, C.byref(t), C.c_float(gamma), x_in, g, x_out, None, None)

    ring, torus = B.Topology.ring(), B.Topology.torus
    assert call(8, 64, 64, ring, x_in=None) == B.EINVAL
    assert call(8, 64, 64, ring, g=None) == B.EINVAL
    assert call(0, 64, 64, ring) == B.EINVAL
    assert call(8, 0, 0, ring) == B.EINVAL
    assert call(8, 64, 63, ring) == B.EINVAL                      # ld < d
    assert call(8, 64, 64, ring, gamma=float("nan")) == B.EINVAL
    assert call(8, 64, 64, ring, g=fake) == B.EINVAL              # G aliases X_out
    assert call(8, 64, 64, ring, x_out=C.c_void_p(0x1100)) == B.EINVAL   # X_out overlaps X_in without being it
    assert call(12, 64, 64, torus(3, 5)) == B.EINVAL              # 3 x 5 is not 12 workers
    # valid requests the fixed array has no room or no kernel for
    assert call(8, (1 << 25) + 1, 0, ring, g=C.c_void_p(1 << 40)) == B.EUNSUPPORTED
    assert call(2, 64, 64, ring) == B.EUNSUPPORTED                # coinciding neighbours need a CSR
    assert call(16, 64, 64, torus(2, 8)) == B.EUNSUPPORTED
    assert call(17 * 16, 64, 64, torus(17, 16)) == B.EUNSUPPORTED # 272 workers: slab beyond the fixed CSR room
    assert call(8, 64, 64, B.Topology.complete()) == B.EUNSUPPORTED
    assert call(8, 64, 64, B.Topology.ring_chord()) == B.EUNSUPPORTED
    rowptr, col, val = B.topology_build(8, ring)
    assert call(8, 64, 64, B.Topology.csr(rowptr, col, val)) == B.EUNSUPPORTED
