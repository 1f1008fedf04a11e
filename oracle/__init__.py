"""ctypes front end of the CPU oracle (TEST INFRASTRUCTURE, fp64).

Only tests, the smoke check and the benchmark's CPU-baseline leg import this
package; it shares nothing with the HIP library.  All arrays are numpy fp64
(int32 for labels and topology indices); the C side does every computation.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dpsgd_oracle.c")
_LIB = os.path.join(_HERE, "libdpsgd_oracle.so")

LSQ, SOFTMAX, MLP, RESNET20 = 0, 1, 2, 3


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (OpenMP over workers only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(build())
        i32p, f64p = C.POINTER(C.c_int32), C.POINTER(C.c_double)
        for name in ("orc_topology_ring", "orc_topology_ring_chord", "orc_topology_complete"):
            getattr(L, name).restype = C.c_int64
            getattr(L, name).argtypes = [C.c_int32, i32p, i32p, f64p]
        L.orc_topology_torus.restype = C.c_int64
        L.orc_topology_torus.argtypes = [C.c_int32, C.c_int32, i32p, i32p, f64p]
        L.orc_topology_dense.restype = None
        L.orc_topology_dense.argtypes = [C.c_int32, i32p, i32p, f64p, f64p]
        L.orc_topology_check.restype = C.c_int32
        L.orc_topology_check.argtypes = [C.c_int32, i32p, i32p, f64p, C.c_double]
        for name in ("orc_mix_step", "orc_mix_step_swapped"):
            getattr(L, name).restype = None
            getattr(L, name).argtypes = [C.c_int32, C.c_int64, i32p, i32p, f64p, f64p, f64p, C.c_double, f64p]
        L.orc_mix_step_momentum.restype = None
        L.orc_mix_step_momentum.argtypes = [C.c_int32, C.c_int64, i32p, i32p, f64p, f64p, f64p, f64p, C.c_double,
                                            C.c_double, f64p, f64p]
        L.orc_mean.restype = None
        L.orc_mean.argtypes = [C.c_int32, C.c_int64, f64p, f64p]
        L.orc_consensus.restype = C.c_double
        L.orc_consensus.argtypes = [C.c_int32, C.c_int64, f64p]
        L.orc_model_dim.restype = C.c_int64
        L.orc_model_dim.argtypes = [C.c_int32, C.c_int32, i32p]
        L.orc_loss_grad.restype = C.c_double
        L.orc_loss_grad.argtypes = [C.c_int32, C.c_int32, i32p, f64p, f64p, C.c_void_p, C.c_int32, f64p, C.c_int32]
        L.orc_grad_all.restype = None
        L.orc_grad_all.argtypes = [C.c_int32, C.c_int32, i32p, C.c_int32, C.c_int64, f64p, f64p, C.c_void_p,
                                   C.c_int32, f64p, f64p, C.c_int32]
        L.orc_num_threads.restype = C.c_int32
        _lib = L
    return _lib


def _f64(a):
    a = np.ascontiguousarray(a, dtype=np.float64)
    return a, a.ctypes.data_as(C.POINTER(C.c_double))


def _i32(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a, a.ctypes.data_as(C.POINTER(C.c_int32))


class Topology:
    """CSR of the weight matrix W (int32 indices, fp64 values)."""

    def __init__(self, n, rowptr, col, val):
        self.n = int(n)
        self.rowptr = np.ascontiguousarray(rowptr, dtype=np.int32)
        self.col = np.ascontiguousarray(col, dtype=np.int32)
        self.val = np.ascontiguousarray(val, dtype=np.float64)

    def with_fp32_values(self) -> "Topology":
        """Same pattern, values rounded to fp32 and widened back (what an fp32 kernel multiplies by)."""
        return Topology(self.n, self.rowptr, self.col, self.val.astype(np.float32).astype(np.float64))

    def dense(self) -> np.ndarray:
        Wd = np.empty((self.n, self.n), dtype=np.float64)
        lib().orc_topology_dense(self.n, _i32(self.rowptr)[1], _i32(self.col)[1], _f64(self.val)[1],
                                 Wd.ctypes.data_as(C.POINTER(C.c_double)))
        return Wd

    def check(self, tol: float = 1e-12) -> int:
        return int(lib().orc_topology_check(self.n, _i32(self.rowptr)[1], _i32(self.col)[1],
                                            _f64(self.val)[1], tol))


def _build_topo(fn, n, *args):
    nnz = fn(*args, None, None, None)
    rowptr = np.zeros(n + 1, dtype=np.int32)
    col = np.zeros(nnz, dtype=np.int32)
    val = np.zeros(nnz, dtype=np.float64)
    fn(*args, rowptr.ctypes.data_as(C.POINTER(C.c_int32)), col.ctypes.data_as(C.POINTER(C.c_int32)),
       val.ctypes.data_as(C.POINTER(C.c_double)))
    return Topology(n, rowptr, col, val)


def ring(n: int) -> Topology:
    return _build_topo(lib().orc_topology_ring, n, n)


def torus(dim0: int, dim1: int) -> Topology:
    return _build_topo(lib().orc_topology_torus, dim0 * dim1, dim0, dim1)


def ring_chord(n: int) -> Topology:
    """Ring plus a link to the farthest node (supplement, scalability experiment); n even, >= 4."""
    if n < 4 or n % 2:
        raise ValueError("ring_chord needs an even n >= 4")
    return _build_topo(lib().orc_topology_ring_chord, n, n)


def complete(n: int) -> Topology:
    return _build_topo(lib().orc_topology_complete, n, n)


def mix_step(topo: Topology, X, G, gamma: float, swapped: bool = False) -> np.ndarray:
    X, Xp = _f64(X)
    G, Gp = _f64(G)
    n, d = X.shape
    assert n == topo.n and G.shape == X.shape
    Xn = np.empty_like(X)
    fn = lib().orc_mix_step_swapped if swapped else lib().orc_mix_step
    fn(n, d, _i32(topo.rowptr)[1], _i32(topo.col)[1], _f64(topo.val)[1], Xp, Gp, float(gamma),
       Xn.ctypes.data_as(C.POINTER(C.c_double)))
    return Xn


def mix_step_momentum(topo: Topology, X, G, V, gamma: float, mu: float):
    """Heavy-ball variant of Algorithm 1 steps 4-5: returns (X_next, V_next)."""
    X, Xp = _f64(X)
    G, Gp = _f64(G)
    V, Vp = _f64(V)
    n, d = X.shape
    assert n == topo.n and G.shape == X.shape and V.shape == X.shape
    Xn, Vn = np.empty_like(X), np.empty_like(X)
    lib().orc_mix_step_momentum(n, d, _i32(topo.rowptr)[1], _i32(topo.col)[1], _f64(topo.val)[1], Xp, Gp, Vp,
                                float(gamma), float(mu), Xn.ctypes.data_as(C.POINTER(C.c_double)),
                                Vn.ctypes.data_as(C.POINTER(C.c_double)))
    return Xn, Vn


def mean(X) -> np.ndarray:
    X, Xp = _f64(X)
    n, d = X.shape
    out = np.empty(d, dtype=np.float64)
    lib().orc_mean(n, d, Xp, out.ctypes.data_as(C.POINTER(C.c_double)))
    return out


def consensus(X) -> float:
    X, Xp = _f64(X)
    n, d = X.shape
    return float(lib().orc_consensus(n, d, Xp))


def model_dim(kind: int, widths) -> int:
    w, wp = _i32(widths)
    nl = len(w) - 1 if kind in (SOFTMAX, MLP) else 0
    return int(lib().orc_model_dim(kind, nl, wp))


def _targets(kind, targets):
    if kind == LSQ:
        t = np.ascontiguousarray(targets, dtype=np.float64)
    else:
        t = np.ascontiguousarray(targets, dtype=np.int32)
    return t, t.ctypes.data_as(C.c_void_p)


def loss_grad(kind: int, widths, x, inputs, targets, want_grad: bool = True, bf16_operands: bool = False):
    """One worker: (loss, grad or None).  inputs [B][features].  ``bf16_operands`` rounds the operands
    of every contraction to bf16 (the precision the bf16 workloads prescribe); sums stay fp64."""
    w, wp = _i32(widths)
    nl = len(w) - 1 if kind in (SOFTMAX, MLP) else 0
    x, xp = _f64(x)
    inp, ip = _f64(inputs)
    B = inp.shape[0]
    t, tp = _targets(kind, targets)
    g = np.empty_like(x) if want_grad else None
    gp = g.ctypes.data_as(C.POINTER(C.c_double)) if want_grad else None
    loss = lib().orc_loss_grad(kind, nl, wp, xp, ip, tp, B, gp, 1 if bf16_operands else 0)
    return float(loss), g


def grad_all(kind: int, widths, X, inputs, targets, bf16_operands: bool = False):
    """All workers: (G [n][d], loss [n]).  inputs [n][B][features], targets [n][B]."""
    w, wp = _i32(widths)
    nl = len(w) - 1 if kind in (SOFTMAX, MLP) else 0
    X, Xp = _f64(X)
    n, d = X.shape
    inp, ip = _f64(inputs)
    B = inp.shape[1]
    t, tp = _targets(kind, targets)
    G = np.empty_like(X)
    loss = np.empty(n, dtype=np.float64)
    lib().orc_grad_all(kind, nl, wp, n, d, Xp, ip, tp, B, G.ctypes.data_as(C.POINTER(C.c_double)),
                       loss.ctypes.data_as(C.POINTER(C.c_double)), 1 if bf16_operands else 0)
    return G, loss


def iteration(kind: int, widths, topo: Topology, gamma: float, X, inputs, targets, bf16_operands: bool = False):
    """One iteration of Algorithm 1: returns (X_next, G, loss)."""
    G, loss = grad_all(kind, widths, X, inputs, targets, bf16_operands)
    return mix_step(topo, X, G, gamma), G, loss


def num_threads() -> int:
    return int(lib().orc_num_threads())
