"""Thin ctypes binding of the C-ABI in ``include/dpsgd.h`` (argument marshalling only).

Tensors are torch tensors on the GPU (torch provides device memory and the stream); every
computation happens inside the library's HIP kernels.  There is no fallback: if the library is
missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libdpsgd_hip.so")

OK, EINVAL, ETOPOLOGY, ENOMEM, EDEVICE, EUNSUPPORTED = range(6)
TOPO_CSR, TOPO_RING, TOPO_TORUS2D, TOPO_COMPLETE, TOPO_RING_CHORD = range(5)
MODEL_LSQ, MODEL_SOFTMAX, MODEL_MLP, MODEL_RESNET20 = range(4)

EXPORTS = (
    "dpsgd_topology_build", "dpsgd_model_dim", "dpsgd_recommended_ld", "dpsgd_create", "dpsgd_destroy", "dpsgd_set_gamma",
    "dpsgd_set_option", "dpsgd_topology_export", "dpsgd_grad", "dpsgd_step", "dpsgd_mix_step", "dpsgd_mix_step_swapped",
    "dpsgd_mix_step_momentum", "dpsgd_mix_step_static", "dpsgd_mean", "dpsgd_read_timing", "dpsgd_strerror",
)


class DpsgdError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {strerror(status)} (status {status})")


class _Topology(C.Structure):
    _fields_ = [("kind", C.c_int32), ("dim0", C.c_int32), ("dim1", C.c_int32),
                ("rowptr", C.POINTER(C.c_int32)), ("colidx", C.POINTER(C.c_int32)), ("vals", C.POINTER(C.c_float))]


class _Model(C.Structure):
    _fields_ = [("kind", C.c_int32), ("n_widths", C.c_int32), ("widths", C.POINTER(C.c_int32)),
                ("compute_bf16", C.c_int32)]


class _Batch(C.Structure):
    _fields_ = [("inputs", C.c_void_p), ("targets", C.c_void_p), ("batch", C.c_int32), ("input_is_bf16", C.c_int32)]


_lib = None


def load():
    """Loads the built library; raises if it has not been built (no fallback path exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_1705_09056_amd.build`")
    L = C.CDLL(LIB_PATH)
    i32p, f32p, i64p, vp = C.POINTER(C.c_int32), C.POINTER(C.c_float), C.POINTER(C.c_int64), C.c_void_p
    L.dpsgd_topology_build.restype = C.c_int
    L.dpsgd_topology_build.argtypes = [C.c_int32, C.POINTER(_Topology), i32p, i32p, f32p, i64p]
    L.dpsgd_model_dim.restype = C.c_int64
    L.dpsgd_model_dim.argtypes = [C.POINTER(_Model)]
    L.dpsgd_recommended_ld.restype = C.c_int64
    L.dpsgd_recommended_ld.argtypes = [C.c_int64, C.POINTER(_Topology)]
    L.dpsgd_create.restype = C.c_int
    L.dpsgd_create.argtypes = [C.POINTER(vp), C.c_int32, C.c_int64, C.c_int64, C.POINTER(_Topology), C.c_float, vp]
    L.dpsgd_destroy.restype = C.c_int
    L.dpsgd_destroy.argtypes = [vp]
    L.dpsgd_set_gamma.restype = C.c_int
    L.dpsgd_set_gamma.argtypes = [vp, C.c_float]
    L.dpsgd_set_option.restype = C.c_int
    L.dpsgd_set_option.argtypes = [vp, C.c_char_p, C.c_int64]
    L.dpsgd_topology_export.restype = C.c_int
    L.dpsgd_topology_export.argtypes = [vp, i32p, i32p, f32p, i64p]
    L.dpsgd_grad.restype = C.c_int
    L.dpsgd_grad.argtypes = [vp, C.POINTER(_Model), vp, C.POINTER(_Batch), vp, vp]
    L.dpsgd_step.restype = C.c_int
    L.dpsgd_step.argtypes = [vp, C.POINTER(_Model), vp, C.POINTER(_Batch), vp, vp, vp]
    for name in ("dpsgd_mix_step", "dpsgd_mix_step_swapped"):
        getattr(L, name).restype = C.c_int
        getattr(L, name).argtypes = [vp, vp, vp, vp, vp]
    L.dpsgd_mix_step_momentum.restype = C.c_int
    L.dpsgd_mix_step_momentum.argtypes = [vp, vp, vp, vp, C.c_float, vp, vp]
    L.dpsgd_mix_step_static.restype = C.c_int
    L.dpsgd_mix_step_static.argtypes = [C.c_int32, C.c_int64, C.c_int64, C.POINTER(_Topology), C.c_float, vp, vp, vp, vp, vp]
    L.dpsgd_mean.restype = C.c_int
    L.dpsgd_mean.argtypes = [vp, vp, vp]
    L.dpsgd_read_timing.restype = C.c_int
    L.dpsgd_read_timing.argtypes = [vp, C.POINTER(C.c_double), i64p]
    L.dpsgd_strerror.restype = C.c_char_p
    L.dpsgd_strerror.argtypes = [C.c_int]
    _lib = L
    return L


def strerror(status: int) -> str:
    return load().dpsgd_strerror(int(status)).decode()


def _check(status: int, where: str):
    if status != OK:
        raise DpsgdError(status, where)


class Topology:
    """Host description of W: a tag (ring / torus / complete / ring with far link) or CSR arrays."""

    def __init__(self, kind: int, dim0: int = 0, dim1: int = 0, rowptr=None, colidx=None, vals=None):
        self.kind, self.dim0, self.dim1 = int(kind), int(dim0), int(dim1)
        self.rowptr = None if rowptr is None else np.ascontiguousarray(rowptr, dtype=np.int32)
        self.colidx = None if colidx is None else np.ascontiguousarray(colidx, dtype=np.int32)
        self.vals = None if vals is None else np.ascontiguousarray(vals, dtype=np.float32)

    @staticmethod
    def ring():
        return Topology(TOPO_RING)

    @staticmethod
    def torus(dim0: int, dim1: int):
        return Topology(TOPO_TORUS2D, dim0, dim1)

    @staticmethod
    def complete():
        return Topology(TOPO_COMPLETE)

    @staticmethod
    def ring_chord():
        return Topology(TOPO_RING_CHORD)

    @staticmethod
    def csr(rowptr, colidx, vals):
        return Topology(TOPO_CSR, 0, 0, rowptr, colidx, vals)

    def _c(self) -> _Topology:
        t = _Topology(self.kind, self.dim0, self.dim1, None, None, None)
        if self.rowptr is not None:
            t.rowptr = self.rowptr.ctypes.data_as(C.POINTER(C.c_int32))
        if self.colidx is not None:
            t.colidx = self.colidx.ctypes.data_as(C.POINTER(C.c_int32))
        if self.vals is not None:
            t.vals = self.vals.ctypes.data_as(C.POINTER(C.c_float))
        return t


def topology_build(n: int, topo: Topology):
    """Host only: (rowptr, colidx, vals) of W as the library stores it."""
    L = load()
    t = topo._c()
    nnz = C.c_int64(0)
    _check(L.dpsgd_topology_build(n, C.byref(t), None, None, None, C.byref(nnz)), "dpsgd_topology_build")
    rowptr = np.zeros(n + 1, dtype=np.int32)
    col = np.zeros(nnz.value, dtype=np.int32)
    val = np.zeros(nnz.value, dtype=np.float32)
    _check(L.dpsgd_topology_build(n, C.byref(t), rowptr.ctypes.data_as(C.POINTER(C.c_int32)),
                                  col.ctypes.data_as(C.POINTER(C.c_int32)),
                                  val.ctypes.data_as(C.POINTER(C.c_float)), C.byref(nnz)), "dpsgd_topology_build")
    return rowptr, col, val


def recommended_ld(d: int, topo: Topology) -> int:
    """Host only: the row stride (floats) dpsgd_recommended_ld suggests for an n x d replica matrix."""
    t = topo._c()
    ld = int(load().dpsgd_recommended_ld(d, C.byref(t)))
    if ld < 0:
        raise DpsgdError(EINVAL, "dpsgd_recommended_ld")
    return ld


def mix_step_static(n: int, d: int, topo: Topology, gamma: float, X_in, G, X_out, consensus=None, ld: int = 0,
                    stream=None):
    """dpsgd_mix_step_static: the mix + step without a context and without any allocation (ring / small torus tags)."""
    import torch
    ld = int(ld) if ld else int(d)
    for t, name in ((X_in, "X_in"), (G, "G"), (X_out, "X_out")):
        if t.dtype != torch.float32 or not t.is_cuda or not t.is_contiguous() or tuple(t.shape) != (n, ld):
            raise ValueError(f"{name} must be a contiguous float32 CUDA tensor of shape ({n}, {ld})")
    if stream is None:
        stream = torch.cuda.current_stream()
    t = topo._c()
    _check(load().dpsgd_mix_step_static(int(n), int(d), ld, C.byref(t), float(gamma), _ptr(X_in), _ptr(G), _ptr(X_out),
                                        _ptr(consensus), C.c_void_p(stream.cuda_stream)), "dpsgd_mix_step_static")


class Model:
    def __init__(self, kind: int, widths: Sequence[int], compute_bf16: bool = False):
        self.kind = int(kind)
        self.widths = np.ascontiguousarray(widths, dtype=np.int32)
        self.compute_bf16 = bool(compute_bf16)

    def _c(self) -> _Model:
        return _Model(self.kind, len(self.widths), self.widths.ctypes.data_as(C.POINTER(C.c_int32)),
                      1 if self.compute_bf16 else 0)

    @property
    def dim(self) -> int:
        m = self._c()
        return int(load().dpsgd_model_dim(C.byref(m)))


def _ptr(t) -> int:
    """Device pointer of a torch tensor (None -> NULL)."""
    return None if t is None else C.c_void_p(t.data_ptr())


class Dpsgd:
    """Owns one dpsgd_ctx.  X, G: torch float32 CUDA tensors of shape [n, ld] (columns d..ld-1 padding)."""

    def __init__(self, n: int, d: int, topo: Topology, gamma: float, ld: int = 0, stream=None):
        import torch
        self._L = load()
        self.n, self.d, self.ld = int(n), int(d), int(ld) if ld else int(d)
        self._topo = topo
        self._handle = C.c_void_p(None)
        if stream is None:
            stream = torch.cuda.current_stream()
        self.stream = stream
        t = topo._c()
        st = self._L.dpsgd_create(C.byref(self._handle), self.n, self.d, self.ld, C.byref(t), float(gamma),
                                  C.c_void_p(stream.cuda_stream))
        _check(st, "dpsgd_create")

    def close(self):
        if getattr(self, "_handle", None) is not None and self._handle.value:
            st = self._L.dpsgd_destroy(self._handle)
            self._handle = C.c_void_p(None)
            _check(st, "dpsgd_destroy")

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()

    def set_gamma(self, gamma: float):
        _check(self._L.dpsgd_set_gamma(self._handle, float(gamma)), "dpsgd_set_gamma")

    def set_option(self, key: str, value: int):
        _check(self._L.dpsgd_set_option(self._handle, key.encode(), int(value)), "dpsgd_set_option")

    def topology_export(self):
        nnz = C.c_int64(0)
        _check(self._L.dpsgd_topology_export(self._handle, None, None, None, C.byref(nnz)), "dpsgd_topology_export")
        rowptr = np.zeros(self.n + 1, dtype=np.int32)
        col = np.zeros(nnz.value, dtype=np.int32)
        val = np.zeros(nnz.value, dtype=np.float32)
        _check(self._L.dpsgd_topology_export(self._handle, rowptr.ctypes.data_as(C.POINTER(C.c_int32)),
                                             col.ctypes.data_as(C.POINTER(C.c_int32)),
                                             val.ctypes.data_as(C.POINTER(C.c_float)), C.byref(nnz)),
               "dpsgd_topology_export")
        return rowptr, col, val

    def _check_mat(self, t, name):
        import torch
        if t.dtype != torch.float32 or not t.is_cuda or not t.is_contiguous() or tuple(t.shape) != (self.n, self.ld):
            raise ValueError(f"{name} must be a contiguous float32 CUDA tensor of shape ({self.n}, {self.ld})")

    def step(self, model: Model, X, inputs, targets, batch: int, G, loss=None, consensus=None,
             input_is_bf16: bool = False):
        """One whole iteration in place (dpsgd_step)."""
        self._grad_like(self._L.dpsgd_step, "dpsgd_step", model, X, inputs, targets, batch, G, loss, input_is_bf16,
                        extra=(_ptr(consensus),))

    def grad(self, model: Model, X, inputs, targets, batch: int, G, loss=None, input_is_bf16: bool = False):
        self._grad_like(self._L.dpsgd_grad, "dpsgd_grad", model, X, inputs, targets, batch, G, loss, input_is_bf16)

    def _grad_like(self, fn, name, model, X, inputs, targets, batch, G, loss, input_is_bf16, extra=()):
        self._check_mat(X, "X")
        self._check_mat(G, "G")
        import torch
        feat = int(np.prod(model.widths[:3])) if model.kind == MODEL_RESNET20 else int(model.widths[0])
        want = torch.bfloat16 if input_is_bf16 else torch.float32
        if inputs.dtype != want or inputs.numel() != self.n * batch * feat or not inputs.is_contiguous():
            raise ValueError("inputs must be contiguous [n][batch][features] of dtype %s" % want)
        tdt = torch.float32 if model.kind == MODEL_LSQ else torch.int32
        if targets.dtype != tdt or targets.numel() != self.n * batch or not targets.is_contiguous():
            raise ValueError("targets must be contiguous [n][batch] of dtype %s" % tdt)
        if loss is not None and (loss.dtype != torch.float32 or loss.numel() < self.n):
            raise ValueError("loss must hold n float32 values")
        m = model._c()
        b = _Batch(C.c_void_p(inputs.data_ptr()), C.c_void_p(targets.data_ptr()), int(batch), 1 if input_is_bf16 else 0)
        _check(fn(self._handle, C.byref(m), _ptr(X), C.byref(b), _ptr(G), _ptr(loss), *extra), name)

    def mix_step(self, X_in, G, X_out, consensus=None, swapped: bool = False):
        self._check_mat(X_in, "X_in")
        self._check_mat(G, "G")
        self._check_mat(X_out, "X_out")
        fn = self._L.dpsgd_mix_step_swapped if swapped else self._L.dpsgd_mix_step
        _check(fn(self._handle, _ptr(X_in), _ptr(G), _ptr(X_out), _ptr(consensus)), "dpsgd_mix_step")

    def mix_step_momentum(self, X_in, G, V, mu: float, X_out, consensus=None):
        """V <- mu V + G (in place); X_out = W X_in - gamma V."""
        for t, name in ((X_in, "X_in"), (G, "G"), (V, "V"), (X_out, "X_out")):
            self._check_mat(t, name)
        _check(self._L.dpsgd_mix_step_momentum(self._handle, _ptr(X_in), _ptr(G), _ptr(V), C.c_float(mu), _ptr(X_out),
                                               _ptr(consensus)), "dpsgd_mix_step_momentum")

    def read_timing(self):
        """(total ms, launches) of the fused kernels bracketed since the last call (option "time_fused")."""
        ms, cnt = C.c_double(0.0), C.c_int64(0)
        _check(self._L.dpsgd_read_timing(self._handle, C.byref(ms), C.byref(cnt)), "dpsgd_read_timing")
        return ms.value, cnt.value

    def mean(self, X, xbar):
        self._check_mat(X, "X")
        if xbar.numel() < self.d:
            raise ValueError("xbar must hold d floats")
        _check(self._L.dpsgd_mean(self._handle, _ptr(X), _ptr(xbar)), "dpsgd_mean")
