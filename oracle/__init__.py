"""CPU oracle of the RRM per-layer update.  TEST INFRASTRUCTURE ONLY.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py`` may
import this package.  It never imports the HIP library or its Python binding, and the HIP
library never calls into it.

* :func:`dense` is the definition of the expected result: the projection layer
  ``P = F * I + b`` / ``P = W I + b`` (Eq. 3, Sec. 3.1), computed by plain nested loops in C
  (``rrm_oracle.c``), integers exactly, floating point in float64.
* :class:`State` / :meth:`State.step` follow Algorithm 1 (Sec. 3.2) for one layer: difference
  with the stored input, weights times the non-zero entries of the difference, sum into the
  stored projection, snapshot.
* :func:`relu_requant_pool` is the nonlinear map ``f`` the int8 conv-stack harness puts between
  layers (the paper leaves ``f`` to the network; this one is the harness's, written in numpy).
* :mod:`oracle.accounting` holds the operation-count formulas of Table 1 / Eq. 6, 9, 10.

bf16 tensors are passed as their 16-bit patterns (``uint16``) and widened exactly here;
binary tensors are passed as +1/-1 ``int8`` arrays, so that the binary case *is* the integer
case, as Sec. 4.3 reduces it ("taking their signs").
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "rrm_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

CONV, FC = 0, 1
I8, BF16, BIN = 0, 1, 2


class _Shape(ctypes.Structure):
    _fields_ = [(k, ctypes.c_int) for k in
                ("kind", "n", "h", "w", "c_in", "c_out", "kh", "kw", "stride", "pad", "groups")]


def build(force: bool = False) -> str:
    """Compile ``rrm_oracle.c`` with gcc into ``oracle/liboracle.so``."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra", "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        P = ctypes.c_void_p
        for name in ("orc_dense_i8", "orc_dense_f64"):
            getattr(L, name).argtypes = [ctypes.POINTER(_Shape), P, P, P, P]
            getattr(L, name).restype = ctypes.c_int
        L.orc_step_i8.argtypes = [ctypes.POINTER(_Shape), P, P, P, P, ctypes.POINTER(ctypes.c_int64)]
        L.orc_step_f64.argtypes = [ctypes.POINTER(_Shape), P, P, P, P, ctypes.c_float, ctypes.POINTER(ctypes.c_int64),
                                   ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_double)]
        L.orc_step_i8.restype = L.orc_step_f64.restype = ctypes.c_int
        L.orc_threads.restype = ctypes.c_int
        L.orc_set_threads.argtypes = [ctypes.c_int]
        _lib = L
    return _lib


def threads() -> int:
    return int(lib().orc_threads())


def set_threads(t: int) -> None:
    lib().orc_set_threads(int(t))


def _cshape(shape) -> _Shape:
    return _Shape(*(int(getattr(shape, k)) for k, _ in _Shape._fields_))


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def bf16_to_f64(bits: np.ndarray) -> np.ndarray:
    """Exact value of bfloat16 patterns as float64."""
    u = np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


def _y_shape(shape):
    if shape.kind == FC:
        return (shape.n, shape.c_out)
    ho = (shape.h + 2 * shape.pad - shape.kh) // shape.stride + 1
    wo = (shape.w + 2 * shape.pad - shape.kw) // shape.stride + 1
    return (shape.n, ho, wo, shape.c_out)


def _as_values(dtype: int, a: Optional[np.ndarray], is_bias=False) -> Optional[np.ndarray]:
    """Bring a boundary-format tensor into the oracle's arithmetic type."""
    if a is None:
        return None
    if dtype == BF16:
        if is_bias:
            return np.ascontiguousarray(a, dtype=np.float64)
        if a.dtype == np.uint16:
            return bf16_to_f64(a)
        return np.ascontiguousarray(a, dtype=np.float64)
    if is_bias:
        return np.ascontiguousarray(a, dtype=np.int32)
    return np.ascontiguousarray(a, dtype=np.int8)


def dense(shape, dtype: int, weights: np.ndarray, bias: Optional[np.ndarray], x: np.ndarray) -> np.ndarray:
    """Eq. 3: the projection layer of one frame.  int32 for I8 / BIN, float64 for BF16."""
    cs = _cshape(shape)
    w = _as_values(dtype, weights)
    b = _as_values(dtype, bias, True)
    xv = _as_values(dtype, x)
    if dtype == BF16:
        y = np.empty(_y_shape(shape), dtype=np.float64)
        lib().orc_dense_f64(ctypes.byref(cs), _ptr(w), _ptr(b), _ptr(xv), _ptr(y))
        return y
    y = np.empty(_y_shape(shape), dtype=np.int32)
    ovf = lib().orc_dense_i8(ctypes.byref(cs), _ptr(w), _ptr(b), _ptr(xv), _ptr(y))
    if ovf:
        raise OverflowError("projection does not fit int32")
    return y


class State:
    """Per-layer state of Algorithm 1: the stored input I_{t-1} and projection P_{t-1}.

    Initial state: I_0 = 0 (Algorithm 1, first line) and P_0 = b, which is Eq. 3 evaluated at
    I_0 = 0; the recurrence itself never adds the bias (Fig. 1: the sparse convolution has no
    bias term).
    """

    def __init__(self, shape, dtype: int, weights: np.ndarray, bias: Optional[np.ndarray]):
        self.shape, self.dtype = shape, dtype
        self.cs = _cshape(shape)
        self.w = _as_values(dtype, weights)
        xs = (shape.n, shape.c_in) if shape.kind == FC else (shape.n, shape.h, shape.w, shape.c_in)
        ys = _y_shape(shape)
        if dtype == BF16:
            self.i_prev = np.zeros(xs, dtype=np.float64)
            self.p_prev = np.zeros(ys, dtype=np.float64)
        else:
            self.i_prev = np.zeros(xs, dtype=np.int8)
            self.p_prev = np.zeros(ys, dtype=np.int32)
        if bias is not None:
            self.p_prev += _as_values(dtype, bias, True).reshape((1,) * (len(ys) - 1) + (-1,))
        self.last_nnz = 0

    def step(self, x_t: np.ndarray, eps: float = 0.0) -> np.ndarray:
        """One (layer, frame) iteration of Algorithm 1; returns P_t (a view of the state).

        ``eps`` > 0 (bf16 only) truncates differences below the threshold (Sec. 3.4, "Improving
        sparsity"); what is truncated is not committed to the stored input, so P = b + W (*) I holds.
        ``last_truncated`` / ``last_truncated_sumsq`` describe the truncated map of this step."""
        xv = _as_values(self.dtype, x_t)
        nnz = ctypes.c_int64(0)
        self.last_truncated, self.last_truncated_sumsq = 0, 0.0
        if self.dtype == BF16:
            ntr, ssq = ctypes.c_int64(0), ctypes.c_double(0.0)
            lib().orc_step_f64(ctypes.byref(self.cs), _ptr(self.w), _ptr(self.i_prev), _ptr(self.p_prev),
                               _ptr(xv), ctypes.c_float(eps), ctypes.byref(nnz), ctypes.byref(ntr), ctypes.byref(ssq))
            self.last_truncated, self.last_truncated_sumsq = int(ntr.value), float(ssq.value)
        else:
            if eps:
                raise ValueError("the truncation threshold is defined for the floating-point path only")
            ovf = lib().orc_step_i8(ctypes.byref(self.cs), _ptr(self.w), _ptr(self.i_prev), _ptr(self.p_prev),
                                    _ptr(xv), ctypes.byref(nnz))
            if ovf:
                raise OverflowError("projection does not fit int32")
        self.last_nnz = int(nnz.value)
        return self.p_prev


def relu_requant_pool(y: np.ndarray, shift: int, pool: bool) -> np.ndarray:
    """Harness-owned nonlinear map between int8 conv layers: ReLU, arithmetic right shift by
    ``shift``, clamp to 127, then (if ``pool``) 3x3 max pooling with stride 2, no padding.
    ``y`` is NHWC int32; the result is NHWC int8."""
    a = np.minimum(np.maximum(y.astype(np.int64), 0) >> int(shift), 127).astype(np.int8)
    if not pool:
        return a
    n, h, w, c = a.shape
    ho, wo = (h - 3) // 2 + 1, (w - 3) // 2 + 1
    out = np.full((n, ho, wo, c), -128, dtype=np.int8)
    for dy in range(3):
        for dx in range(3):
            out = np.maximum(out, a[:, dy:dy + 2 * ho - 1:2, dx:dx + 2 * wo - 1:2, :])
    return out


def calibrate_shift(y: np.ndarray, q: float = 99.9) -> int:
    """Smallest right shift that brings the q-th percentile of ReLU(y) to at most 127."""
    v = float(np.percentile(np.maximum(y, 0), q))
    s = 0
    while (int(v) >> s) > 127:
        s += 1
    return s
