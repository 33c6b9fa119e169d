"""ctypes binding of ``include/rrm.h`` (same names, argument marshalling only)."""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))

CONV, FC = 0, 1
I8, BF16, BIN = 0, 1, 2

RRM_OK = 0
RRM_ERR_RANGE = -7


def lib_path() -> str:
    return os.path.join(_HERE, "lib", "librrm_hip.so")


class Shape(ctypes.Structure):
    """``rrm_shape``"""
    _fields_ = [(k, ctypes.c_int) for k in
                ("kind", "n", "h", "w", "c_in", "c_out", "kh", "kw", "stride", "pad", "groups")]

    @classmethod
    def of(cls, s) -> "Shape":
        return cls(*(int(getattr(s, k)) for k, _ in cls._fields_))


class Stats(ctypes.Structure):
    """``rrm_stats``"""
    _fields_ = [("steps", ctypes.c_uint64), ("delta_steps", ctypes.c_uint64), ("changed_elems", ctypes.c_uint64),
                ("changed_units", ctypes.c_uint64), ("active_tiles", ctypes.c_uint64), ("total_tiles", ctypes.c_uint64),
                ("range_error", ctypes.c_int32), ("tile_positions", ctypes.c_int32),
                ("truncated_elems", ctypes.c_uint64), ("truncated_sumsq", ctypes.c_double)]

    def as_dict(self):
        return {k: (float if k == "truncated_sumsq" else int)(getattr(self, k)) for k, _ in self._fields_}


class StackEntry(ctypes.Structure):
    """``rrm_stack_entry``"""
    _fields_ = [("layer", ctypes.c_void_p), ("shift", ctypes.c_int), ("pool", ctypes.c_int)]


class RRMError(RuntimeError):
    def __init__(self, status: int, msg: str):
        super().__init__(f"rrm status {status}: {msg}")
        self.status = status


_lib = None


def lib():
    """Load the built HIP library; fails loudly when it has not been built."""
    global _lib
    if _lib is None:
        path = lib_path()
        if not os.path.exists(path):
            raise RuntimeError(f"{path} is missing: build it with __graft_entry__.build() "
                               "(python -m paper_1802_09723_amd.build)")
        # torch bundles its own HIP runtime under the same soname; importing it first makes the
        # loader bind this library to that copy, so that streams and pointers are shared.
        import torch  # noqa: F401
        L = ctypes.CDLL(path)
        _assert_single_hip_runtime()
        P, I = ctypes.c_void_p, ctypes.c_int
        L.rrm_layer_create.argtypes = [P, P, ctypes.POINTER(Shape), I, ctypes.POINTER(P)]
        L.rrm_step.argtypes = [P, P, P, P]
        L.rrm_dense.argtypes = [P, P, P, P]
        L.rrm_dense_noalloc.argtypes = [P, P, P, P]
        L.rrm_reset.argtypes = [P, P]
        L.rrm_snapshot.argtypes = [P, ctypes.POINTER(P), ctypes.POINTER(P)]
        L.rrm_read_snapshot.argtypes = [P, P, P, P]
        L.rrm_set_option.argtypes = [P, ctypes.c_char_p, ctypes.c_long]
        L.rrm_get_stats.argtypes = [P, ctypes.POINTER(Stats)]
        L.rrm_get_kernel_times.argtypes = [P, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double),
                                           ctypes.POINTER(I)]
        L.rrm_layer_destroy.argtypes = [P]
        L.rrm_layer_destroy.restype = None
        L.rrm_status_string.argtypes = [I]
        L.rrm_status_string.restype = ctypes.c_char_p
        L.rrm_last_error.restype = ctypes.c_char_p
        L.rrm_aux_relu_requant_pool_i8.argtypes = [P, P, I, I, I, I, I, I, P]
        L.rrm_aux_relu_requant_pool_changed_i8.argtypes = [P, P, I, I, P]
        L.rrm_set_threshold.argtypes = [P, ctypes.c_float]
        L.rrm_step_from_projection.argtypes = [P, P, I, I, P, P]
        L.rrm_stack_step.argtypes = [ctypes.POINTER(StackEntry), I, P, P, P]
        L.rrm_aux_probe_mfma.argtypes = [I, P, I, I, P]
        L.rrm_aux_probe_copy.argtypes = [P, P, ctypes.c_size_t, P]
        L.rrm_aux_probe_mfma.restype = L.rrm_aux_probe_copy.restype = I
        for f in ("rrm_layer_create", "rrm_step", "rrm_dense", "rrm_dense_noalloc", "rrm_reset", "rrm_snapshot", "rrm_read_snapshot", "rrm_set_option",
                  "rrm_get_stats", "rrm_get_kernel_times", "rrm_aux_relu_requant_pool_i8",
                  "rrm_aux_relu_requant_pool_changed_i8", "rrm_set_threshold", "rrm_step_from_projection", "rrm_stack_step"):
            getattr(L, f).restype = I
        _lib = L
    return _lib


def _assert_single_hip_runtime() -> None:
    """Two copies of the HIP runtime in one process do not share streams: refuse that."""
    try:
        with open("/proc/self/maps") as f:
            libs = {line.split()[-1] for line in f if "libamdhip64" in line}
    except OSError:  # pragma: no cover
        return
    if len(libs) > 1:
        raise RuntimeError(f"two HIP runtimes are loaded in this process: {sorted(libs)}")


def _check(st: int, allow_range: bool = False) -> int:
    if st != RRM_OK and not (allow_range and st == RRM_ERR_RANGE):
        raise RRMError(st, lib().rrm_last_error().decode())
    return st


def _stream_ptr(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream or None
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


def _dptr(t) -> Optional[int]:
    """Device pointer of a torch CUDA tensor (or a raw integer pointer)."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("expected a contiguous CUDA tensor")
    return t.data_ptr()


class Layer:
    """One linear layer with its device-resident snapshots (``rrm_layer``)."""

    def __init__(self, shape, dtype: int, weights: np.ndarray, bias: Optional[np.ndarray] = None):
        """``weights`` / ``bias``: host numpy arrays in the boundary formats of ``rrm.h``
        (int8; bf16 patterns as uint16; binary already bit-packed into uint32 words)."""
        self.shape, self.dtype = shape, dtype
        w = np.ascontiguousarray(weights)
        b = None
        if bias is not None:
            b = np.ascontiguousarray(bias, dtype=np.float32 if dtype == BF16 else np.int32)
        cs = Shape.of(shape)
        h = ctypes.c_void_p()
        _check(lib().rrm_layer_create(w.ctypes.data, None if b is None else b.ctypes.data, ctypes.byref(cs), dtype,
                                      ctypes.byref(h)))
        self._h = h

    # -- the C calls --------------------------------------------------------------------------
    def step(self, x_t, y_out=None, stream=None) -> None:
        _check(lib().rrm_step(self._h, _dptr(x_t), _dptr(y_out), _stream_ptr(stream)))

    def step_from_projection(self, producer: "Layer", shift: int, pool: bool, y_out=None, stream=None) -> None:
        """``rrm_step_from_projection``: this layer's input is f(producer's stored projection)."""
        _check(lib().rrm_step_from_projection(self._h, producer._h, int(shift), int(bool(pool)), _dptr(y_out),
                                              _stream_ptr(stream)))

    def dense(self, x, y, stream=None) -> None:
        _check(lib().rrm_dense(self._h, _dptr(x), _dptr(y), _stream_ptr(stream)))

    def dense_noalloc(self, x, y, stream=None) -> None:
        _check(lib().rrm_dense_noalloc(self._h, _dptr(x), _dptr(y), _stream_ptr(stream)))

    def reset(self, stream=None) -> None:
        _check(lib().rrm_reset(self._h, _stream_ptr(stream)))

    def set_threshold(self, epsilon: float) -> None:
        """Truncation threshold of a bf16 layer's input difference (``rrm_set_threshold``)."""
        _check(lib().rrm_set_threshold(self._h, float(epsilon)))

    def relu_requant_pool_changed(self, out, shift, pool, stream=None) -> None:
        """Harness nonlinearity on the stored projection, recomputing only what the last step changed
        (``rrm_aux_relu_requant_pool_changed_i8``); ``out`` must hold the previous call's result."""
        _check(lib().rrm_aux_relu_requant_pool_changed_i8(self._h, _dptr(out), int(shift), int(bool(pool)),
                                                           _stream_ptr(stream)))

    def snapshot_ptrs(self):
        xs, ys = ctypes.c_void_p(), ctypes.c_void_p()
        _check(lib().rrm_snapshot(self._h, ctypes.byref(xs), ctypes.byref(ys)))
        return xs.value, ys.value

    def set_option(self, key: str, value: int) -> None:
        _check(lib().rrm_set_option(self._h, key.encode(), int(value)))

    def stats(self, allow_range_error: bool = False) -> dict:
        s = Stats()
        _check(lib().rrm_get_stats(self._h, ctypes.byref(s)), allow_range=allow_range_error)
        return s.as_dict()

    def kernel_times(self):
        """(scan_us, compute_us, steps) summed since "profile" was switched on / last read."""
        a, c, n = ctypes.c_double(), ctypes.c_double(), ctypes.c_int()
        _check(lib().rrm_get_kernel_times(self._h, ctypes.byref(a), ctypes.byref(c), ctypes.byref(n)))
        return a.value, c.value, n.value

    def destroy(self) -> None:
        if getattr(self, "_h", None):
            lib().rrm_layer_destroy(self._h)
            self._h = None

    def __del__(self):  # pragma: no cover
        try:
            self.destroy()
        except Exception:
            pass

    # -- conveniences for tests and the bench (copies, not part of the hot path) ---------------
    @property
    def y_shape(self):
        s = self.shape
        if s.kind == FC:
            return (s.n, s.c_out)
        return (s.n, (s.h + 2 * s.pad - s.kh) // s.stride + 1, (s.w + 2 * s.pad - s.kw) // s.stride + 1, s.c_out)

    def y_snapshot(self):
        """Copy of the stored projection as a torch tensor (rrm_read_snapshot; synchronises)."""
        import torch
        out = torch.empty(self.y_shape, dtype=torch.float32 if self.dtype == BF16 else torch.int32, device="cuda")
        _check(lib().rrm_read_snapshot(self._h, None, out.data_ptr(), _stream_ptr(None)))
        torch.cuda.synchronize()
        return out

    def x_snapshot_bytes(self):
        """Copy of the stored input as a uint8 torch tensor (rrm_read_snapshot; synchronises)."""
        import torch
        s = self.shape
        per = {I8: 1, BF16: 2}.get(self.dtype)
        n_el = s.n * s.c_in if s.kind == FC else s.n * s.h * s.w * s.c_in
        nbytes = n_el * per if per else n_el // 8
        out = torch.empty((nbytes,), dtype=torch.uint8, device="cuda")
        _check(lib().rrm_read_snapshot(self._h, out.data_ptr(), None, _stream_ptr(None)))
        torch.cuda.synchronize()
        return out


def stack_step(layers, shifts, pools, x_t, f_out=None, stream=None) -> None:
    """``rrm_stack_step``: one frame through a stack of int8 conv layers with the fused nonlinearity."""
    arr = (StackEntry * len(layers))(*[StackEntry(L._h, int(s), int(bool(p))) for L, s, p in zip(layers, shifts, pools)])
    _check(lib().rrm_stack_step(arr, len(layers), _dptr(x_t), _dptr(f_out), _stream_ptr(stream)))


def probe_mfma(dtype: int, sink, iters: int, workgroups: int, stream=None) -> None:
    """``rrm_aux_probe_mfma``: register-resident matrix-core loop (a measurement probe)."""
    _check(lib().rrm_aux_probe_mfma(int(dtype), _dptr(sink), int(iters), int(workgroups), _stream_ptr(stream)))


def probe_copy(dst, src, nbytes: int, stream=None) -> None:
    """``rrm_aux_probe_copy``: streaming copy of `nbytes` bytes (a measurement probe)."""
    _check(lib().rrm_aux_probe_copy(_dptr(dst), _dptr(src), int(nbytes), _stream_ptr(stream)))


def relu_requant_pool_i8(y, out, n, h, w, c, shift, pool, stream=None) -> None:
    """Harness nonlinearity between int8 conv layers (``rrm_aux_relu_requant_pool_i8``)."""
    _check(lib().rrm_aux_relu_requant_pool_i8(_dptr(y), _dptr(out), n, h, w, c, int(shift), int(bool(pool)),
                                               _stream_ptr(stream)))
