"""ctypes front-end of the CPU oracle (`adascale_oracle.c`).  TEST INFRASTRUCTURE ONLY:
imported by the tests, the smoke check and the benchmark's CPU-baseline leg, never by the
product path.  Holds marshalling only; the arithmetic is in the C file.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Sequence

import numpy as np

from . import build as _build

F32, BF16 = 0, 1
LAGGED_R, EST_M1M2 = 1, 2


class State(C.Structure):
    _fields_ = [("step", C.c_int64), ("tau", C.c_double), ("r", C.c_double), ("lr_eff", C.c_double),
                ("sum_sq", C.c_double), ("sq_mean", C.c_double), ("sigma2_hat", C.c_double),
                ("mu2_hat", C.c_double), ("sigma2_bar", C.c_double), ("mu2_bar", C.c_double),
                ("done", C.c_int32)]

    def as_dict(self) -> dict:
        return {n: getattr(self, n) for n, _ in self._fields_}


_libs: dict = {}


def _lib(openmp: bool) -> C.CDLL:
    key = bool(openmp)
    if key not in _libs:
        _build.build(force=False)
        lib = C.CDLL(_build.LIB_OMP if openmp else _build.LIB)
        lib.oracle_create.restype = C.c_void_p
        lib.oracle_create.argtypes = [C.c_int, C.c_int, C.c_double, C.c_double, C.c_double, C.c_double,
                                      C.c_void_p, C.c_int64, C.c_uint32]
        lib.oracle_destroy.argtypes = [C.c_void_p]
        lib.oracle_get_state.argtypes = [C.c_void_p, C.POINTER(State)]
        lib.oracle_set_state.argtypes = [C.c_void_p, C.c_int64, C.c_double, C.c_double, C.c_double, C.c_double]
        lib.oracle_set_scale.argtypes = [C.c_void_p, C.c_int, C.c_double]
        lib.oracle_begin_step.argtypes = [C.c_void_p]
        lib.oracle_accumulate.argtypes = [C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p]
        lib.oracle_gain.argtypes = [C.c_void_p]
        lib.oracle_apply.argtypes = [C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p]
        lib.oracle_advance.argtypes = [C.c_void_p]
        lib.oracle_num_threads.restype = C.c_int
        _libs[key] = lib
    return _libs[key]


def _as_grad_array(a, dtype: int) -> np.ndarray:
    """Contiguous numpy array holding the gradient's bit pattern (bf16 as uint16)."""
    want = np.float32 if dtype == F32 else np.uint16
    a = np.ascontiguousarray(a)
    if a.dtype != want:
        raise TypeError(f"gradient array has dtype {a.dtype}, expected {want}")
    return a.reshape(-1)


class Oracle:
    """One AdaScale training state on the CPU; w and v live in fp64 numpy arrays owned by the caller."""

    def __init__(self, S: int, lr_table: Sequence[float], momentum: float = 0.9, weight_decay: float = 0.0,
                 theta: float = -1.0, eps: float = 1e-6, grad_dtype: int = F32, flags: int = 0,
                 openmp: bool = False):
        self._l = _lib(openmp)
        lr = np.ascontiguousarray(lr_table, dtype=np.float32)
        self._h = self._l.oracle_create(S, grad_dtype, momentum, weight_decay, theta, eps,
                                        lr.ctypes.data, lr.size, flags)
        if not self._h:
            raise ValueError("oracle_create rejected the configuration")
        self.S, self.grad_dtype = S, grad_dtype

    def __del__(self):
        if getattr(self, "_h", None):
            self._l.oracle_destroy(self._h)
            self._h = None

    @property
    def threads(self) -> int:
        return int(self._l.oracle_num_threads())

    def state(self) -> State:
        s = State()
        self._l.oracle_get_state(self._h, C.byref(s))
        return s

    def set_state(self, step: int, tau: float, sigma2_bar: float, mu2_bar: float, r: float = 1.0) -> None:
        self._l.oracle_set_state(self._h, step, tau, sigma2_bar, mu2_bar, r)

    def set_scale(self, S: int, theta: float = -1.0) -> None:
        self._l.oracle_set_scale(self._h, S, theta)
        self.S = S

    def step(self, w: List[np.ndarray], v: List[np.ndarray], grads: List[List[np.ndarray]]) -> State:
        """One iteration.  w[k], v[k]: fp64 arrays updated in place; grads[i][k]: replica i, tensor k
        (float32, or uint16 holding bf16 bits).  Returns the state after the iteration."""
        if len(grads) != self.S:
            raise ValueError("need S gradient lists")
        l, h = self._l, self._h
        gbars = []
        l.oracle_begin_step(h)
        for k in range(len(w)):
            n = w[k].size
            gk = [_as_grad_array(grads[i][k], self.grad_dtype) for i in range(self.S)]
            if any(a.size != n for a in gk):
                raise ValueError("gradient / parameter size mismatch")
            ptrs = (C.c_void_p * self.S)(*[a.ctypes.data for a in gk])
            gb = np.empty(n, dtype=np.float64)
            l.oracle_accumulate(h, n, ptrs, gb.ctypes.data)
            gbars.append(gb)
        l.oracle_gain(h)
        for k in range(len(w)):
            for a in (w[k], v[k]):
                if a.dtype != np.float64 or not a.flags.c_contiguous:
                    raise TypeError("w and v must be contiguous float64 arrays")
            l.oracle_apply(h, w[k].size, w[k].ctypes.data, v[k].ctypes.data, gbars[k].ctypes.data)
        l.oracle_advance(h)
        self.last_gbar = gbars
        return self.state()
