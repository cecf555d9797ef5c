"""ctypes binding of include/adascale.h and include/adascale_diag.h: same entry points, argument
marshalling only.

PyTorch appears here only as the owner of device memory and streams: tensors are passed
down as raw device pointers and the current stream as a raw hipStream_t.  There is no
fallback path: if the HIP library is missing, loading fails with an error.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

import numpy as np

F32, BF16 = 0, 1
LAGGED_R, EST_NORM_RATIO, NO_POINTER_CHECK, COOPERATIVE_LAUNCH = 1, 2, 4, 8
_CODES = {0: "OK", 1: "EINVAL", 2: "ENOMEM", 3: "EHIP", 4: "ESTATE"}

FORCE_NONE, FORCE_GENERAL, FORCE_FUSED, FORCE_STREAMING = 0, 1, 2, 3

# adascale.h: the interface of the method
EXPORTS = ["adascale_init", "adascale_step", "adascale_get_state", "adascale_set_state",
           "adascale_set_scale", "adascale_destroy", "adascale_last_error", "adascale_step_flat"]
# adascale_diag.h: diagnostics, instrumentation, test knobs
EXPORTS_DIAG = ["adascale_step_bytes", "adascale_step_moved_bytes", "adascale_profile_begin", "adascale_profile_end",
                "adascale_uses_fused_step", "adascale_step_path", "adascale_kernel_shape", "adascale_plan",
                "adascale_init_tuned", "adascale_fail_next_barrier"]


class AdaScaleError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"adascale: {_CODES.get(code, code)}: {msg}")
        self.code = code


class Config(C.Structure):
    _fields_ = [("S", C.c_int32), ("n_tensors", C.c_int32), ("numel", C.POINTER(C.c_int64)),
                ("grad_dtype", C.c_int32), ("momentum", C.c_double), ("weight_decay", C.c_double),
                ("theta", C.c_double), ("eps", C.c_double), ("lr_table", C.POINTER(C.c_float)),
                ("lr_table_len", C.c_int64), ("device", C.c_int32), ("flags", C.c_uint32)]


class State(C.Structure):
    _fields_ = [("step", C.c_int64), ("tau", C.c_double), ("r", C.c_double), ("lr_eff", C.c_double),
                ("sum_sq", C.c_double), ("sq_mean", C.c_double), ("sigma2_hat", C.c_double),
                ("mu2_hat", C.c_double), ("sigma2_bar", C.c_double), ("mu2_bar", C.c_double),
                ("done", C.c_int32)]

    def as_dict(self) -> dict:
        return {n: getattr(self, n) for n, _ in self._fields_}


class FlatStep(C.Structure):
    """adascale_flat_step: the argument record of adascale_step_flat."""
    _fields_ = [("S", C.c_int32), ("grad_dtype", C.c_int32), ("numel", C.c_int64), ("momentum", C.c_double),
                ("weight_decay", C.c_double), ("theta", C.c_double), ("eps", C.c_double), ("flags", C.c_uint32),
                ("device", C.c_int32), ("w", C.c_void_p), ("mom", C.c_void_p), ("grads", C.POINTER(C.c_void_p)),
                ("lr_table", C.c_void_p), ("lr_table_len", C.c_int64), ("state", C.c_void_p)]


FLAT_MAX_SCALE = 64
FLAT_MAX_NUMEL = (1 << 40) - 1


class Tuning(C.Structure):
    """adascale_tuning: knobs for tests and measurements; all zero = the library's own choices."""
    _fields_ = [("force_path", C.c_int32), ("fused_max_grid", C.c_int32), ("fused_min_percent", C.c_int32),
                ("stream_via_scratch", C.c_int32), ("barrier_spin_limit", C.c_int64),
                ("burst_tiles", C.c_int32), ("burst_window_ticks", C.c_int32)]


class PlanInfo(C.Structure):
    _fields_ = [("full_tiles", C.c_int64), ("ragged_tiles", C.c_int64), ("path", C.c_int32),
                ("fused_grid", C.c_int32), ("tiles_per_workgroup", C.c_int32), ("register_tiles", C.c_int32),
                ("lds_tiles", C.c_int32), ("on_chip_percent", C.c_int32), ("stream_grid", C.c_int32)]

    def as_dict(self) -> dict:
        return {n: getattr(self, n) for n, _ in self._fields_}


def library_path() -> str:
    return os.path.join(os.path.dirname(os.path.abspath(__file__)), "libadascale.so")


_lib: Optional[C.CDLL] = None


def load_library() -> C.CDLL:
    """Load libadascale.so; raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is None:
        path = library_path()
        if not os.path.exists(path):
            raise ImportError(f"{path} is missing: build it with `python -m paper_2007_05105_amd.build` "
                              "(hipcc, gfx950); there is no fallback implementation")
        lib = C.CDLL(path)
        lib.adascale_init.argtypes = [C.POINTER(Config), C.POINTER(C.c_void_p)]
        lib.adascale_init.restype = C.c_int
        lib.adascale_step.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        lib.adascale_step.restype = C.c_int
        lib.adascale_get_state.argtypes = [C.c_void_p, C.POINTER(State), C.c_void_p]
        lib.adascale_get_state.restype = C.c_int
        lib.adascale_set_state.argtypes = [C.c_void_p, C.c_int64, C.c_double, C.c_double, C.c_double, C.c_void_p]
        lib.adascale_set_state.restype = C.c_int
        lib.adascale_set_scale.argtypes = [C.c_void_p, C.c_int32, C.c_double]
        lib.adascale_set_scale.restype = C.c_int
        lib.adascale_destroy.argtypes = [C.c_void_p]
        lib.adascale_destroy.restype = None
        lib.adascale_last_error.argtypes = [C.c_void_p]
        lib.adascale_last_error.restype = C.c_char_p
        lib.adascale_step_bytes.argtypes = [C.c_void_p]
        lib.adascale_step_bytes.restype = C.c_int64
        lib.adascale_profile_begin.argtypes = [C.c_void_p, C.c_int32]
        lib.adascale_profile_begin.restype = C.c_int
        lib.adascale_profile_end.argtypes = [C.c_void_p, C.POINTER(C.c_double), C.POINTER(C.c_int32)]
        lib.adascale_profile_end.restype = C.c_int
        lib.adascale_uses_fused_step.argtypes = [C.c_void_p]
        lib.adascale_uses_fused_step.restype = C.c_int
        lib.adascale_step_path.argtypes = [C.c_void_p]
        lib.adascale_step_path.restype = C.c_int
        lib.adascale_kernel_shape.argtypes = [C.c_int32, C.c_int32, C.POINTER(C.c_int32)]
        lib.adascale_kernel_shape.restype = C.c_int
        lib.adascale_plan.argtypes = [C.POINTER(Config), C.POINTER(Tuning), C.c_int32, C.c_int64, C.POINTER(PlanInfo)]
        lib.adascale_plan.restype = C.c_int
        lib.adascale_step_flat.argtypes = [C.POINTER(FlatStep), C.c_void_p]
        lib.adascale_step_flat.restype = C.c_int
        lib.adascale_init_tuned.argtypes = [C.POINTER(Config), C.POINTER(Tuning), C.POINTER(C.c_void_p)]
        lib.adascale_init_tuned.restype = C.c_int
        lib.adascale_fail_next_barrier.argtypes = [C.c_void_p]
        lib.adascale_fail_next_barrier.restype = C.c_int
        lib.adascale_step_moved_bytes.argtypes = [C.c_void_p]
        lib.adascale_step_moved_bytes.restype = C.c_int64
        _lib = lib
    return _lib


def kernel_shape(grad_dtype: int, S: int):
    """adascale_kernel_shape: (mask, (loads per half-group, half-groups, padded replica slots))."""
    shape = (C.c_int32 * 3)()
    mask = load_library().adascale_kernel_shape(grad_dtype, S, shape)
    return mask, tuple(shape)


def plan(numel: Sequence[int], S: int, grad_dtype: int = F32, flags: int = 0, compute_units: int = 256,
         lds_bytes: int = 160 * 1024, tuning: Optional[Tuning] = None) -> dict:
    """adascale_plan: what adascale_init would decide for this parameter list on a device with the
    given compute units and LDS per workgroup (defaults: MI355X); needs no device."""
    lib = load_library()
    n = (C.c_int64 * len(numel))(*[int(x) for x in numel])
    cfg = Config(S, len(numel), n, grad_dtype, 0.0, 0.0, -1.0, 0.0, None, 0, 0, flags)
    info = PlanInfo()
    rc = lib.adascale_plan(C.byref(cfg), C.byref(tuning) if tuning is not None else None, compute_units, lds_bytes,
                           C.byref(info))
    if rc != 0:
        raise AdaScaleError(rc, lib.adascale_last_error(None).decode())
    d = info.as_dict()
    d["path"] = ("general", "fused", "streaming")[d["path"]]
    return d


def step_flat(w, mom, grads: Sequence, lr_table_dev, state_dev, momentum: float = 0.9, weight_decay: float = 0.0,
              theta: float = -1.0, eps: float = 1e-6, grad_dtype: int = F32, flags: int = 0, device: int = 0,
              stream=None, numel: Optional[int] = None) -> None:
    """adascale_step_flat: one iteration on one flat tensor with nothing allocated.  w, mom: fp32
    device tensors; grads: S device tensors; lr_table_dev: fp32 device tensor; state_dev: device
    tensor of at least sizeof(adascale_state) bytes holding the state record (zeros = fresh run)."""
    lib = load_library()
    n = int(w.numel()) if numel is None else int(numel)
    ptrs = (C.c_void_p * len(grads))(*[int(g.data_ptr()) for g in grads])
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    args = FlatStep(len(grads), grad_dtype, n, momentum, weight_decay, theta, eps, flags, device,
                    int(w.data_ptr()), int(mom.data_ptr()), ptrs, int(lr_table_dev.data_ptr()),
                    int(lr_table_dev.numel()), int(state_dev.data_ptr()))
    rc = lib.adascale_step_flat(C.byref(args), C.c_void_p(int(getattr(stream, "cuda_stream", stream))))
    if rc != 0:
        raise AdaScaleError(rc, lib.adascale_last_error(None).decode())


def _ptr_array(tensors: Sequence) -> "C.Array":
    return (C.c_void_p * len(tensors))(*[int(t.data_ptr()) if t is not None else 0 for t in tensors])


class AdaScale:
    """adascale_init / adascale_step / adascale_get_state on lists of torch tensors."""

    def __init__(self, numel: Sequence[int], S: int, lr_table, momentum: float = 0.9,
                 weight_decay: float = 0.0, theta: float = -1.0, eps: float = 1e-6,
                 grad_dtype: int = F32, device: int = 0, flags: int = 0, tuning: Optional[Tuning] = None):
        self._lib = load_library()
        self._h = C.c_void_p()
        n = (C.c_int64 * len(numel))(*[int(x) for x in numel])
        lr = np.ascontiguousarray(lr_table, dtype=np.float32)
        cfg = Config(S, len(numel), n, grad_dtype, momentum, weight_decay, theta, eps,
                     lr.ctypes.data_as(C.POINTER(C.c_float)), lr.size, device, flags)
        if tuning is None:
            rc = self._lib.adascale_init(C.byref(cfg), C.byref(self._h))
        else:
            rc = self._lib.adascale_init_tuned(C.byref(cfg), C.byref(tuning), C.byref(self._h))
        if rc != 0:
            raise AdaScaleError(rc, self._lib.adascale_last_error(None).decode())
        self.S, self.numel, self.grad_dtype, self.device = S, list(numel), grad_dtype, device
        self._cache_key = None
        self._cache = None

    def _check(self, rc: int) -> None:
        if rc != 0:
            raise AdaScaleError(rc, self._lib.adascale_last_error(self._h).decode())

    @staticmethod
    def _stream(stream) -> int:
        if stream is None:
            import torch
            return int(torch.cuda.current_stream().cuda_stream)
        return int(getattr(stream, "cuda_stream", stream))

    def step(self, w: List, mom: List, grads: List[List], stream=None) -> None:
        """One iteration: w[k], mom[k] fp32 device tensors updated in place; grads[i][k] is
        replica i's gradient of tensor k.  Asynchronous on `stream` (default: torch's current).
        The pointer arrays are rebuilt only when the tensor objects differ from the last call's;
        after giving one of them new storage in place (`t.data = ...`, `t.set_()`), call
        `invalidate()`."""
        if len(grads) != self.S or len(w) != len(self.numel) or len(mom) != len(self.numel):
            raise ValueError("need S gradient lists and N parameter / momentum tensors")
        key = (tuple(id(t) for t in w), tuple(id(t) for t in mom), tuple(id(t) for g in grads for t in g))
        if key != self._cache_key:
            for k, n in enumerate(self.numel):
                for t in [w[k], mom[k]] + [g[k] for g in grads]:
                    if t.numel() != n or not t.is_contiguous():
                        raise ValueError(f"tensor {k}: expected {n} contiguous elements")
            flat = [t for g in grads for t in g]
            self._cache = (_ptr_array(w), _ptr_array(mom), _ptr_array(flat), (list(w), list(mom), flat))
            self._cache_key = key
        pw, pm, pg, _ = self._cache
        self._check(self._lib.adascale_step(self._h, pw, pm, pg, C.c_void_p(self._stream(stream))))

    def invalidate(self) -> None:
        """Forget the cached pointer arrays (see `step`)."""
        self._cache_key = None
        self._cache = None

    def step_raw(self, pw, pm, pg, stream: int) -> int:
        """adascale_step on prebuilt ctypes pointer arrays; returns the status code."""
        return self._lib.adascale_step(self._h, pw, pm, pg, C.c_void_p(stream))

    def get_state(self, stream=None) -> State:
        st = State()
        self._check(self._lib.adascale_get_state(self._h, C.byref(st), C.c_void_p(self._stream(stream))))
        return st

    def set_state(self, step: int, tau: float, sigma2_bar: float, mu2_bar: float, stream=None) -> None:
        self._check(self._lib.adascale_set_state(self._h, step, tau, sigma2_bar, mu2_bar,
                                                 C.c_void_p(self._stream(stream))))

    def set_scale(self, S: int, theta: float = -1.0) -> None:
        self._check(self._lib.adascale_set_scale(self._h, S, theta))
        self.S = S
        self._cache_key = None

    def profile_begin(self, max_steps: int) -> None:
        self._check(self._lib.adascale_profile_begin(self._h, max_steps))

    def profile_end(self):
        """(ms_reduce, ms_scalars, ms_update) averaged over the recorded steps, and their number."""
        ms = (C.c_double * 3)()
        n = C.c_int32()
        self._check(self._lib.adascale_profile_end(self._h, ms, C.byref(n)))
        return (ms[0], ms[1], ms[2]), n.value

    def uses_fused_step(self) -> bool:
        return bool(self._lib.adascale_uses_fused_step(self._h))

    def step_path(self) -> str:
        return ("general", "fused", "streaming")[self._lib.adascale_step_path(self._h)]

    def step_bytes(self) -> int:
        return int(self._lib.adascale_step_bytes(self._h))

    def step_moved_bytes(self) -> int:
        return int(self._lib.adascale_step_moved_bytes(self._h))

    def fail_next_barrier(self) -> None:
        self._check(self._lib.adascale_fail_next_barrier(self._h))

    def last_error(self) -> str:
        return self._lib.adascale_last_error(self._h).decode()

    def close(self) -> None:
        if getattr(self, "_h", None) and self._h.value:
            self._lib.adascale_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
