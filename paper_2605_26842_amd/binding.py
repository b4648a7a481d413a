"""ctypes binding of libmona.so: the same entry points as include/mona.h, plus a
small convenience class that keeps the arena tensor alive.

Argument marshalling only -- every arithmetic step of the optimizer runs in the
HIP kernels behind the C ABI.  PyTorch is used for device memory (the arena,
the callers' parameter and gradient tensors) and for the current stream.
There is no fallback: if the shared library is missing, loading fails.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmona.so")

MONA_OK, MONA_EINVAL, MONA_ESHAPE, MONA_ENOMEM, MONA_EHIP, MONA_EUNSUPPORTED = 0, -1, -2, -3, -4, -5
MONA_F32, MONA_BF16 = 0, 1
MONA_FLAG_FIRST_DIFF_ZERO, MONA_FLAG_KEEP_O, MONA_FLAG_MUON_ONLY = 0x1, 0x2, 0x4
MONA_VIEW_G_PREV, MONA_VIEW_A, MONA_VIEW_M, MONA_VIEW_NORM, MONA_VIEW_O, MONA_VIEW_C = 0, 1, 2, 3, 4, 5
MONA_ACCEL_TWO_BUFFER, MONA_ACCEL_ONE_BUFFER, MONA_ACCEL_CALLER_SLOT = 0, 1, 2
MONA_STATUS_ZERO_NORM, MONA_STATUS_NONFINITE, MONA_STATUS_RESCALED = 0x1, 0x2, 0x4
MONA_NS_SCHEDULE_AUTO, MONA_NS_SCHEDULE_LITERAL, MONA_NS_SCHEDULE_FUSED, MONA_NS_SCHEDULE_PAIRS = 0, 1, 2, 3
MONA_OVERLAP_OFF, MONA_OVERLAP_LATE_GROUP = 0, 1

EXPORTED = (
    "mona_state_size", "mona_init_state", "mona_step", "mona_step_streaming", "mona_step_noalloc", "mona_free_state",
    "mona_state_view",
    "mona_state_export_size", "mona_state_export", "mona_state_import", "mona_state_step_count",
    "mona_state_status", "mona_set_profiling", "mona_last_step_times", "mona_mean_step_times", "mona_last_step_launches",
    "mona_plan_info", "mona_last_error", "mona_version",
    "mona_adamw_state_size", "mona_adamw_init_state", "mona_adamw_step", "mona_adamw_free_state",
    "mona_adamw_state_view", "mona_adamw_state_export_size", "mona_adamw_state_export",
    "mona_adamw_state_import", "mona_adamw_state_step_count",
)
MONA_ADAMW_VIEW_M, MONA_ADAMW_VIEW_V = 0, 1


class mona_vector(C.Structure):
    _fields_ = [("w", C.c_void_p), ("g", C.c_void_p), ("n", C.c_int64), ("w_dtype", C.c_int32), ("g_dtype", C.c_int32)]


class mona_adamw_hparams(C.Structure):
    _fields_ = [("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float), ("eps", C.c_float),
                ("weight_decay", C.c_float)]


class mona_matrix(C.Structure):
    _fields_ = [("w", C.c_void_p), ("g", C.c_void_p), ("m", C.c_int32), ("n", C.c_int32),
                ("w_dtype", C.c_int32), ("g_dtype", C.c_int32)]


class mona_hparams(C.Structure):
    _fields_ = [("lr", C.c_float), ("momentum", C.c_float), ("beta_a", C.c_float), ("alpha", C.c_float),
                ("weight_decay", C.c_float), ("ns_steps", C.c_int32), ("ns_a", C.c_float),
                ("ns_b", C.c_float), ("ns_c", C.c_float), ("ns_eps", C.c_float),
                ("gamma_coeff", C.c_float), ("flags", C.c_uint32)]


class mona_options(C.Structure):
    _fields_ = [("ns_precision", C.c_int32), ("state_dtype", C.c_int32), ("accel_form", C.c_int32),
                ("max_streams", C.c_int32), ("ns_schedule", C.c_int32), ("overlap", C.c_int32),
                ("reserved", C.c_int32 * 2)]


class mona_view(C.Structure):
    _fields_ = [("ptr", C.c_void_p), ("rows", C.c_int32), ("cols", C.c_int32), ("ld", C.c_int32),
                ("dtype", C.c_int32)]


class mona_launch_time(C.Structure):
    _fields_ = [("kind", C.c_int32), ("group", C.c_int32), ("iter", C.c_int32), ("tile", C.c_int32),
                ("m", C.c_int32), ("n", C.c_int32), ("count", C.c_int32), ("ms", C.c_float),
                ("flops", C.c_double)]


class MonaError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"libmona error {code}: {message}")
        self.code = code


_lib: Optional[C.CDLL] = None


def load_library(path: Optional[str] = None) -> C.CDLL:
    """dlopen libmona.so and declare the prototypes.  Raises if the library is absent."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    p = path or LIB_PATH
    if not os.path.exists(p):
        raise FileNotFoundError(
            f"{p} not found: build it first (python -c 'import __graft_entry__ as g; g.build()' "
            f"or python paper_2605_26842_amd/build.py); there is no fallback path")
    lib = C.CDLL(p)
    vp, i32, i64, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t
    P = C.POINTER
    lib.mona_state_size.argtypes = [P(mona_matrix), i32, P(mona_options), P(sz)]
    lib.mona_init_state.argtypes = [P(mona_matrix), i32, P(mona_options), vp, sz, vp, P(vp)]
    lib.mona_step.argtypes = [vp, P(mona_matrix), i32, P(mona_hparams), vp]
    lib.mona_step_streaming.argtypes = [vp, P(mona_matrix), P(vp), i32, P(mona_hparams), vp]
    lib.mona_step_noalloc.argtypes = [P(mona_matrix), P(mona_options), vp, vp, vp, P(mona_hparams), i64, vp]
    lib.mona_free_state.argtypes = [vp]
    lib.mona_state_view.argtypes = [vp, i32, i32, P(mona_view)]
    lib.mona_state_export_size.argtypes = [vp, P(sz)]
    lib.mona_state_export.argtypes = [vp, vp, sz, vp]
    lib.mona_state_import.argtypes = [vp, vp, sz, i64, vp]
    lib.mona_state_step_count.argtypes = [vp, P(i64)]
    lib.mona_state_status.argtypes = [vp, P(C.c_uint32), i32, vp]
    lib.mona_adamw_state_size.argtypes = [P(mona_vector), i32, P(sz)]
    lib.mona_adamw_init_state.argtypes = [P(mona_vector), i32, vp, sz, vp, P(vp)]
    lib.mona_adamw_step.argtypes = [vp, P(mona_vector), i32, P(mona_adamw_hparams), vp]
    lib.mona_adamw_free_state.argtypes = [vp]
    lib.mona_adamw_state_view.argtypes = [vp, i32, i32, P(vp), P(i64)]
    lib.mona_adamw_state_export_size.argtypes = [vp, P(sz)]
    lib.mona_adamw_state_export.argtypes = [vp, vp, sz, vp]
    lib.mona_adamw_state_import.argtypes = [vp, vp, sz, i64, vp]
    lib.mona_adamw_state_step_count.argtypes = [vp, P(i64)]
    lib.mona_set_profiling.argtypes = [vp, i32]
    lib.mona_last_step_times.argtypes = [vp, P(C.c_float)]
    lib.mona_mean_step_times.argtypes = [vp, P(C.c_float), P(i32)]
    lib.mona_last_step_launches.argtypes = [vp, P(mona_launch_time), i32, P(i32)]
    lib.mona_plan_info.argtypes = [vp, i32, P(i64), P(C.c_double), P(C.c_double)]
    for name in EXPORTED:
        getattr(lib, name).restype = C.c_int
    lib.mona_last_error.restype = C.c_char_p
    lib.mona_last_error.argtypes = []
    lib.mona_version.restype = C.c_char_p
    lib.mona_version.argtypes = []
    if path is None:
        _lib = lib
    return lib


def _check(rc: int) -> None:
    if rc != MONA_OK:
        raise MonaError(rc, load_library().mona_last_error().decode())


def _dtype_code(t: torch.dtype) -> int:
    if t == torch.float32:
        return MONA_F32
    if t == torch.bfloat16:
        return MONA_BF16
    raise TypeError(f"unsupported dtype {t}: parameters and gradients must be float32 or bfloat16")


def make_hparams(hp) -> mona_hparams:
    """From any object with the fields of workloads.HParams."""
    return mona_hparams(hp.lr, hp.momentum, hp.beta_a, hp.alpha, hp.weight_decay, hp.ns_steps,
                        hp.ns_a, hp.ns_b, hp.ns_c, hp.ns_eps, hp.gamma_coeff, hp.flags)


def make_matrices(weights: Sequence[torch.Tensor], grads: Optional[Sequence[torch.Tensor]] = None,
                  g_dtype: torch.dtype = torch.float32):
    """Array of mona_matrix descriptors for 2-D contiguous tensors."""
    n = len(weights)
    arr = (mona_matrix * n)()
    for i, w in enumerate(weights):
        if w.dim() != 2 or not w.is_contiguous():
            raise ValueError(f"matrix {i}: parameters must be contiguous 2-D tensors")
        g = None if grads is None else grads[i]
        if g is not None and (g.shape != w.shape or not g.is_contiguous()):
            raise ValueError(f"matrix {i}: gradient must be contiguous and shaped like the parameter")
        arr[i].w = w.data_ptr()
        arr[i].g = 0 if g is None else g.data_ptr()
        arr[i].m, arr[i].n = int(w.shape[0]), int(w.shape[1])
        arr[i].w_dtype = _dtype_code(w.dtype)
        arr[i].g_dtype = _dtype_code(g.dtype if g is not None else g_dtype)
    return arr


# ---- thin functional layer: same names as the C entry points -------------------------------
def mona_state_size(mats, count: int, opts: Optional[mona_options] = None) -> int:
    out = C.c_size_t(0)
    _check(load_library().mona_state_size(mats, count, C.byref(opts) if opts is not None else None, C.byref(out)))
    return out.value


def mona_init_state(mats, count: int, opts: Optional[mona_options], arena: torch.Tensor, stream: int) -> int:
    handle = C.c_void_p(0)
    _check(load_library().mona_init_state(mats, count, C.byref(opts) if opts is not None else None,
                                          arena.data_ptr(), arena.numel() * arena.element_size(), stream,
                                          C.byref(handle)))
    return handle.value


def mona_step(state: int, mats, count: int, hp: mona_hparams, stream: int) -> None:
    _check(load_library().mona_step(state, mats, count, C.byref(hp), stream))


def mona_step_streaming(state: int, mats, slots, count: int, hp: mona_hparams, stream: int) -> None:
    _check(load_library().mona_step_streaming(state, mats, slots, count, C.byref(hp), stream))


def mona_step_noalloc(mat, opts: Optional[mona_options], g_prev: int, acc: int, mom: int, hp: mona_hparams, k: int,
                      stream: int) -> None:
    """One step of one matrix with caller-kept state arrays (device addresses) and the library's static workspace."""
    _check(load_library().mona_step_noalloc(mat, C.byref(opts) if opts is not None else None, g_prev, acc, mom,
                                            C.byref(hp), k, stream))


def mona_free_state(state: int) -> None:
    _check(load_library().mona_free_state(state))


def mona_state_view(state: int, i: int, kind: int) -> mona_view:
    v = mona_view()
    _check(load_library().mona_state_view(state, i, kind, C.byref(v)))
    return v


class MonaOptimizer:
    """Owns the arena and the state handle for a fixed list of parameter matrices."""

    def __init__(self, weights: Sequence[torch.Tensor], ns_precision: int = 0,
                 state_dtype: torch.dtype = torch.float32, g_dtype: torch.dtype = torch.float32,
                 accel_form: int = MONA_ACCEL_TWO_BUFFER, max_streams: int = 0,
                 ns_schedule: int = MONA_NS_SCHEDULE_AUTO, overlap: int = MONA_OVERLAP_OFF):
        if not weights:
            raise ValueError("need at least one matrix")
        self.lib = load_library()
        self.device = weights[0].device
        if self.device.type != "cuda":
            raise RuntimeError("MonaOptimizer needs parameters on a GPU (no CPU path exists)")
        self.weights = list(weights)
        self.count = len(self.weights)
        self.g_dtype = g_dtype
        self.opts = mona_options(ns_precision, _dtype_code(state_dtype), accel_form, max_streams, ns_schedule,
                                 overlap, (C.c_int32 * 2)())
        self.accel_form = accel_form
        self.ns_precision = ns_precision
        self.state_dtype = state_dtype
        shapes_only = make_matrices(self.weights, None, g_dtype)
        self.arena_bytes = mona_state_size(shapes_only, self.count, self.opts)
        self.arena = torch.empty(self.arena_bytes, dtype=torch.uint8, device=self.device)
        with torch.cuda.device(self.device):
            stream = torch.cuda.current_stream(self.device).cuda_stream
            self.state = mona_init_state(shapes_only, self.count, self.opts, self.arena, stream)
        self._mats = None
        self._mats_key = None

    def close(self) -> None:
        if getattr(self, "state", None):
            mona_free_state(self.state)
            self.state = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _stream(self) -> int:
        return torch.cuda.current_stream(self.device).cuda_stream

    def step(self, grads: Sequence[torch.Tensor], hp, slots: Optional[Sequence[torch.Tensor]] = None) -> None:
        """One MONA step over all matrices (asynchronous on torch's current stream).  `slots`: the
        caller-kept previous-gradient arrays of a MONA_ACCEL_CALLER_SLOT state."""
        key = tuple(g.data_ptr() for g in grads)
        if key != self._mats_key:
            self._mats = make_matrices(self.weights, grads)
            self._mats_key = key
        hpc = hp if isinstance(hp, mona_hparams) else make_hparams(hp)
        if slots is None:
            mona_step(self.state, self._mats, self.count, hpc, self._stream())
            return
        arr = (C.c_void_p * self.count)()
        for i, t in enumerate(slots):
            if t.shape != self.weights[i].shape or not t.is_contiguous() or t.dtype != self.state_dtype:
                raise ValueError(f"slot {i}: must be contiguous, shaped like the parameter, of the state dtype")
            arr[i] = t.data_ptr()
        mona_step_streaming(self.state, self._mats, arr, self.count, hpc, self._stream())

    # ---- views of the state as torch tensors (no copy) ----
    def view(self, i: int, kind: int) -> torch.Tensor:
        v = mona_state_view(self.state, i, kind)
        dtype = torch.float32 if v.dtype == MONA_F32 else torch.bfloat16
        esize = 4 if v.dtype == MONA_F32 else 2
        off = v.ptr - self.arena.data_ptr()
        flat = self.arena[off: off + (v.rows * v.ld) * esize].view(dtype)
        return flat.view(v.rows, v.ld)[:, : v.cols]

    def g_prev(self, i): return self.view(i, MONA_VIEW_G_PREV)
    def accel(self, i): return self.view(i, MONA_VIEW_A)
    def carry(self, i): return self.view(i, MONA_VIEW_C)
    def momentum(self, i): return self.view(i, MONA_VIEW_M)
    def norm(self, i): return self.view(i, MONA_VIEW_NORM)
    def last_o(self, i): return self.view(i, MONA_VIEW_O)

    def status(self) -> List[int]:
        out = (C.c_uint32 * self.count)()
        _check(self.lib.mona_state_status(self.state, out, self.count, self._stream()))
        return list(out)

    def step_count(self) -> int:
        k = C.c_int64(0)
        _check(self.lib.mona_state_step_count(self.state, C.byref(k)))
        return k.value

    def export_state(self) -> torch.Tensor:
        n = C.c_size_t(0)
        _check(self.lib.mona_state_export_size(self.state, C.byref(n)))
        buf = torch.empty(n.value, dtype=torch.uint8, device=self.device)
        _check(self.lib.mona_state_export(self.state, buf.data_ptr(), n.value, self._stream()))
        return buf

    def import_state(self, buf: torch.Tensor, step_count: int) -> None:
        _check(self.lib.mona_state_import(self.state, buf.data_ptr(), buf.numel(), step_count, self._stream()))

    def set_profiling(self, level: int) -> None:
        _check(self.lib.mona_set_profiling(self.state, level))

    def last_step_times(self):
        """(elementwise ms, Newton-Schulz ms, separate-update ms, whole-step ms) of the last step."""
        out = (C.c_float * 4)()
        _check(self.lib.mona_last_step_times(self.state, out))
        return tuple(out)

    def mean_step_times(self):
        """The same four figures averaged over the steps profiled since set_profiling (at most the last 32),
        and the number of steps averaged."""
        out = (C.c_float * 4)()
        n = C.c_int32(0)
        _check(self.lib.mona_mean_step_times(self.state, out, C.byref(n)))
        return tuple(out), n.value

    def last_step_launches(self):
        n = C.c_int32(0)
        _check(self.lib.mona_last_step_launches(self.state, None, 0, C.byref(n)))
        arr = (mona_launch_time * max(n.value, 1))()
        _check(self.lib.mona_last_step_launches(self.state, arr, n.value, C.byref(n)))
        return [dict(kind=r.kind, group=r.group, iter=r.iter, tile=r.tile, m=r.m, n=r.n, count=r.count,
                     ms=r.ms, flops=r.flops) for r in arr[: n.value]]

    def plan_info(self, ns_steps: int):
        launches, flops, nbytes = C.c_int64(0), C.c_double(0), C.c_double(0)
        _check(self.lib.mona_plan_info(self.state, ns_steps, C.byref(launches), C.byref(flops), C.byref(nbytes)))
        return dict(ns_launches=launches.value, ns_flops_issued=flops.value, elementwise_bytes=nbytes.value)


# ---- AdamW for the parameters that are not matrices ----------------------------------------
def make_vectors(params: Sequence[torch.Tensor], grads: Optional[Sequence[torch.Tensor]] = None,
                 g_dtype: torch.dtype = torch.float32):
    """Array of mona_vector descriptors for contiguous tensors of any shape."""
    arr = (mona_vector * len(params))()
    for i, w in enumerate(params):
        if not w.is_contiguous():
            raise ValueError(f"tensor {i}: parameters must be contiguous")
        g = None if grads is None else grads[i]
        if g is not None and (g.shape != w.shape or not g.is_contiguous()):
            raise ValueError(f"tensor {i}: gradient must be contiguous and shaped like the parameter")
        arr[i].w = w.data_ptr()
        arr[i].g = 0 if g is None else g.data_ptr()
        arr[i].n = int(w.numel())
        arr[i].w_dtype = _dtype_code(w.dtype)
        arr[i].g_dtype = _dtype_code(g.dtype if g is not None else g_dtype)
    return arr


def mona_adamw_state_size(vecs, count: int) -> int:
    out = C.c_size_t(0)
    _check(load_library().mona_adamw_state_size(vecs, count, C.byref(out)))
    return out.value


def mona_adamw_step(state: int, vecs, count: int, hp: mona_adamw_hparams, stream: int) -> None:
    _check(load_library().mona_adamw_step(state, vecs, count, C.byref(hp), stream))


class AdamWOptimizer:
    """Owns the arena and the state handle for a fixed list of non-matrix parameters."""

    def __init__(self, params: Sequence[torch.Tensor], g_dtype: torch.dtype = torch.float32):
        if not params:
            raise ValueError("need at least one tensor")
        self.lib = load_library()
        self.device = params[0].device
        if self.device.type != "cuda":
            raise RuntimeError("AdamWOptimizer needs parameters on a GPU (no CPU path exists)")
        self.params = list(params)
        self.count = len(self.params)
        self.g_dtype = g_dtype
        shapes_only = make_vectors(self.params, None, g_dtype)
        self.arena_bytes = mona_adamw_state_size(shapes_only, self.count)
        self.arena = torch.empty(self.arena_bytes, dtype=torch.uint8, device=self.device)
        handle = C.c_void_p(0)
        _check(self.lib.mona_adamw_init_state(shapes_only, self.count, self.arena.data_ptr(), self.arena_bytes,
                                              self._stream(), C.byref(handle)))
        self.state = handle.value

    def _stream(self) -> int:
        with torch.cuda.device(self.device):
            return torch.cuda.current_stream(self.device).cuda_stream

    def __del__(self):
        st = getattr(self, "state", None)
        if st:
            self.lib.mona_adamw_free_state(st)
            self.state = None

    def step(self, grads: Sequence[torch.Tensor], hp) -> None:
        """hp: a mona_adamw_hparams, or any object with lr, beta1, beta2, eps, weight_decay."""
        if not isinstance(hp, mona_adamw_hparams):
            hp = mona_adamw_hparams(hp.lr, hp.beta1, hp.beta2, hp.eps, hp.weight_decay)
        vecs = make_vectors(self.params, grads)
        mona_adamw_step(self.state, vecs, self.count, hp, self._stream())

    def view(self, i: int, kind: int) -> torch.Tensor:
        ptr, n = C.c_void_p(0), C.c_int64(0)
        _check(self.lib.mona_adamw_state_view(self.state, i, kind, C.byref(ptr), C.byref(n)))
        off = ptr.value - self.arena.data_ptr()
        return self.arena[off: off + n.value * 4].view(torch.float32).view(self.params[i].shape)

    def exp_avg(self, i): return self.view(i, MONA_ADAMW_VIEW_M)
    def exp_avg_sq(self, i): return self.view(i, MONA_ADAMW_VIEW_V)

    def step_count(self) -> int:
        t = C.c_int64(0)
        _check(self.lib.mona_adamw_state_step_count(self.state, C.byref(t)))
        return t.value

    def export_state(self) -> torch.Tensor:
        n = C.c_size_t(0)
        _check(self.lib.mona_adamw_state_export_size(self.state, C.byref(n)))
        buf = torch.empty(n.value, dtype=torch.uint8, device=self.device)
        _check(self.lib.mona_adamw_state_export(self.state, buf.data_ptr(), n.value, self._stream()))
        return buf

    def import_state(self, buf: torch.Tensor, step_count: int) -> None:
        _check(self.lib.mona_adamw_state_import(self.state, buf.data_ptr(), buf.numel(), step_count, self._stream()))
