"""ctypes binding of libgbmuf.so: argument marshalling only, same names as include/gbmuf.h.

Device buffers are passed as integers (``tensor.data_ptr()``) or as any object with a
``data_ptr()`` method; streams as ``torch.cuda.Stream.cuda_stream`` integers (0/None = the
default stream).  Nothing here computes: every step runs in the library's kernels.  If the
library has not been built the import of this module fails loudly.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import numpy as np
import torch  # noqa: F401  -- first: libgbmuf must bind to the HIP runtime that torch has loaded, not a second copy

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libgbmuf.so")

GBMUF_OK, GBMUF_EINVAL, GBMUF_ENOMEM, GBMUF_EDEVICE, GBMUF_EUNSUPPORTED = 0, 1, 2, 3, 4
MODE_NO_RESTART, MODE_PAPER, MODE_LITERAL, MODE_GOSSIP_MA = 0, 1, 2, 3
SAMPLING_AUTO, SAMPLING_IN_KERNEL, SAMPLING_SEPARATE = 0, 1, 2
SWEEP_AUTO, SWEEP_FORWARD = 0, 1
LAYOUT_ROWS, LAYOUT_BLOCKED = 0, 1
MAX_K = 1024
STATIC_TABLE_ENTRIES = 1 << 19


class GbmufError(RuntimeError):
    def __init__(self, code: int, what: str):
        self.code = code
        detail = _lib.gbmuf_last_error_detail().decode()
        super().__init__(f"{what}: {strerror(code)} (status {code})" + (f" [{detail}]" if detail else ""))


class Info(ctypes.Structure):
    _fields_ = [("m", ctypes.c_int32), ("K", ctypes.c_int32), ("q", ctypes.c_int32), ("p", ctypes.c_int32),
                ("C", ctypes.c_int32), ("has_device", ctypes.c_int32), ("P", ctypes.c_int64),
                ("n_tiles", ctypes.c_int64), ("tile_columns", ctypes.c_int32), ("threads", ctypes.c_int32),
                ("seed", ctypes.c_uint64), ("mixed_q", ctypes.c_int32), ("has_periods", ctypes.c_int32),
                ("in_kernel_sampling", ctypes.c_int32), ("tile_columns_blocked", ctypes.c_int32),
                ("threads_blocked", ctypes.c_int32), ("workgroups_per_cu_blocked", ctypes.c_int32),
                ("tile_columns_blocked_ma", ctypes.c_int32), ("min_block_floats", ctypes.c_int32)]


class PlanDesc(ctypes.Structure):
    _fields_ = [("struct_size", ctypes.c_uint32), ("m", ctypes.c_int32), ("K", ctypes.c_int32), ("q", ctypes.c_int32),
                ("comp_offsets", ctypes.c_void_p), ("q_per_component", ctypes.c_void_p), ("periods", ctypes.c_void_p),
                ("p", ctypes.c_int32), ("reserved0", ctypes.c_int32), ("seed", ctypes.c_uint64),
                ("tile_threads", ctypes.c_int32), ("tile_slots", ctypes.c_int32), ("sampling", ctypes.c_int32),
                ("sweep", ctypes.c_int32), ("cache_hints", ctypes.c_int32), ("workgroups_per_cu", ctypes.c_int32)]


class State(ctypes.Structure):
    """gbmuf_state_t: where theta, omega, delta are (device pointers as integers) and how they are laid out."""
    _fields_ = [("theta", ctypes.c_void_p), ("omega", ctypes.c_void_p), ("delta", ctypes.c_void_p),
                ("worker_stride", ctypes.c_int64), ("block_floats", ctypes.c_int64), ("block_stride", ctypes.c_int64)]


class Layout(ctypes.Structure):
    _fields_ = [("worker_stride", ctypes.c_int64), ("block_floats", ctypes.c_int64), ("block_stride", ctypes.c_int64),
                ("omega_offset", ctypes.c_int64), ("delta_offset", ctypes.c_int64), ("arena_floats", ctypes.c_int64)]


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        # nothing built yet: build once with hipcc; there is no other (CPU, eager) path to fall back to
        try:
            from .build import build_library
            build_library(verbose=False)
        except Exception as e:  # noqa: BLE001
            raise ImportError(
                f"{LIB_PATH} is missing and could not be built ({e!r}): run "
                "python -c 'import __graft_entry__ as g; g.build()'.  There is no fallback path.") from e
    L = ctypes.CDLL(LIB_PATH)
    i32, i64, u64, f32, vp = ctypes.c_int32, ctypes.c_int64, ctypes.c_uint64, ctypes.c_float, ctypes.c_void_p
    L.gbmuf_plan.argtypes = [ctypes.POINTER(vp), vp, i32, i32, i32, i32, u64]
    L.gbmuf_plan_create.argtypes = [ctypes.POINTER(vp), ctypes.POINTER(PlanDesc)]
    L.gbmuf_plan_destroy.argtypes = [vp]
    L.gbmuf_plan_info.argtypes = [vp, ctypes.POINTER(Info)]
    L.gbmuf_candidates_host.argtypes = [vp, i32, vp]
    L.gbmuf_neighbours_host.argtypes = [vp, u64, vp]
    L.gbmuf_neighbours_device.argtypes = [vp, u64, vp, vp]
    L.gbmuf_sync.argtypes = [vp, vp, vp, vp, i64, f32, f32, i32, u64, vp]
    L.gbmuf_sync_table.argtypes = [vp, vp, vp, vp, vp, i64, f32, f32, i32, vp]
    L.gbmuf_sync_step.argtypes = [vp, vp, vp, vp, i64, f32, f32, i32, u64, vp]
    L.gbmuf_final_average.argtypes = [vp, vp, i64, vp, vp]
    sp = ctypes.POINTER(State)
    L.gbmuf_sync_state.argtypes = [vp, sp, f32, f32, i32, u64, vp]
    L.gbmuf_sync_step_state.argtypes = [vp, sp, f32, f32, i32, u64, vp]
    L.gbmuf_sync_static.argtypes = [vp, sp, f32, f32, i32, u64, vp]
    L.gbmuf_sync_static.restype = ctypes.c_int
    L.gbmuf_sync_table_state.argtypes = [vp, vp, sp, f32, f32, i32, vp]
    L.gbmuf_final_average_state.argtypes = [vp, sp, vp, vp]
    L.gbmuf_state_copy.argtypes = [vp, sp, sp, i32, vp]
    L.gbmuf_recommend_layout.argtypes = [vp, i64, i32, i32, ctypes.POINTER(Layout)]
    for name in ("gbmuf_plan_create", "gbmuf_sync_step", "gbmuf_final_average", "gbmuf_sync_state",
                 "gbmuf_sync_step_state", "gbmuf_sync_table_state", "gbmuf_final_average_state", "gbmuf_state_copy",
                 "gbmuf_recommend_layout"):
        getattr(L, name).restype = ctypes.c_int
    L.gbmuf_probe_copy.argtypes = [vp, vp, i64, i32, vp]
    L.gbmuf_probe_copy.restype = ctypes.c_int
    L.gbmuf_strerror.argtypes = [ctypes.c_int]
    L.gbmuf_strerror.restype = ctypes.c_char_p
    L.gbmuf_last_error_detail.argtypes = []
    L.gbmuf_last_error_detail.restype = ctypes.c_char_p
    for name in ("gbmuf_plan", "gbmuf_plan_destroy", "gbmuf_plan_info", "gbmuf_candidates_host",
                 "gbmuf_neighbours_host", "gbmuf_neighbours_device", "gbmuf_sync", "gbmuf_sync_table"):
        getattr(L, name).restype = ctypes.c_int
    return L


_lib = _load()


def lib() -> ctypes.CDLL:
    return _lib


def strerror(code: int) -> str:
    return _lib.gbmuf_strerror(code).decode()


def _dev(x) -> Optional[int]:
    if x is None:
        return None
    if hasattr(x, "data_ptr"):
        return int(x.data_ptr())
    return int(x)


def _stream(s) -> Optional[int]:
    if s is None:
        return None
    if hasattr(s, "cuda_stream"):
        return int(s.cuda_stream) or None
    return int(s) or None


def recommend_layout(P: int, K: int, kind: int = LAYOUT_BLOCKED, plan: "Optional[Plan]" = None) -> Layout:
    out = Layout()
    rc = _lib.gbmuf_recommend_layout(plan._h if plan is not None else None, P, K, kind, ctypes.byref(out))
    if rc != GBMUF_OK:
        raise GbmufError(rc, "gbmuf_recommend_layout")
    return out


def make_state(theta, omega, delta, worker_stride: int, block_floats: int = 0, block_stride: int = 0) -> State:
    return State(_dev(theta), _dev(omega), _dev(delta), worker_stride, block_floats, block_stride)


def probe_copy(dst_dev, src_dev, n_floats: int, flags: int = 0, stream=None) -> None:
    rc = _lib.gbmuf_probe_copy(_dev(dst_dev), _dev(src_dev), n_floats, flags, _stream(stream))
    if rc != GBMUF_OK:
        raise GbmufError(rc, "gbmuf_probe_copy")


class Plan:
    """Owns one ``gbmuf_plan_t``.  Methods mirror the C entry points one to one."""

    def __init__(self, comp_offsets: Sequence[int], K: int, q=0, p: int = 0, seed: int = 0, periods=None,
                 tile=None, sampling: int = SAMPLING_AUTO, sweep: int = SWEEP_AUTO, cache_hints: int = 0,
                 workgroups_per_cu: int = 0):
        """gbmuf_plan_create.  ``q``: an int, or a sequence of m ints (neighbours per component).
        ``periods``: m sync periods H_i or None.  ``tile``: (threads, slots) or None."""
        off = np.ascontiguousarray(comp_offsets, dtype=np.int64)
        if off.ndim != 1 or off.size < 1:
            raise GbmufError(GBMUF_EINVAL, "gbmuf_plan_create")
        m = off.size - 1
        d = PlanDesc()
        d.struct_size = ctypes.sizeof(PlanDesc)
        d.m, d.K, d.p, d.seed = m, K, p, seed & 0xFFFFFFFFFFFFFFFF
        d.comp_offsets = off.ctypes.data
        keep = [off]
        if np.ndim(q) == 0:
            d.q = int(q)
        else:
            qv = np.ascontiguousarray(q, dtype=np.int32)
            if qv.shape != (m,):
                raise GbmufError(GBMUF_EINVAL, "gbmuf_plan_create")
            d.q_per_component = qv.ctypes.data if m else None
            keep.append(qv)
        if periods is not None:
            h = np.ascontiguousarray(periods, dtype=np.int32)
            if h.shape != (m,):
                raise GbmufError(GBMUF_EINVAL, "gbmuf_plan_create")
            d.periods = h.ctypes.data if m else None
            keep.append(h)
        if tile is not None:
            d.tile_threads, d.tile_slots = int(tile[0]), int(tile[1])
        d.sampling, d.sweep, d.cache_hints, d.workgroups_per_cu = sampling, sweep, cache_hints, workgroups_per_cu
        self._h = ctypes.c_void_p()
        rc = _lib.gbmuf_plan_create(ctypes.byref(self._h), ctypes.byref(d))
        del keep
        if rc != GBMUF_OK:
            self._h = ctypes.c_void_p()
            raise GbmufError(rc, "gbmuf_plan_create")
        self.info = self.plan_info()

    def destroy(self) -> None:
        if getattr(self, "_h", None) is not None and self._h:
            _lib.gbmuf_plan_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass

    def plan_info(self) -> Info:
        info = Info()
        rc = _lib.gbmuf_plan_info(self._h, ctypes.byref(info))
        if rc != GBMUF_OK:
            raise GbmufError(rc, "gbmuf_plan_info")
        return info

    def candidates_host(self, w: int) -> np.ndarray:
        out = np.zeros(max(self.info.C, 1), dtype=np.int32)
        rc = _lib.gbmuf_candidates_host(self._h, w, out.ctypes.data_as(ctypes.c_void_p))
        if rc != GBMUF_OK:
            raise GbmufError(rc, "gbmuf_candidates_host")
        return out[: self.info.C].copy()

    def neighbours_host(self, round: int) -> np.ndarray:
        out = np.full((self.info.m, self.info.K, self.info.q), -1, dtype=np.int32)
        rc = _lib.gbmuf_neighbours_host(self._h, round, out.ctypes.data_as(ctypes.c_void_p))
        if rc != GBMUF_OK:
            raise GbmufError(rc, "gbmuf_neighbours_host")
        return out

    def neighbours_device(self, round: int, out_dev, stream=None) -> None:
        rc = _lib.gbmuf_neighbours_device(self._h, round, _dev(out_dev), _stream(stream))
        if rc != GBMUF_OK:
            raise GbmufError(rc, "gbmuf_neighbours_device")

    def sync(self, replicas, global_, delta, worker_stride: int, eta: float, zeta: float,
             nesterov: int = MODE_PAPER, round: int = 0, stream=None) -> None:
        rc = _lib.gbmuf_sync(self._h, _dev(replicas), _dev(global_), _dev(delta), worker_stride, eta, zeta,
                             nesterov, round, _stream(stream))
        if rc != GBMUF_OK:
            raise GbmufError(rc, "gbmuf_sync")

    def sync_step(self, replicas, global_, delta, worker_stride: int, eta: float, zeta: float,
                  nesterov: int = MODE_PAPER, step: int = 0, stream=None) -> None:
        rc = _lib.gbmuf_sync_step(self._h, _dev(replicas), _dev(global_), _dev(delta), worker_stride, eta, zeta,
                                  nesterov, step, _stream(stream))
        if rc != GBMUF_OK:
            raise GbmufError(rc, "gbmuf_sync_step")

    def final_average(self, replicas, worker_stride: int, out_dev, stream=None) -> None:
        rc = _lib.gbmuf_final_average(self._h, _dev(replicas), worker_stride, _dev(out_dev), _stream(stream))
        if rc != GBMUF_OK:
            raise GbmufError(rc, "gbmuf_final_average")

    def sync_table(self, nbr_dev, replicas, global_, delta, worker_stride: int, eta: float, zeta: float,
                   nesterov: int = MODE_PAPER, stream=None) -> None:
        rc = _lib.gbmuf_sync_table(self._h, _dev(nbr_dev), _dev(replicas), _dev(global_), _dev(delta),
                                   worker_stride, eta, zeta, nesterov, _stream(stream))
        if rc != GBMUF_OK:
            raise GbmufError(rc, "gbmuf_sync_table")

    def sync_state(self, state: State, eta: float, zeta: float, nesterov: int = MODE_PAPER, round: int = 0,
                   stream=None) -> None:
        rc = _lib.gbmuf_sync_state(self._h, ctypes.byref(state), eta, zeta, nesterov, round, _stream(stream))
        if rc != GBMUF_OK:
            raise GbmufError(rc, "gbmuf_sync_state")

    def sync_static(self, state: State, eta: float, zeta: float, nesterov: int = MODE_PAPER, round: int = 0,
                    stream=None) -> None:
        rc = _lib.gbmuf_sync_static(self._h, ctypes.byref(state), eta, zeta, nesterov, round, _stream(stream))
        if rc != GBMUF_OK:
            raise GbmufError(rc, "gbmuf_sync_static")

    def sync_step_state(self, state: State, eta: float, zeta: float, nesterov: int = MODE_PAPER, step: int = 0,
                        stream=None) -> None:
        rc = _lib.gbmuf_sync_step_state(self._h, ctypes.byref(state), eta, zeta, nesterov, step, _stream(stream))
        if rc != GBMUF_OK:
            raise GbmufError(rc, "gbmuf_sync_step_state")

    def sync_table_state(self, nbr_dev, state: State, eta: float, zeta: float, nesterov: int = MODE_PAPER,
                         stream=None) -> None:
        rc = _lib.gbmuf_sync_table_state(self._h, _dev(nbr_dev), ctypes.byref(state), eta, zeta, nesterov,
                                         _stream(stream))
        if rc != GBMUF_OK:
            raise GbmufError(rc, "gbmuf_sync_table_state")

    def final_average_state(self, state: State, out_dev, stream=None) -> None:
        rc = _lib.gbmuf_final_average_state(self._h, ctypes.byref(state), _dev(out_dev), _stream(stream))
        if rc != GBMUF_OK:
            raise GbmufError(rc, "gbmuf_final_average_state")

    def state_copy(self, dst: State, src: State, which: int = 7, stream=None) -> None:
        rc = _lib.gbmuf_state_copy(self._h, ctypes.byref(dst), ctypes.byref(src), which, _stream(stream))
        if rc != GBMUF_OK:
            raise GbmufError(rc, "gbmuf_state_copy")
