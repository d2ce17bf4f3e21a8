"""CPU oracle of the random-gossip BMUF synchronisation step -- TEST INFRASTRUCTURE ONLY.

Thin ctypes wrapper around ``oracle/gbmuf_oracle.c`` (plain C, written from Algorithm 1
and Definition 1 of "A Random Gossip BMUF Process for Neural Language Modeling").  Only
the tests, ``__graft_entry__.smoke()`` and ``bench.py``'s ``cpu_baseline`` leg may import
this package; the product path never does and shares no code with it.

Every function takes and returns numpy arrays; parameter arrays are ``[K, stride]``
C-contiguous ``float32`` or ``float64`` (the dtype selects the fp32 or the fp64 writing of
the update) and are updated in place.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libgbmuf_oracle.so")
_SOURCES = [os.path.join(_HERE, "gbmuf_oracle.c"), os.path.join(_HERE, "gbmuf_oracle_update.inc")]

MODE_NO_RESTART = 0   # classical block momentum: theta' = omega', block starts from omega
MODE_PAPER = 1        # Algorithm 1 as printed: block starts from omega + eta*Delta
MODE_LITERAL = 2      # G = avg - omega, restart kept
MODE_GOSSIP_MA = 3    # theta' = average only


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no FMA contraction, OpenMP over elements)."""
    stale = force or not os.path.exists(_LIB_PATH) or any(
        os.path.getmtime(s) > os.path.getmtime(_LIB_PATH) for s in _SOURCES)
    if stale:
        cmd = ["gcc", "-std=c99", "-O2", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC",
               "-Wall", "-Wextra", "-o", _LIB_PATH, _SOURCES[0]]
        subprocess.run(cmd, check=True, cwd=_HERE)
    return _LIB_PATH


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB_PATH)
        i32, i64, u64 = ctypes.c_int32, ctypes.c_int64, ctypes.c_uint64
        vp = ctypes.c_void_p
        L.gbmuf_oracle_philox4x32_10.argtypes = [vp, vp, vp]
        L.gbmuf_oracle_philox4x32_10.restype = None
        L.gbmuf_oracle_default_p.argtypes = [i32]
        L.gbmuf_oracle_default_p.restype = i32
        L.gbmuf_oracle_ring_candidates.argtypes = [i32, i32, i32, vp]
        L.gbmuf_oracle_ring_candidates.restype = i32
        L.gbmuf_oracle_sample.argtypes = [i32, i32, i32, u64, u64, i32, i32, vp]
        L.gbmuf_oracle_neighbour_table.argtypes = [i32, i32, i32, i32, u64, u64, vp]
        L.gbmuf_oracle_neighbour_table_q.argtypes = [i32, i32, i32, vp, i32, u64, u64, vp]
        for suffix, real in (("f32", ctypes.c_float), ("f64", ctypes.c_double)):
            f = getattr(L, "gbmuf_oracle_sync_table_" + suffix)
            f.argtypes = [vp, i32, i32, i32, vp, vp, vp, vp, vp, i64, real, real, i32]
            f = getattr(L, "gbmuf_oracle_sync_" + suffix)
            f.argtypes = [vp, i32, i32, i32, i32, u64, u64, vp, vp, vp, vp, i64, real, real, i32]
            f = getattr(L, "gbmuf_oracle_sync_table_q_" + suffix)
            f.argtypes = [vp, i32, i32, vp, i32, vp, vp, vp, vp, vp, i64, real, real, i32]
            f = getattr(L, "gbmuf_oracle_sync_q_" + suffix)
            f.argtypes = [vp, i32, i32, i32, vp, u64, u64, vp, vp, vp, vp, i64, real, real, i32]
            f = getattr(L, "gbmuf_oracle_final_average_" + suffix)
            f.argtypes = [i32, i64, vp, i64, vp]
        L.gbmuf_oracle_threads.restype = ctypes.c_int
        _lib = L
    return _lib


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _check(rc: int, what: str) -> None:
    if rc != 0:
        raise ValueError(f"oracle {what}: status {rc} ({ {1: 'EINVAL', 2: 'ENOMEM'}.get(rc, '?') })")


def threads() -> int:
    return int(lib().gbmuf_oracle_threads())


def philox4x32_10(ctr, key) -> np.ndarray:
    c = np.ascontiguousarray(ctr, dtype=np.uint32)
    k = np.ascontiguousarray(key, dtype=np.uint32)
    assert c.shape == (4,) and k.shape == (2,)
    out = np.zeros(4, dtype=np.uint32)
    lib().gbmuf_oracle_philox4x32_10(_ptr(c), _ptr(k), _ptr(out))
    return out


def default_p(K: int) -> int:
    return int(lib().gbmuf_oracle_default_p(K))


def ring_candidates(w: int, K: int, p: int) -> np.ndarray:
    buf = np.zeros(max(K, 1), dtype=np.int32)
    C = lib().gbmuf_oracle_ring_candidates(w, K, p, _ptr(buf))
    return buf[:C].copy()


def sample(K: int, p: int, q: int, seed: int, round: int, w: int, i: int) -> np.ndarray:
    out = np.zeros(max(q, 1), dtype=np.int32)
    _check(lib().gbmuf_oracle_sample(K, p, q, seed, round, w, i, _ptr(out)), "sample")
    return out[:q].copy()


def neighbour_table(m: int, K: int, p: int, q, seed: int, round: int, width=None) -> np.ndarray:
    """Neighbour table of one sync.  ``q`` an int: ``[m, K, q]``.  ``q`` a sequence of m ints
    (component i draws q[i] neighbours): ``[m, K, width]`` (width defaults to max q), rows
    filled with -1 beyond their q[i] entries."""
    if np.ndim(q) == 0:
        out = np.zeros((m, K, int(q)), dtype=np.int32)
        _check(lib().gbmuf_oracle_neighbour_table(m, K, p, int(q), seed, round, _ptr(out)), "neighbour_table")
        return out
    qv = np.ascontiguousarray(q, dtype=np.int32)
    assert qv.shape == (m,)
    width = int(qv.max(initial=0)) if width is None else int(width)
    out = np.zeros((m, K, width), dtype=np.int32)
    _check(lib().gbmuf_oracle_neighbour_table_q(m, K, p, _ptr(qv), width, seed, round, _ptr(out)), "neighbour_table_q")
    return out


def _state_args(off, theta, omega, delta):
    off = np.ascontiguousarray(off, dtype=np.int64)
    assert theta.ndim == 2 and theta.flags.c_contiguous and theta.dtype in (np.float32, np.float64)
    for a in (omega, delta):
        assert a is None or (a.shape == theta.shape and a.dtype == theta.dtype and a.flags.c_contiguous)
    suffix = "f32" if theta.dtype == np.float32 else "f64"
    return off, suffix, theta.shape[0], theta.shape[1]


def sync_table(off, nbr, theta, omega, delta, eta, zeta, mode=MODE_PAPER, active=None, q=None) -> None:
    """One sync with a caller-supplied neighbour table (in place): ``[m, K, q]``, or, with
    ``q`` a sequence of m ints, ``[m, K, width]`` of which component i uses q[i] entries."""
    off, suffix, K, stride = _state_args(off, theta, omega, delta)
    m = len(off) - 1
    nbr = np.ascontiguousarray(nbr, dtype=np.int32)
    assert nbr.ndim == 3 and nbr.shape[0] == m and nbr.shape[1] == K
    act = None if active is None else np.ascontiguousarray(active, dtype=np.uint8)
    assert act is None or act.shape == (m,)
    if q is None:
        f = getattr(lib(), "gbmuf_oracle_sync_table_" + suffix)
        _check(f(_ptr(off), m, K, nbr.shape[2], _ptr(nbr), _ptr(act), _ptr(theta), _ptr(omega), _ptr(delta),
                 stride, eta, zeta, mode), "sync_table")
        return
    qv = np.ascontiguousarray(q, dtype=np.int32)
    assert qv.shape == (m,)
    f = getattr(lib(), "gbmuf_oracle_sync_table_q_" + suffix)
    _check(f(_ptr(off), m, K, _ptr(qv), nbr.shape[2], _ptr(nbr), _ptr(act), _ptr(theta), _ptr(omega), _ptr(delta),
             stride, eta, zeta, mode), "sync_table_q")


def sync(off, K, p, q, seed, round, theta, omega, delta, eta, zeta, mode=MODE_PAPER, active=None) -> None:
    """One sync with neighbours drawn for ``(seed, round)`` (in place); ``q`` an int, or a
    sequence of m ints (component i draws q[i] neighbours)."""
    off, suffix, K2, stride = _state_args(off, theta, omega, delta)
    assert K2 == K
    m = len(off) - 1
    act = None if active is None else np.ascontiguousarray(active, dtype=np.uint8)
    assert act is None or act.shape == (m,)
    if np.ndim(q) != 0:
        qv = np.ascontiguousarray(q, dtype=np.int32)
        assert qv.shape == (m,)
        f = getattr(lib(), "gbmuf_oracle_sync_q_" + suffix)
        _check(f(_ptr(off), m, K, p, _ptr(qv), seed, round, _ptr(act), _ptr(theta), _ptr(omega), _ptr(delta),
                 stride, eta, zeta, mode), "sync_q")
        return
    f = getattr(lib(), "gbmuf_oracle_sync_" + suffix)
    _check(f(_ptr(off), m, K, p, q, seed, round, _ptr(act), _ptr(theta), _ptr(omega), _ptr(delta),
             stride, eta, zeta, mode), "sync")


def final_average(theta, P=None) -> np.ndarray:
    """(1/K) * sum over workers of theta (Algorithm 1, RETURN)."""
    assert theta.ndim == 2 and theta.flags.c_contiguous
    K, stride = theta.shape
    P = stride if P is None else P
    suffix = "f32" if theta.dtype == np.float32 else "f64"
    out = np.zeros(P, dtype=theta.dtype)
    f = getattr(lib(), "gbmuf_oracle_final_average_" + suffix)
    _check(f(K, P, _ptr(theta), stride, _ptr(out)), "final_average")
    return out
