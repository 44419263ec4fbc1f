"""ctypes front end of the CPU oracle in tempo_oracle.c.

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's CPU-baseline leg.  The GPU library never imports it.

It compiles tempo_oracle.c with gcc (fp64, no fast-math) on first use and
marshals numpy arrays; it contains no arithmetic of its own.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "tempo_oracle.c")
_LIB = os.path.join(_HERE, "libtempo_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle into oracle/libtempo_oracle.so and return its path."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra",
             "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _bind(path: str):
    """Open a built oracle library and declare its signatures."""
    if True:
        lib = ctypes.CDLL(path)
        ip = ctypes.POINTER(ctypes.c_int)
        dp = ctypes.POINTER(ctypes.c_double)
        lib.tempo_oracle_visible_range.argtypes = [ctypes.c_int] * 3 + [ip] * 7
        lib.tempo_oracle_visible_range.restype = ctypes.c_int
        lib.tempo_oracle_tile_visible_count.argtypes = [ctypes.c_int] * 4
        lib.tempo_oracle_tile_visible_count.restype = ctypes.c_int
        lib.tempo_oracle_append_slot.argtypes = [ctypes.c_int, ctypes.c_int, ip, ip]
        lib.tempo_oracle_append_slot.restype = ctypes.c_int
        lib.tempo_oracle_release.argtypes = [ctypes.c_int] * 3 + [ip, ip]
        lib.tempo_oracle_release.restype = ctypes.c_int
        lib.tempo_oracle_ring_blocks.argtypes = [ctypes.c_int] * 3
        lib.tempo_oracle_ring_blocks.restype = ctypes.c_int
        lib.tempo_oracle_attend.argtypes = [dp, dp, dp] + [ctypes.c_int] * 5 + [ip, ctypes.c_int,
                                                                             ctypes.c_double, dp]
        lib.tempo_oracle_attend.restype = ctypes.c_int
        lib.tempo_oracle_rope.argtypes = [dp, ctypes.c_int, ctypes.c_int, ctypes.c_int, ip, ctypes.c_double, dp]
        lib.tempo_oracle_rope.restype = ctypes.c_int
        lib.tempo_oracle_rope_table.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_double, dp, dp]
        lib.tempo_oracle_rope_table.restype = ctypes.c_int
        lib.tempo_oracle_discounted_sum.argtypes = [dp, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_double, dp]
        lib.tempo_oracle_discounted_sum.restype = ctypes.c_int
        lib.tempo_oracle_threads.argtypes = []
        lib.tempo_oracle_threads.restype = ctypes.c_int
    return lib


def _load():
    global _lib
    if _lib is None:
        _lib = _bind(build())
    return _lib


def visible_range(t: int, window: int, Z: int) -> dict:
    """Integer quantities of step t (window = visible keys, 0 = causal)."""
    vals = [ctypes.c_int(0) for _ in range(7)]
    rc = _load().tempo_oracle_visible_range(t, window, Z, *[ctypes.byref(v) for v in vals])
    if rc != 0:
        raise ValueError("oracle: bad argument to visible_range")
    names = ["lo", "hi", "first_tile", "last_tile", "n_tiles", "first_tile_skip", "last_tile_valid"]
    return {n: v.value for n, v in zip(names, vals)}


def tile_visible_count(t: int, window: int, Z: int, n: int) -> int:
    rc = _load().tempo_oracle_tile_visible_count(t, window, Z, n)
    if rc < 0:
        raise ValueError("oracle: bad argument to tile_visible_count")
    return rc


def append_slot(t: int, Z: int):
    tile, slot = ctypes.c_int(0), ctypes.c_int(0)
    rc = _load().tempo_oracle_append_slot(t, Z, ctypes.byref(tile), ctypes.byref(slot))
    if rc != 0:
        raise ValueError("oracle: bad argument to append_slot")
    return tile.value, slot.value


def release(t: int, window: int, Z: int):
    """(dead_keys, dead_tiles) once step t has been answered (Section 5.2, deallocations)."""
    keys, tiles = ctypes.c_int(0), ctypes.c_int(0)
    rc = _load().tempo_oracle_release(t, window, Z, ctypes.byref(keys), ctypes.byref(tiles))
    if rc != 0:
        raise ValueError("oracle: bad argument to release")
    return keys.value, tiles.value


def ring_blocks(window: int, Z: int, queries: int = 1) -> int:
    """Blocks per sequence of a circular store that serves `queries` steps per call (Section 6)."""
    rc = _load().tempo_oracle_ring_blocks(window, Z, queries)
    if rc < 0:
        raise ValueError("oracle: bad argument to ring_blocks")
    return rc


def attend(q, K, V, t, window: int, scale: float) -> np.ndarray:
    """q [B][Hq][D], K/V [B][T][Hkv][D], t int or [B] ints -> out [B][Hq][D] (fp64)."""
    q = np.ascontiguousarray(q, dtype=np.float64)
    K = np.ascontiguousarray(K, dtype=np.float64)
    V = np.ascontiguousarray(V, dtype=np.float64)
    B, Hq, D = q.shape
    Bk, T, Hkv, Dk = K.shape
    if V.shape != K.shape or Bk != B or Dk != D:
        raise ValueError("oracle: q/K/V shapes disagree")
    tt = np.ascontiguousarray(np.broadcast_to(np.asarray(t, dtype=np.int32), (B,)), dtype=np.int32)
    out = np.empty((B, Hq, D), dtype=np.float64)
    dp = ctypes.POINTER(ctypes.c_double)
    rc = _load().tempo_oracle_attend(
        q.ctypes.data_as(dp), K.ctypes.data_as(dp), V.ctypes.data_as(dp),
        B, T, Hq, Hkv, D, tt.ctypes.data_as(ctypes.POINTER(ctypes.c_int)),
        int(window), float(scale), out.ctypes.data_as(dp))
    if rc != 0:
        raise ValueError("oracle: bad argument to attend")
    return out


def rope(x, t, theta: float) -> np.ndarray:
    """x [B][H][D], t int or [B] positions -> rotated copy (fp64)."""
    x = np.ascontiguousarray(x, dtype=np.float64)
    B, H, D = x.shape
    tt = np.ascontiguousarray(np.broadcast_to(np.asarray(t, dtype=np.int32), (B,)), dtype=np.int32)
    y = np.empty_like(x)
    dp = ctypes.POINTER(ctypes.c_double)
    rc = _load().tempo_oracle_rope(x.ctypes.data_as(dp), B, H, D, tt.ctypes.data_as(ctypes.POINTER(ctypes.c_int)),
                                   float(theta), y.ctypes.data_as(dp))
    if rc != 0:
        raise ValueError("oracle: bad argument to rope")
    return y


def rope_table(positions: int, D: int, theta: float):
    """(cos, sin) tables [positions][D/2] (fp64)."""
    if D < 2 or D % 2:
        raise ValueError("oracle: bad argument to rope_table")
    c = np.empty((positions, D // 2), dtype=np.float64)
    s = np.empty_like(c)
    dp = ctypes.POINTER(ctypes.c_double)
    rc = _load().tempo_oracle_rope_table(positions, D, float(theta), c.ctypes.data_as(dp), s.ctypes.data_as(dp))
    if rc != 0:
        raise ValueError("oracle: bad argument to rope_table")
    return c, s


def discounted_sum(r, n: int, gamma: float) -> np.ndarray:
    """r [B][T] -> g [B][T] (fp64): g[b][t] = sum_k gamma^k r[b][t+k] over t .. min(t+n, T)-1 (n = 0: t .. T-1)."""
    r = np.ascontiguousarray(r, dtype=np.float64)
    if r.ndim != 2:
        raise ValueError("oracle: discounted_sum takes [B][T]")
    B, T = r.shape
    g = np.empty_like(r)
    dp = ctypes.POINTER(ctypes.c_double)
    rc = _load().tempo_oracle_discounted_sum(r.ctypes.data_as(dp), B, T, int(n), float(gamma), g.ctypes.data_as(dp))
    if rc != 0:
        raise ValueError("oracle: bad argument to discounted_sum")
    return g


def threads() -> int:
    return _load().tempo_oracle_threads()
