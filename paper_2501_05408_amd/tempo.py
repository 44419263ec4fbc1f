"""Thin Python binding of libtempo's C ABI (include/tempo.h).

Argument marshalling only: every function here has the name and the meaning of
the C entry point it forwards to, and no step of the path is computed in Python.
Device buffers are passed as torch tensors (their data_ptr() is taken) or as raw
integer addresses; torch is used by callers for device memory and streams only.

The shared library is loaded from paper_2501_05408_amd/lib/libtempo.so.  If it
has not been built yet it is compiled (hipcc, gfx950) on first use; if it cannot
be loaded the import of a GPU entry point fails loudly -- there is no fallback.
"""
from __future__ import annotations

import ctypes
import os

from . import build as _build

TEMPO_BF16 = 0
TEMPO_F32 = 1

TEMPO_OK = 0
TEMPO_ERR_NULL = -1
TEMPO_ERR_SHAPE = -2
TEMPO_ERR_RANGE = -3
TEMPO_ERR_WORKSPACE = -4
TEMPO_ERR_DTYPE = -5
TEMPO_ERR_LAUNCH = -6


class tempo_kv(ctypes.Structure):
    _fields_ = [
        ("k_pool", ctypes.c_void_p),
        ("v_pool", ctypes.c_void_p),
        ("block_table", ctypes.c_void_p),
        ("num_blocks", ctypes.c_int32),
        ("max_blocks_per_seq", ctypes.c_int32),
        ("block_size", ctypes.c_int32),
        ("num_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32),
        ("dtype", ctypes.c_int32),
        ("ring_blocks", ctypes.c_int32),
    ]


class tempo_plan(ctypes.Structure):
    _fields_ = [
        ("tokens_per_split", ctypes.c_int32),
        ("num_splits", ctypes.c_int32),
        ("waves", ctypes.c_int32),
    ]

    def __repr__(self):
        return (f"tempo_plan(tokens_per_split={self.tokens_per_split}, "
                f"num_splits={self.num_splits}, waves={self.waves})")


class tempo_rope(ctypes.Structure):
    _fields_ = [
        ("cos", ctypes.c_void_p),
        ("sin", ctypes.c_void_p),
        ("positions", ctypes.c_int32),
        ("head_dim", ctypes.c_int32),
    ]


class TempoError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {tempo_strerror(status)} (status {status})")


_lib = None

_i32 = ctypes.c_int32
_vp = ctypes.c_void_p
_kvp = ctypes.POINTER(tempo_kv)
_planp = ctypes.POINTER(tempo_plan)
_ropep = ctypes.POINTER(tempo_rope)
_i32p = ctypes.POINTER(ctypes.c_int32)

# name -> (restype, argtypes); kept in the order of include/tempo.h
SIGNATURES = {
    "tempo_visible_range": (ctypes.c_int, [_i32, _i32, _i32] + [_i32p] * 6),
    "tempo_append_slot": (ctypes.c_int, [_i32, _i32, _i32p, _i32p]),
    "tempo_kv_release": (ctypes.c_int, [_i32, _i32, _i32, _i32p, _i32p]),
    "tempo_ring_blocks": (ctypes.c_int, [_i32, _i32, _i32, _i32p]),
    "tempo_kv_element_offset": (ctypes.c_int64, [_kvp, _i32, _i32, _i32, _i32, _i32]),
    "tempo_kv_pool_bytes": (ctypes.c_size_t, [_kvp]),
    "tempo_attn_plan": (ctypes.c_int, [_kvp, _i32, _i32, _i32, _i32, _i32, _planp]),
    "tempo_attn_workspace_bytes": (ctypes.c_size_t, [_kvp, _i32, _i32, _i32]),
    "tempo_strerror": (ctypes.c_char_p, [ctypes.c_int]),
    "tempo_kv_append": (ctypes.c_int, [_kvp, _vp, _vp, _i32, _i32, _vp, _vp]),
    "tempo_kv_gather": (ctypes.c_int, [_kvp, _vp, _vp, _i32, _i32, _i32, _vp]),
    "tempo_attn_decode_causal": (ctypes.c_int, [_kvp, _vp, _vp, _i32, _i32, _i32, _vp, ctypes.c_float,
                                                _vp, ctypes.c_size_t, _vp]),
    "tempo_attn_decode_window": (ctypes.c_int, [_kvp, _vp, _vp, _i32, _i32, _i32, _vp, _i32,
                                                ctypes.c_float, _vp, ctypes.c_size_t, _vp]),
    "tempo_decode_step_causal": (ctypes.c_int, [_kvp, _vp, _vp, _vp, _vp, _i32, _i32, _i32, _vp,
                                                ctypes.c_float, _vp, ctypes.c_size_t, _vp]),
    "tempo_decode_step_window": (ctypes.c_int, [_kvp, _vp, _vp, _vp, _vp, _i32, _i32, _i32, _vp, _i32,
                                                ctypes.c_float, _vp, ctypes.c_size_t, _vp]),
    "tempo_attn_worklist_bytes": (ctypes.c_size_t, [_kvp, _i32, _i32, _i32, _i32]),
    "tempo_attn_worklist_build": (ctypes.c_int, [_kvp, _i32, _i32, _i32, _vp, _i32, _vp, ctypes.c_size_t, _vp]),
    "tempo_decode_step_ragged": (ctypes.c_int, [_kvp, _vp, _vp, _vp, _vp, _i32, _i32, _i32, _vp, _i32,
                                                ctypes.c_float, _vp, _vp, ctypes.c_size_t, _vp]),
    "tempo_decode_step_causal_noalloc": (ctypes.c_int, [_kvp, _vp, _vp, _vp, _vp, _i32, _i32, _i32, _vp,
                                                        ctypes.c_float, _vp]),
    "tempo_attn_decode_padded_causal": (ctypes.c_int, [_kvp, _vp, _vp, _i32, _i32, _i32, _vp, _i32, ctypes.c_float,
                                                       _vp, ctypes.c_size_t, _vp]),
    "tempo_rope_rotate": (ctypes.c_int, [_ropep, _vp, _vp, _i32, _i32, _i32, _i32, _vp, _vp]),
    "tempo_rope_kv_append": (ctypes.c_int, [_kvp, _ropep, _vp, _vp, _i32, _i32, _vp, _vp]),
    "tempo_rope_decode_step_causal": (ctypes.c_int, [_kvp, _ropep, _vp, _vp, _vp, _vp, _i32, _i32, _i32, _vp,
                                                     ctypes.c_float, _vp, ctypes.c_size_t, _vp]),
    "tempo_rope_decode_step_window": (ctypes.c_int, [_kvp, _ropep, _vp, _vp, _vp, _vp, _i32, _i32, _i32, _vp,
                                                     _i32, ctypes.c_float, _vp, ctypes.c_size_t, _vp]),
    "tempo_attn_block_causal": (ctypes.c_int, [_kvp, _vp, _vp, _i32, _i32, _i32, _i32, _vp, ctypes.c_float,
                                               _vp, ctypes.c_size_t, _vp]),
    "tempo_attn_block_window": (ctypes.c_int, [_kvp, _vp, _vp, _i32, _i32, _i32, _i32, _vp, _i32,
                                               ctypes.c_float, _vp, ctypes.c_size_t, _vp]),
    "tempo_prefill_causal": (ctypes.c_int, [_kvp, _vp, _vp, _vp, _vp, _i32, _i32, _i32, _i32, _vp, ctypes.c_float,
                                            _vp, ctypes.c_size_t, _vp]),
    "tempo_prefill_window": (ctypes.c_int, [_kvp, _vp, _vp, _vp, _vp, _i32, _i32, _i32, _i32, _vp, _i32,
                                            ctypes.c_float, _vp, ctypes.c_size_t, _vp]),
    "tempo_rope_prefill_causal": (ctypes.c_int, [_kvp, _ropep, _vp, _vp, _vp, _vp, _i32, _i32, _i32, _i32, _vp,
                                                 ctypes.c_float, _vp, ctypes.c_size_t, _vp]),
    "tempo_rope_prefill_window": (ctypes.c_int, [_kvp, _ropep, _vp, _vp, _vp, _vp, _i32, _i32, _i32, _i32, _vp, _i32,
                                                 ctypes.c_float, _vp, ctypes.c_size_t, _vp]),
    "tempo_prefill_launches": (ctypes.c_int, [_kvp, _i32, _i32, _i32]),
    "tempo_prefill_workspace_bytes": (ctypes.c_size_t, [_kvp, _i32, _i32, _i32]),
    "tempo_attn_block_with_plan": (ctypes.c_int, [_kvp, _vp, _vp, _i32, _i32, _i32, _i32, _vp, _i32, ctypes.c_float,
                                                  _planp, _vp, ctypes.c_size_t, _vp]),
    "tempo_attn_block_plan": (ctypes.c_int, [_kvp, _i32, _i32, _i32, _i32, _i32, _i32, _planp]),
    "tempo_attn_block_workspace_bytes": (ctypes.c_size_t, [_kvp, _i32, _i32, _i32, _i32]),
    "tempo_kv_append_block": (ctypes.c_int, [_kvp, _vp, _vp, _i32, _i32, _vp, _i32, _vp]),
    "tempo_rope_kv_append_block": (ctypes.c_int, [_kvp, _ropep, _vp, _vp, _i32, _i32, _vp, _i32, _vp]),
    "tempo_rope_attn_block_causal": (ctypes.c_int, [_kvp, _ropep, _vp, _vp, _i32, _i32, _i32, _i32, _vp,
                                                    ctypes.c_float, _vp, ctypes.c_size_t, _vp]),
    "tempo_rope_attn_block_window": (ctypes.c_int, [_kvp, _ropep, _vp, _vp, _i32, _i32, _i32, _i32, _vp, _i32,
                                                    ctypes.c_float, _vp, ctypes.c_size_t, _vp]),
    "tempo_attn_decode_partial": (ctypes.c_int, [_kvp, _vp, _vp, _vp, _i32, _i32, _i32, _vp, _i32,
                                                 ctypes.c_float, _planp, _vp, ctypes.c_size_t, _vp]),
    "tempo_attn_decode_combine": (ctypes.c_int, [_kvp, _vp, _i32, _i32, _i32, _vp, _i32, _planp, _vp,
                                                 ctypes.c_size_t, _vp]),
    "tempo_attn_plan_workspace_bytes": (ctypes.c_size_t, [_kvp, _i32, _i32, _planp]),
    "tempo_discounted_sum": (ctypes.c_int, [_vp, _vp, _i32, _i32, _i32, ctypes.c_float, _vp]),
    "tempo_stream_read": (ctypes.c_int, [_vp, ctypes.c_size_t, _vp, _i32, _vp]),
    "tempo_stream_copy": (ctypes.c_int, [_vp, _vp, ctypes.c_size_t, _i32, _vp]),
}


def library_path() -> str:
    return _build.LIB


def _hip_runtimes_mapped():
    """Paths of the HIP runtime libraries mapped into this process."""
    found = set()
    try:
        with open("/proc/self/maps") as f:
            for line in f:
                if "libamdhip64" in line:
                    found.add(line.split()[-1])
    except OSError:
        pass
    return sorted(found)


def load():
    """Open libtempo.so (building it first only if it does not exist).

    The library must run on the same HIP runtime as the tensors it is handed.
    PyTorch ships its own copy of that runtime, so torch is imported first: the
    dynamic loader then resolves libtempo's dependency to the copy already in the
    process.  Two runtimes in one process is an error, not a fallback."""
    global _lib
    if _lib is None:
        try:
            import torch  # noqa: F401  (loads torch's HIP runtime before ours is resolved)
        except ImportError:
            pass
        path = _build.LIB
        if not os.path.exists(path):
            _build.build(force=True)
        lib = ctypes.CDLL(path)
        runtimes = _hip_runtimes_mapped()
        if len(runtimes) > 1:
            raise RuntimeError("two HIP runtimes are loaded in this process: " + ", ".join(runtimes))
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(lib, name)  # AttributeError if the library lacks a declared symbol
            fn.restype = res
            fn.argtypes = args
        _lib = lib
    return _lib


def _ptr(x):
    if x is None:
        return None
    if hasattr(x, "data_ptr"):
        return x.data_ptr()
    return int(x)


_raw_stream = None


def _stream(stream):
    """hipStream_t of `stream` (a torch stream, a raw handle, or None = torch's current stream)."""
    global _raw_stream
    if stream is None:
        if _raw_stream is None:
            import torch
            fast = getattr(torch._C, "_cuda_getCurrentRawStream", None)
            if fast is not None:
                _raw_stream = lambda: fast(torch.cuda.current_device())
            else:
                _raw_stream = lambda: torch.cuda.current_stream().cuda_stream
        return _raw_stream()
    return _ptr(getattr(stream, "cuda_stream", stream))


def _check(rc: int, where: str):
    if rc != TEMPO_OK:
        raise TempoError(rc, where)


def make_kv(k_pool, v_pool, block_table, num_blocks, max_blocks_per_seq, block_size, num_kv_heads,
            head_dim, dtype, ring_blocks=0) -> tempo_kv:
    """Fill a tempo_kv descriptor; the caller keeps the tensors alive."""
    return tempo_kv(_ptr(k_pool), _ptr(v_pool), _ptr(block_table), num_blocks, max_blocks_per_seq,
                    block_size, num_kv_heads, head_dim, dtype, ring_blocks)


def make_rope(cos_table, sin_table, head_dim) -> tempo_rope:
    """Fill a tempo_rope descriptor from two [positions][head_dim/2] fp32 device tensors."""
    return tempo_rope(_ptr(cos_table), _ptr(sin_table), int(cos_table.shape[0]), head_dim)


# ---- pure host functions -------------------------------------------------------
def tempo_visible_range(t: int, window: int, Z: int) -> dict:
    vals = [ctypes.c_int32(0) for _ in range(6)]
    _check(load().tempo_visible_range(t, window, Z, *[ctypes.byref(v) for v in vals]),
           "tempo_visible_range")
    names = ["lo", "hi", "first_tile", "last_tile", "first_tile_skip", "last_tile_valid"]
    return {n: v.value for n, v in zip(names, vals)}


def tempo_append_slot(t: int, Z: int):
    tile, slot = ctypes.c_int32(0), ctypes.c_int32(0)
    _check(load().tempo_append_slot(t, Z, ctypes.byref(tile), ctypes.byref(slot)), "tempo_append_slot")
    return tile.value, slot.value


def tempo_kv_release(t: int, window: int, Z: int):
    keys, tiles = ctypes.c_int32(0), ctypes.c_int32(0)
    _check(load().tempo_kv_release(t, window, Z, ctypes.byref(keys), ctypes.byref(tiles)), "tempo_kv_release")
    return keys.value, tiles.value


def tempo_ring_blocks(window: int, Z: int, queries: int = 1) -> int:
    ring = ctypes.c_int32(0)
    _check(load().tempo_ring_blocks(window, Z, queries, ctypes.byref(ring)), "tempo_ring_blocks")
    return ring.value


def tempo_kv_element_offset(kv: tempo_kv, which: int, block: int, head: int, slot: int, d: int) -> int:
    return load().tempo_kv_element_offset(ctypes.byref(kv), which, block, head, slot, d)


def tempo_kv_pool_bytes(kv: tempo_kv) -> int:
    return load().tempo_kv_pool_bytes(ctypes.byref(kv))


def tempo_attn_plan(kv: tempo_kv, batch: int, num_q_heads: int, t_max: int, window: int = 0,
                    ragged: bool = False) -> tempo_plan:
    plan = tempo_plan()
    _check(load().tempo_attn_plan(ctypes.byref(kv), batch, num_q_heads, t_max, window, int(ragged),
                                  ctypes.byref(plan)),
           "tempo_attn_plan")
    return plan


def tempo_attn_workspace_bytes(kv: tempo_kv, batch: int, num_q_heads: int, max_t: int) -> int:
    return load().tempo_attn_workspace_bytes(ctypes.byref(kv), batch, num_q_heads, max_t)


def tempo_attn_plan_workspace_bytes(kv: tempo_kv, batch: int, num_q_heads: int, plan: tempo_plan) -> int:
    return load().tempo_attn_plan_workspace_bytes(ctypes.byref(kv), batch, num_q_heads, ctypes.byref(plan))


def tempo_strerror(status: int) -> str:
    return load().tempo_strerror(status).decode()


# ---- device entry points ---------------------------------------------------------
def tempo_kv_append(kv, k_new, v_new, batch, t, t_per_seq=None, stream=None):
    _check(load().tempo_kv_append(ctypes.byref(kv), _ptr(k_new), _ptr(v_new), batch, t, _ptr(t_per_seq),
                                  _stream(stream)), "tempo_kv_append")


def tempo_kv_gather(kv, k_out, v_out, batch, j0, count, stream=None):
    _check(load().tempo_kv_gather(ctypes.byref(kv), _ptr(k_out), _ptr(v_out), batch, j0, count,
                                  _stream(stream)), "tempo_kv_gather")


def tempo_attn_decode_causal(kv, q, out, batch, num_q_heads, t, t_per_seq, scale, workspace,
                             workspace_bytes, stream=None):
    _check(load().tempo_attn_decode_causal(ctypes.byref(kv), _ptr(q), _ptr(out), batch, num_q_heads, t,
                                           _ptr(t_per_seq), scale, _ptr(workspace), workspace_bytes,
                                           _stream(stream)), "tempo_attn_decode_causal")


def tempo_attn_decode_window(kv, q, out, batch, num_q_heads, t, t_per_seq, window, scale, workspace,
                             workspace_bytes, stream=None):
    _check(load().tempo_attn_decode_window(ctypes.byref(kv), _ptr(q), _ptr(out), batch, num_q_heads, t,
                                           _ptr(t_per_seq), window, scale, _ptr(workspace),
                                           workspace_bytes, _stream(stream)), "tempo_attn_decode_window")


def tempo_decode_step_causal(kv, q, k_new, v_new, out, batch, num_q_heads, t, t_per_seq, scale, workspace,
                             workspace_bytes, stream=None):
    _check(load().tempo_decode_step_causal(ctypes.byref(kv), _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(out),
                                           batch, num_q_heads, t, _ptr(t_per_seq), scale, _ptr(workspace),
                                           workspace_bytes, _stream(stream)), "tempo_decode_step_causal")


def tempo_decode_step_window(kv, q, k_new, v_new, out, batch, num_q_heads, t, t_per_seq, window, scale,
                             workspace, workspace_bytes, stream=None):
    _check(load().tempo_decode_step_window(ctypes.byref(kv), _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(out),
                                           batch, num_q_heads, t, _ptr(t_per_seq), window, scale,
                                           _ptr(workspace), workspace_bytes, _stream(stream)),
           "tempo_decode_step_window")


def tempo_attn_worklist_bytes(kv, batch, num_q_heads, t_max, window=0) -> int:
    return load().tempo_attn_worklist_bytes(ctypes.byref(kv), batch, num_q_heads, t_max, window)


def tempo_attn_worklist_build(kv, batch, num_q_heads, t_max, t_per_seq, window, worklist, worklist_bytes,
                              stream=None):
    _check(load().tempo_attn_worklist_build(ctypes.byref(kv), batch, num_q_heads, t_max, _ptr(t_per_seq), window,
                                            _ptr(worklist), worklist_bytes, _stream(stream)),
           "tempo_attn_worklist_build")


def tempo_decode_step_ragged(kv, q, k_new, v_new, out, batch, num_q_heads, t_max, t_per_seq, window, scale,
                             worklist, workspace, workspace_bytes, stream=None):
    _check(load().tempo_decode_step_ragged(ctypes.byref(kv), _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(out), batch,
                                           num_q_heads, t_max, _ptr(t_per_seq), window, scale, _ptr(worklist),
                                           _ptr(workspace), workspace_bytes, _stream(stream)),
           "tempo_decode_step_ragged")


def tempo_decode_step_causal_noalloc(kv, q, k_new, v_new, out, batch, num_q_heads, t, t_per_seq, scale,
                                     stream=None):
    _check(load().tempo_decode_step_causal_noalloc(ctypes.byref(kv), _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(out),
                                                   batch, num_q_heads, t, _ptr(t_per_seq), scale,
                                                   _stream(stream)),
           "tempo_decode_step_causal_noalloc")


def tempo_attn_decode_padded_causal(kv, q, out, batch, num_q_heads, t, t_per_seq, t_pad, scale, workspace,
                                    workspace_bytes, stream=None):
    _check(load().tempo_attn_decode_padded_causal(ctypes.byref(kv), _ptr(q), _ptr(out), batch, num_q_heads, t,
                                                  _ptr(t_per_seq), t_pad, scale, _ptr(workspace),
                                                  workspace_bytes, _stream(stream)),
           "tempo_attn_decode_padded_causal")


def tempo_rope_rotate(rope, x, y, dtype, batch, heads, t, t_per_seq=None, stream=None):
    _check(load().tempo_rope_rotate(ctypes.byref(rope), _ptr(x), _ptr(y), dtype, batch, heads, t,
                                    _ptr(t_per_seq), _stream(stream)), "tempo_rope_rotate")


def tempo_rope_kv_append(kv, rope, k_raw, v_new, batch, t, t_per_seq=None, stream=None):
    _check(load().tempo_rope_kv_append(ctypes.byref(kv), ctypes.byref(rope), _ptr(k_raw), _ptr(v_new), batch, t,
                                       _ptr(t_per_seq), _stream(stream)), "tempo_rope_kv_append")


def tempo_rope_decode_step_causal(kv, rope, q_raw, k_raw, v_new, out, batch, num_q_heads, t, t_per_seq, scale,
                                  workspace, workspace_bytes, stream=None):
    _check(load().tempo_rope_decode_step_causal(ctypes.byref(kv), ctypes.byref(rope), _ptr(q_raw), _ptr(k_raw),
                                                _ptr(v_new), _ptr(out), batch, num_q_heads, t, _ptr(t_per_seq),
                                                scale, _ptr(workspace), workspace_bytes, _stream(stream)),
           "tempo_rope_decode_step_causal")


def tempo_rope_decode_step_window(kv, rope, q_raw, k_raw, v_new, out, batch, num_q_heads, t, t_per_seq, window,
                                  scale, workspace, workspace_bytes, stream=None):
    _check(load().tempo_rope_decode_step_window(ctypes.byref(kv), ctypes.byref(rope), _ptr(q_raw), _ptr(k_raw),
                                                _ptr(v_new), _ptr(out), batch, num_q_heads, t, _ptr(t_per_seq),
                                                window, scale, _ptr(workspace), workspace_bytes,
                                                _stream(stream)), "tempo_rope_decode_step_window")


def tempo_attn_block_causal(kv, q, out, batch, num_q_heads, queries, t, t_per_seq, scale, workspace,
                            workspace_bytes, stream=None):
    _check(load().tempo_attn_block_causal(ctypes.byref(kv), _ptr(q), _ptr(out), batch, num_q_heads, queries,
                                          t, _ptr(t_per_seq), scale, _ptr(workspace), workspace_bytes,
                                          _stream(stream)), "tempo_attn_block_causal")


def tempo_attn_block_window(kv, q, out, batch, num_q_heads, queries, t, t_per_seq, window, scale, workspace,
                            workspace_bytes, stream=None):
    _check(load().tempo_attn_block_window(ctypes.byref(kv), _ptr(q), _ptr(out), batch, num_q_heads, queries,
                                          t, _ptr(t_per_seq), window, scale, _ptr(workspace),
                                          workspace_bytes, _stream(stream)), "tempo_attn_block_window")


def tempo_prefill_causal(kv, q, k_new, v_new, out, batch, num_q_heads, t, count, count_per_seq, scale,
                         workspace, workspace_bytes, stream=None):
    _check(load().tempo_prefill_causal(ctypes.byref(kv), _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(out), batch,
                                       num_q_heads, t, count, _ptr(count_per_seq), scale, _ptr(workspace),
                                       workspace_bytes, _stream(stream)), "tempo_prefill_causal")


def tempo_prefill_window(kv, q, k_new, v_new, out, batch, num_q_heads, t, count, count_per_seq, window, scale,
                         workspace, workspace_bytes, stream=None):
    _check(load().tempo_prefill_window(ctypes.byref(kv), _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(out), batch,
                                       num_q_heads, t, count, _ptr(count_per_seq), window, scale,
                                       _ptr(workspace), workspace_bytes, _stream(stream)),
           "tempo_prefill_window")


def tempo_rope_prefill_causal(kv, rope, q_raw, k_raw, v_new, out, batch, num_q_heads, t, count, count_per_seq,
                              scale, workspace, workspace_bytes, stream=None):
    _check(load().tempo_rope_prefill_causal(ctypes.byref(kv), ctypes.byref(rope), _ptr(q_raw), _ptr(k_raw),
                                            _ptr(v_new), _ptr(out), batch, num_q_heads, t, count,
                                            _ptr(count_per_seq), scale, _ptr(workspace), workspace_bytes,
                                            _stream(stream)), "tempo_rope_prefill_causal")


def tempo_rope_prefill_window(kv, rope, q_raw, k_raw, v_new, out, batch, num_q_heads, t, count, count_per_seq,
                              window, scale, workspace, workspace_bytes, stream=None):
    _check(load().tempo_rope_prefill_window(ctypes.byref(kv), ctypes.byref(rope), _ptr(q_raw), _ptr(k_raw),
                                            _ptr(v_new), _ptr(out), batch, num_q_heads, t, count,
                                            _ptr(count_per_seq), window, scale, _ptr(workspace), workspace_bytes,
                                            _stream(stream)), "tempo_rope_prefill_window")


def tempo_prefill_launches(kv: tempo_kv, batch: int, num_q_heads: int, count: int) -> int:
    return load().tempo_prefill_launches(ctypes.byref(kv), batch, num_q_heads, count)


def tempo_prefill_workspace_bytes(kv: tempo_kv, batch: int, num_q_heads: int, max_t: int) -> int:
    return load().tempo_prefill_workspace_bytes(ctypes.byref(kv), batch, num_q_heads, max_t)


def tempo_attn_block_with_plan(kv, q, out, batch, num_q_heads, queries, t, t_per_seq, window, scale, plan,
                               workspace, workspace_bytes, stream=None):
    _check(load().tempo_attn_block_with_plan(ctypes.byref(kv), _ptr(q), _ptr(out), batch, num_q_heads, queries,
                                             t, _ptr(t_per_seq), window, scale, ctypes.byref(plan),
                                             _ptr(workspace), workspace_bytes, _stream(stream)),
           "tempo_attn_block_with_plan")


def tempo_attn_block_plan(kv: tempo_kv, batch: int, num_q_heads: int, queries: int, t_max: int,
                          window: int = 0, ragged: bool = False) -> tempo_plan:
    plan = tempo_plan()
    _check(load().tempo_attn_block_plan(ctypes.byref(kv), batch, num_q_heads, queries, t_max, window,
                                        int(ragged), ctypes.byref(plan)), "tempo_attn_block_plan")
    return plan


def tempo_attn_block_workspace_bytes(kv: tempo_kv, batch: int, num_q_heads: int, queries: int,
                                     max_t: int) -> int:
    return load().tempo_attn_block_workspace_bytes(ctypes.byref(kv), batch, num_q_heads, queries, max_t)


def tempo_kv_append_block(kv, k_new, v_new, batch, t, t_per_seq, count, stream=None):
    _check(load().tempo_kv_append_block(ctypes.byref(kv), _ptr(k_new), _ptr(v_new), batch, t,
                                        _ptr(t_per_seq), count, _stream(stream)), "tempo_kv_append_block")


def tempo_rope_kv_append_block(kv, rope, k_raw, v_new, batch, t, t_per_seq, count, stream=None):
    _check(load().tempo_rope_kv_append_block(ctypes.byref(kv), ctypes.byref(rope), _ptr(k_raw), _ptr(v_new), batch,
                                             t, _ptr(t_per_seq), count, _stream(stream)),
           "tempo_rope_kv_append_block")


def tempo_rope_attn_block_causal(kv, rope, q_raw, out, batch, num_q_heads, queries, t, t_per_seq, scale, workspace,
                                 workspace_bytes, stream=None):
    _check(load().tempo_rope_attn_block_causal(ctypes.byref(kv), ctypes.byref(rope), _ptr(q_raw), _ptr(out), batch,
                                               num_q_heads, queries, t, _ptr(t_per_seq), scale, _ptr(workspace),
                                               workspace_bytes, _stream(stream)), "tempo_rope_attn_block_causal")


def tempo_rope_attn_block_window(kv, rope, q_raw, out, batch, num_q_heads, queries, t, t_per_seq, window, scale,
                                 workspace, workspace_bytes, stream=None):
    _check(load().tempo_rope_attn_block_window(ctypes.byref(kv), ctypes.byref(rope), _ptr(q_raw), _ptr(out), batch,
                                               num_q_heads, queries, t, _ptr(t_per_seq), window, scale,
                                               _ptr(workspace), workspace_bytes, _stream(stream)),
           "tempo_rope_attn_block_window")


def tempo_attn_decode_partial(kv, q, k_new, v_new, batch, num_q_heads, t, t_per_seq, window, scale, plan,
                              workspace, workspace_bytes, stream=None):
    _check(load().tempo_attn_decode_partial(ctypes.byref(kv), _ptr(q), _ptr(k_new), _ptr(v_new), batch,
                                            num_q_heads, t,
                                            _ptr(t_per_seq), window, scale, ctypes.byref(plan),
                                            _ptr(workspace), workspace_bytes, _stream(stream)),
           "tempo_attn_decode_partial")


def tempo_attn_decode_combine(kv, out, batch, num_q_heads, t, t_per_seq, window, plan, workspace,
                              workspace_bytes, stream=None):
    _check(load().tempo_attn_decode_combine(ctypes.byref(kv), _ptr(out), batch, num_q_heads, t,
                                            _ptr(t_per_seq), window, ctypes.byref(plan), _ptr(workspace),
                                            workspace_bytes, _stream(stream)),
           "tempo_attn_decode_combine")


def tempo_discounted_sum(r, g, batch, T, n, gamma, stream=None):
    _check(load().tempo_discounted_sum(_ptr(r), _ptr(g), batch, T, n, gamma, _stream(stream)), "tempo_discounted_sum")


def tempo_stream_read(src, nbytes, sink, workgroups, stream=None):
    _check(load().tempo_stream_read(_ptr(src), nbytes, _ptr(sink), workgroups, _stream(stream)),
           "tempo_stream_read")


def tempo_stream_copy(src, dst, nbytes, workgroups, stream=None):
    _check(load().tempo_stream_copy(_ptr(src), _ptr(dst), nbytes, workgroups, _stream(stream)),
           "tempo_stream_copy")
