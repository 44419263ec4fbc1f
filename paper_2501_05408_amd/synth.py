"""Seeded synthetic inputs for the decode-attention path.

This module only manufactures numbers. It holds none of the method's
arithmetic (no softmax, no ranges, no block indexing), so both the CPU oracle
side of a test and the GPU side may take their inputs from it.

Two sources:

* ``normal(seed, tensor_id, shape)`` -- a stateless, counter-based N(0,1)
  generator in numpy: element ``i`` of tensor ``tensor_id`` under ``seed`` is a
  pure function of ``(seed, tensor_id, i)`` (a 64-bit mixing hash feeding a
  Box-Muller transform in fp64).  Any step of a long decode can therefore be
  regenerated without storing the others.
* ``device_normal(shape, seed, dtype, device)`` -- bulk N(0,1) made on the GPU
  by torch's seeded generator, for pools of several GiB that a numpy loop on
  the host could not fill in reasonable time.  The oracle side of such a test
  reads the very same values back from device memory.

bf16 helpers round to nearest-even, which is what "inputs in bf16" means for
every bf16 workload: values are drawn in fp32, rounded once, and that rounded
value is what both sides see.
"""
from __future__ import annotations

import numpy as np

_MASK = np.uint64(0xFFFFFFFFFFFFFFFF)


def _mix64(x: np.ndarray) -> np.ndarray:
    """The splitmix64 output function (public-domain finaliser), vectorised."""
    x = x.astype(np.uint64, copy=True)
    with np.errstate(over="ignore"):
        x += np.uint64(0x9E3779B97F4A7C15)
        x ^= x >> np.uint64(30)
        x *= np.uint64(0xBF58476D1CE4E5B9)
        x ^= x >> np.uint64(27)
        x *= np.uint64(0x94D049BB133111EB)
        x ^= x >> np.uint64(31)
    return x


def uniform_bits(seed: int, tensor_id: int, start: int, count: int) -> np.ndarray:
    """64 pseudo-random bits per element for flat indices start..start+count-1."""
    with np.errstate(over="ignore"):
        key = _mix64(np.array([seed & 0xFFFFFFFFFFFFFFFF], dtype=np.uint64))
        key = _mix64(key ^ np.uint64(tensor_id & 0xFFFFFFFFFFFFFFFF))
        idx = np.arange(start, start + count, dtype=np.uint64)
        return _mix64(idx * np.uint64(0xD1342543DE82EF95) + key[0])


def normal(seed: int, tensor_id: int, shape, start: int = 0) -> np.ndarray:
    """i.i.d. N(0,1) values in fp64, shape ``shape``, element i <- counter start+i."""
    count = int(np.prod(shape)) if len(shape) else 1
    out = np.empty(count, dtype=np.float64)
    chunk = 1 << 22
    for c0 in range(0, count, chunk):
        n = min(chunk, count - c0)
        bits = uniform_bits(seed, tensor_id, start + c0, n)
        # Two 32-bit halves -> two uniforms; u1 in (0,1], u2 in [0,1).
        hi = (bits >> np.uint64(32)).astype(np.float64)
        lo = (bits & np.uint64(0xFFFFFFFF)).astype(np.float64)
        u1 = (hi + 1.0) / 4294967296.0
        u2 = lo / 4294967296.0
        out[c0:c0 + n] = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)
    return out.reshape(shape)


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round fp32/fp64 values to the nearest bf16 (ties to even); returns fp32
    holding exactly-representable bf16 values."""
    f = np.ascontiguousarray(x, dtype=np.float32)
    u = f.view(np.uint32).astype(np.uint64)
    rounded = ((u + np.uint64(0x7FFF) + ((u >> np.uint64(16)) & np.uint64(1)))
               & np.uint64(0xFFFF0000)).astype(np.uint32)
    return rounded.view(np.float32).reshape(f.shape)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of values that are already bf16-representable."""
    f = np.ascontiguousarray(x, dtype=np.float32)
    return (f.view(np.uint32) >> np.uint32(16)).astype(np.uint16).reshape(f.shape)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen uint16 bf16 bit patterns to fp32."""
    u = np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).reshape(b.shape)


def normal_as(seed: int, tensor_id: int, shape, dtype: str, start: int = 0) -> np.ndarray:
    """N(0,1) drawn in fp64, rounded once to ``dtype`` ("bf16" or "f32"); the
    result is fp32 holding the rounded values exactly."""
    x = normal(seed, tensor_id, shape, start).astype(np.float32)
    if dtype == "bf16":
        return round_to_bf16(x)
    if dtype == "f32":
        return x
    raise ValueError(f"unknown dtype {dtype!r}")


def permutation(seed: int, tensor_id: int, n: int) -> np.ndarray:
    """A seeded permutation of 0..n-1 (argsort of hashed keys), int32."""
    keys = uniform_bits(seed, tensor_id, 0, n)
    return np.argsort(keys, kind="stable").astype(np.int32)


def integers(seed: int, tensor_id: int, n: int, lo: int, hi: int) -> np.ndarray:
    """n seeded integers uniform in [lo, hi] inclusive, int32."""
    bits = uniform_bits(seed, tensor_id, 0, n)
    span = np.uint64(hi - lo + 1)
    return (lo + (bits % span).astype(np.int64)).astype(np.int32)


def device_normal(shape, seed: int, dtype, device):
    """Bulk N(0,1) generated on ``device`` by torch's seeded generator."""
    import torch

    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    out = torch.empty(shape, dtype=dtype, device=device)
    out.normal_(0.0, 1.0, generator=g)
    return out
