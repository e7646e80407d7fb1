"""Seeded synthetic inputs shared by the CPU oracle and the HIP path.

This module holds no arithmetic of the training method: it only turns a
(global seed, tensor name) pair into reproducible arrays -- standard normal
values, uniform integer labels -- and casts them to the storage type a
workload asks for.  Both the oracle and the GPU path are handed the arrays it
returns, so neither side ever generates its own inputs.

Generator: a counter-based splitmix64 stream.  The stream for a tensor is
seeded by mixing the global seed with an FNV-1a hash of the tensor's name, so
every tensor is independent of the order in which tensors are requested.
Uniform doubles use the top 53 bits; normals use the Box-Muller transform in
fp64 on consecutive pairs of uniforms.
"""
from __future__ import annotations

import numpy as np

GLOBAL_SEED = 20250923

_GAMMA = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_MASK64 = (1 << 64) - 1


def _mix_scalar(z: int) -> int:
    z &= _MASK64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _MASK64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _MASK64
    return z ^ (z >> 31)


def name_hash(name: str) -> int:
    """FNV-1a, 64 bit, over the UTF-8 bytes of a tensor name."""
    h = 0xCBF29CE484222325
    for byte in name.encode("utf-8"):
        h ^= byte
        h = (h * 0x100000001B3) & _MASK64
    return h


def stream_seed(name: str, seed: int = GLOBAL_SEED) -> int:
    return _mix_scalar(_mix_scalar(seed) ^ name_hash(name))


def _splitmix64_words(s0: int, count: int) -> np.ndarray:
    """Words 1..count of the splitmix64 sequence whose state starts at s0 (word k mixes s0 + k*gamma)."""
    idx = np.arange(1, count + 1, dtype=np.uint64)
    with np.errstate(over="ignore"):
        z = np.uint64(s0 & _MASK64) + idx * _GAMMA
        z = (z ^ (z >> np.uint64(30))) * _M1
        z = (z ^ (z >> np.uint64(27))) * _M2
        z = z ^ (z >> np.uint64(31))
    return z


def raw_u64(name: str, count: int, seed: int = GLOBAL_SEED) -> np.ndarray:
    """`count` 64-bit words of the stream that belongs to `name`."""
    return _splitmix64_words(stream_seed(name, seed), count)


def uniform01(name: str, count: int, seed: int = GLOBAL_SEED) -> np.ndarray:
    """Uniform doubles in [0, 1) from the top 53 bits of each word."""
    return (raw_u64(name, count, seed) >> np.uint64(11)).astype(np.float64) * (1.0 / (1 << 53))


def normal(name: str, shape, std: float = 1.0, seed: int = GLOBAL_SEED) -> np.ndarray:
    """N(0, std^2) values in fp64, Box-Muller on consecutive uniform pairs."""
    shape = tuple(int(d) for d in np.atleast_1d(shape))
    count = int(np.prod(shape)) if shape else 1
    pairs = (count + 1) // 2
    u = uniform01(name, 2 * pairs, seed)
    u1 = 1.0 - u[0::2]  # (0, 1]: log is finite
    u2 = u[1::2]
    r = np.sqrt(-2.0 * np.log(u1))
    out = np.empty(2 * pairs, dtype=np.float64)
    out[0::2] = r * np.cos(2.0 * np.pi * u2)
    out[1::2] = r * np.sin(2.0 * np.pi * u2)
    return (out[:count] * std).reshape(shape)


def labels(name: str, count: int, classes: int, seed: int = GLOBAL_SEED) -> np.ndarray:
    """Uniform integer labels in [0, classes)."""
    return (raw_u64(name, count, seed) % np.uint64(classes)).astype(np.int32)


# ---------------------------------------------------------------------------
# storage casts (no method arithmetic: plain IEEE rounding)
# ---------------------------------------------------------------------------

def round_f32(x: np.ndarray) -> np.ndarray:
    """Round to fp32, return the rounded values widened back to fp64."""
    return np.asarray(x, dtype=np.float64).astype(np.float32).astype(np.float64)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp -> bfloat16 bit patterns (uint16): ONE rounding to nearest, ties to even, from the value given.

    An fp64 value is not rounded to fp32 on the way (two roundings to nearest can land one bfloat16 step
    away from the single one): it is first cut to fp32 towards zero, with the last fp32 bit set when
    anything was cut off, which keeps every case of the final rounding -- below, at or above the halfway
    point -- what it was.  NaN gives a quiet NaN of the same sign; values at or beyond the halfway point
    above the largest finite bfloat16 give infinity."""
    v = np.ascontiguousarray(np.asarray(x, dtype=np.float64))
    with np.errstate(over="ignore", invalid="ignore"):
        f = v.astype(np.float32)
        too_big = np.abs(f.astype(np.float64)) > np.abs(v)            # fp32 rounding went away from zero
        f = np.where(too_big, np.nextafter(f, np.float32(0.0)), f).astype(np.float32)
    u = np.ascontiguousarray(f).view(np.uint32).copy()
    inexact = np.isfinite(v) & (f.astype(np.float64) != v)
    u = np.where(inexact, u | np.uint32(1), u)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    with np.errstate(over="ignore"):
        rounded = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    sign = (u >> np.uint32(16)) & np.uint32(0x8000)
    rounded = np.where(np.isnan(v), sign | np.uint32(0x7FC0), rounded)
    return rounded.astype(np.uint16)


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    u = np.asarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


def round_bf16(x: np.ndarray) -> np.ndarray:
    """Round to bfloat16 (nearest even), return the values widened to fp64."""
    x = np.asarray(x)
    return bf16_bits_to_f64(bf16_bits(x)).reshape(x.shape)
