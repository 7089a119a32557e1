"""Counter-based Gaussian generator: splitmix64 -> Box-Muller.

Element i of a tensor drawn with seed s uses the two 64-bit words
splitmix64(s + 2i) and splitmix64(s + 2i + 1); the result therefore does not
depend on chunking or on the order tensors are generated in.
"""
import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)


def _splitmix64(counter):
    """Finaliser of splitmix64 applied to (counter+1)*golden, vectorised."""
    with np.errstate(over="ignore"):
        z = (counter + np.uint64(1)) * _GOLDEN
        z = (z ^ (z >> np.uint64(30))) * _M1
        z = (z ^ (z >> np.uint64(27))) * _M2
        z = z ^ (z >> np.uint64(31))
    return z


def _unit_open(bits):
    """Map 64 random bits to a double in (0, 1]."""
    return ((bits >> np.uint64(11)).astype(np.float64) + 1.0) * (1.0 / 9007199254740992.0)


def _fill(out, base, lo, hi, sigma):
    idx = np.arange(lo, hi, dtype=np.uint64)
    with np.errstate(over="ignore"):
        c0 = base + idx * np.uint64(2)
    u1 = _unit_open(_splitmix64(c0))
    u2 = _unit_open(_splitmix64(c0 + np.uint64(1)))
    z = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)
    out[lo:hi] = (z * sigma).astype(np.float32)


def normal(seed, n, sigma=1.0, chunk=1 << 20):
    """n samples of N(0, sigma^2) as float32 (generated in float64, then cast)."""
    out = np.empty(n, dtype=np.float32)
    base = np.uint64((int(seed) * 0x100000001B3) & 0xFFFFFFFFFFFFFFFF)
    spans = [(lo, min(n, lo + chunk)) for lo in range(0, n, chunk)]
    workers = min(8, os.cpu_count() or 1, len(spans))
    if workers <= 1:
        for lo, hi in spans:
            _fill(out, base, lo, hi, sigma)
    else:
        with ThreadPoolExecutor(workers) as ex:
            list(ex.map(lambda s: _fill(out, base, s[0], s[1], sigma), spans))
    return out


def to_bf16_bits(x_f32):
    """Round float32 to bfloat16 (round-to-nearest-even); returns uint16 bit patterns."""
    u = np.ascontiguousarray(x_f32, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits_u16):
    """Widen bfloat16 bit patterns back to float32 (exact)."""
    return (bits_u16.astype(np.uint32) << np.uint32(16)).view(np.float32)


def quantize(x_f32, dtype):
    """Value an input takes once stored in `dtype` ('f32' or 'bf16'), as float32."""
    if dtype == "f32":
        return np.ascontiguousarray(x_f32, dtype=np.float32)
    if dtype == "bf16":
        return bf16_bits_to_f32(to_bf16_bits(x_f32)).reshape(np.shape(x_f32))
    raise ValueError(dtype)
