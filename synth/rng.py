"""Counter-based Gaussian generator: element i of a named tensor depends only on
(seed, name, i), so any two code bases that implement these few lines produce the same
tensor without exchanging data.

    key  = mix(seed XOR (fnv1a64(name) * PHI64))
    z    = mix(key + i)
    u1   = ((z >> 40) + 1) / 2^24          in (0, 1]
    u2   = ((z >> 16) & 0xFFFFFF) / 2^24   in [0, 1)
    g    = sqrt(-2 ln u1) * cos(2 pi u2)   (float64 arithmetic)
    out  = float32(float64(float32(std)) * g), optionally rounded to bf16 (nearest-even)

mix(x) is the splitmix64 output function applied to x + PHI64.
"""
import os

import numpy as np

PHI64 = 0x9E3779B97F4A7C15
_M64 = (1 << 64) - 1


def fnv1a64(name: str) -> int:
    h = 0xCBF29CE484222325
    for b in name.encode("ascii"):
        h ^= b
        h = (h * 0x100000001B3) & _M64
    return h


def _mix_int(x: int) -> int:
    z = (x + PHI64) & _M64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _M64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _M64
    return z ^ (z >> 31)


def _mix_vec(x: np.ndarray) -> np.ndarray:
    z = x + np.uint64(PHI64)
    z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
    z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
    return z ^ (z >> np.uint64(31))


def tensor_key(seed: int, name: str) -> int:
    return _mix_int((seed & _M64) ^ ((fnv1a64(name) * PHI64) & _M64))


def _gaussian_chunk(key, out, lo, hi, start, std):
    with np.errstate(over="ignore"):
        idx = np.arange(start + lo, start + hi, dtype=np.uint64)
        z = _mix_vec(key + idx)
        u1 = ((z >> np.uint64(40)).astype(np.float64) + 1.0) * (1.0 / 16777216.0)
        u2 = ((z >> np.uint64(16)) & np.uint64(0xFFFFFF)).astype(np.float64) * (1.0 / 16777216.0)
        g = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)
        out[lo:hi] = (float(np.float32(std)) * g).astype(np.float32)


def gaussian(seed: int, name: str, n: int, std: float = 1.0, start: int = 0) -> np.ndarray:
    """float32 array of n values, elements start..start+n-1 of tensor `name`."""
    key = np.uint64(tensor_key(seed, name))
    out = np.empty(n, dtype=np.float32)
    chunk = 1 << 20
    spans = [(lo, min(n, lo + chunk)) for lo in range(0, n, chunk)]
    if len(spans) <= 2:
        for lo, hi in spans:
            _gaussian_chunk(key, out, lo, hi, start, std)
    else:   # NumPy releases the GIL inside its loops, so threads scale
        from concurrent.futures import ThreadPoolExecutor
        with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as ex:
            list(ex.map(lambda s: _gaussian_chunk(key, out, s[0], s[1], start, std), spans))
    return out


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit patterns (uint16), round-to-nearest-even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (r >> np.uint32(16)).astype(np.uint16)


def bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_bf16(x: np.ndarray) -> np.ndarray:
    """float32 values rounded to the nearest bf16-representable float32."""
    return bits_to_f32(bf16_bits(x)).reshape(np.shape(x))


def gaussian_bf16(seed: int, name: str, n: int, std: float = 1.0) -> np.ndarray:
    """As `gaussian`, then rounded to bf16; returned as float32 holding bf16 values."""
    return round_bf16(gaussian(seed, name, n, std))
