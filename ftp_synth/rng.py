"""Seeded synthetic tensor generators (inputs only; no arithmetic of the method).

Counter-based splitmix64 streams, one per named tensor, so the CPU oracle tests
and the GPU harness see byte-identical inputs without sharing anything else.
Uniform values are the top 24 bits of a draw divided by 2**24; normal values
are Box-Muller in fp64, cast to fp32 at the end.
"""
import numpy as np

MASTER_SEED = 20240909
_MASK = (1 << 64) - 1
_GOLDEN = 0x9E3779B97F4A7C15


def fnv1a64(name: str) -> int:
    h = 0xCBF29CE484222325
    for b in name.encode("utf-8"):
        h ^= b
        h = (h * 0x100000001B3) & _MASK
    return h


def tensor_seed(name: str, master_seed: int = MASTER_SEED) -> int:
    return (master_seed ^ fnv1a64(name)) & _MASK


def splitmix64(seed: int, n: int, start: int = 0) -> np.ndarray:
    """Draws start..start+n-1 of the splitmix64 stream with the given seed."""
    with np.errstate(over="ignore"):
        idx = np.arange(start + 1, start + n + 1, dtype=np.uint64)
        z = np.uint64(seed & _MASK) + idx * np.uint64(_GOLDEN)
        z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
        z = z ^ (z >> np.uint64(31))
    return z


_CHUNK = 1 << 22


def uniform01(name: str, shape, master_seed: int = MASTER_SEED) -> np.ndarray:
    """fp32 tensor uniform on [0,1)."""
    n = int(np.prod(shape))
    seed = tensor_seed(name, master_seed)
    out = np.empty(n, dtype=np.float32)
    for s in range(0, n, _CHUNK):
        m = min(_CHUNK, n - s)
        u = splitmix64(seed, m, s)
        out[s:s + m] = ((u >> np.uint64(40)).astype(np.float64) / float(1 << 24)).astype(np.float32)
    return out.reshape(shape)


def normal(name: str, shape, std: float = 1.0, master_seed: int = MASTER_SEED) -> np.ndarray:
    """fp32 tensor N(0, std^2): element 2k and 2k+1 are the cos and sin branch of pair k."""
    n = int(np.prod(shape))
    seed = tensor_seed(name, master_seed)
    out = np.empty(n + (n & 1), dtype=np.float32)
    npairs = out.size // 2
    pchunk = _CHUNK // 2
    for s in range(0, npairs, pchunk):
        m = min(pchunk, npairs - s)
        u = splitmix64(seed, 2 * m, 2 * s)
        u1 = ((u[0::2] >> np.uint64(11)).astype(np.float64) + 1.0) / float(1 << 53)   # (0,1]
        u2 = (u[1::2] >> np.uint64(11)).astype(np.float64) / float(1 << 53)           # [0,1)
        r = np.sqrt(-2.0 * np.log(u1)) * std
        out[2 * s:2 * (s + m):2] = (r * np.cos(2.0 * np.pi * u2)).astype(np.float32)
        out[2 * s + 1:2 * (s + m):2] = (r * np.sin(2.0 * np.pi * u2)).astype(np.float32)
    return out[:n].reshape(shape)


def to_bf16_rne(a: np.ndarray) -> np.ndarray:
    """Rounds fp32 values to the nearest bf16 (ties to even); returns fp32 holding those values."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    with np.errstate(over="ignore"):
        r = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    r = r & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of bf16-representable fp32 values."""
    return (np.ascontiguousarray(a, dtype=np.float32).view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def bf16_from_bits(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)
