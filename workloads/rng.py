"""Counter-based random numbers that do not depend on any library's generator.

Element ``i`` of a stream with seed ``s`` is a pure function of ``(s, i)``:
a SplitMix64 finaliser applied to ``s + (i + 1) * golden``.  Uniform doubles
use the top 53 bits; normal deviates use the Box-Muller transform on two
independent streams.  The values are therefore stable across numpy / torch
versions and can be regenerated element by element.

bfloat16 helpers here only change the *storage format* of generated inputs
(round-to-nearest-even to 8 significant bits) so that the CPU oracle and the
GPU path are handed exactly the same stored values.
"""

import numpy as np

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)


def _mix(z: np.ndarray) -> np.ndarray:
    with np.errstate(over="ignore"):
        z = (z ^ (z >> np.uint64(30))) * _M1
        z = (z ^ (z >> np.uint64(27))) * _M2
        z = z ^ (z >> np.uint64(31))
    return z


def _unit(seed: int, n: int, stream: int) -> np.ndarray:
    """n doubles in [0, 1): element i of sub-stream ``stream`` of ``seed``."""
    with np.errstate(over="ignore"):
        base = _mix(np.array([np.uint64(seed) * np.uint64(2) + np.uint64(stream)],
                             dtype=np.uint64))[0]
        ctr = (np.arange(1, n + 1, dtype=np.uint64)) * _GOLDEN + base
    bits = _mix(ctr) >> np.uint64(11)
    return bits.astype(np.float64) * (1.0 / 9007199254740992.0)


def uniform(seed: int, shape, lo: float = 0.0, hi: float = 1.0) -> np.ndarray:
    n = int(np.prod(shape))
    return (lo + (hi - lo) * _unit(seed, n, 0)).reshape(shape)


def normal(seed: int, shape, std: float = 1.0) -> np.ndarray:
    n = int(np.prod(shape))
    u1 = 1.0 - _unit(seed, n, 0)          # (0, 1]
    u2 = _unit(seed, n, 1)
    z = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)
    return (std * z).reshape(shape)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp64/fp32 values to bfloat16 (nearest even); return uint16 bit patterns."""
    f = np.ascontiguousarray(x, dtype=np.float32)
    u = f.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    with np.errstate(over="ignore"):
        r = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_from_bits(b: np.ndarray) -> np.ndarray:
    """uint16 bfloat16 bit patterns -> float64 values (exact)."""
    u = b.astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Values of x rounded to the nearest bfloat16, returned as float64."""
    return bf16_from_bits(bf16_bits(x)).reshape(np.shape(x))
