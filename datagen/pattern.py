"""numpy twin of datagen/pattern.h: the seeded payload word of a logical element.

No layout or routing arithmetic: (seed, kind, tensor id, global linear index) -> word.
"""
import numpy as np

_M64 = (1 << 64) - 1


def mix64(seed, kind, tensor, linear):
    """Vectorised over ``linear`` (array of uint64).  Returns uint64."""
    lin = np.asarray(linear, dtype=np.uint64)
    with np.errstate(over="ignore"):
        z = np.uint64(seed & _M64) ^ (np.uint64(0x9E3779B97F4A7C15) * (lin + np.uint64(1)))
        key = ((int(tensor) << 2) | (int(kind) & 3)) * 0xD1B54A32D192ED03 & _M64
        z = z + np.uint64(key)
        z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
        return z ^ (z >> np.uint64(31))


def seed_for_rank(seed, rank_salt, rank):
    return (seed + rank_salt * (rank + 1)) & _M64


def word(seed, kind, tensor, linear):
    """uint16 for kind 0 (bf16 payload), uint32 for kinds 1..3 (fp32 payload)."""
    z = mix64(seed, kind, tensor, linear)
    if kind == 0:
        return (z & np.uint64(0xFFFF)).astype(np.uint16)
    return (z & np.uint64(0xFFFFFFFF)).astype(np.uint32)
