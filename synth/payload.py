"""Seeded synthetic payload values.

Everything is drawn from numpy's Philox (a counter-based generator) keyed by
``(seed, stream)``, so a buffer is reproducible from two integers.  No function
here adds, rounds or compares payload values the way the data path does: bf16
bit patterns are produced by TRUNCATING an fp32 draw (dropping its low 16 bits),
never by the round-to-nearest-even step the reduction uses.
"""
import numpy as np
from numpy.random import Generator, Philox


def rng(seed: int, stream: int) -> Generator:
    return Generator(Philox(key=[int(seed) & (2**64 - 1), int(stream) & (2**64 - 1)]))


def uniform_f32(seed: int, stream: int, n: int) -> np.ndarray:
    """n fp32 values, uniform on [-1, 1)."""
    x = rng(seed, stream).random(int(n), dtype=np.float32)
    x *= np.float32(2.0)
    x -= np.float32(1.0)
    return x


def normal_bf16(seed: int, stream: int, n: int) -> np.ndarray:
    """n bf16 bit patterns (uint16): normal(0,1) fp32 draws with the low 16 bits dropped."""
    g = rng(seed, stream)
    out = np.empty(int(n), dtype=np.uint16)
    blk = 1 << 24
    for lo in range(0, int(n), blk):
        hi = min(int(n), lo + blk)
        x = g.standard_normal(hi - lo, dtype=np.float32)
        out[lo:hi] = (x.view(np.uint32) >> np.uint32(16)).astype(np.uint16)
    return out


def uniform_bf16(seed: int, stream: int, n: int) -> np.ndarray:
    """n bf16 bit patterns: uniform[-1,1) fp32 draws with the low 16 bits dropped."""
    x = uniform_f32(seed, stream, n)
    return (x.view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def small_int(seed: int, stream: int, n: int, lo: int = -8, hi: int = 8) -> np.ndarray:
    """n int64 values uniform on {lo..hi}; callers encode them with ints_as()."""
    return rng(seed, stream).integers(lo, hi + 1, int(n), dtype=np.int64)


def ints_as(values: np.ndarray, dtype_code: int) -> np.ndarray:
    """Encode small integers (|v| <= 256) exactly as fp32 values or bf16 bit patterns.

    Integers of at most 8 significant bits have an fp32 encoding whose low 16
    bits are zero, so taking the high half is an exact conversion, not a rounding.
    """
    f = np.asarray(values).astype(np.float32)
    if dtype_code == 0:
        return f
    if dtype_code == 3:
        return np.asarray(values).astype(np.int32)
    if dtype_code == 2:
        h = f.astype(np.float16)
        assert np.array_equal(h.astype(np.float32), f), "value not exactly representable in binary16"
        return h.view(np.uint16)
    bits = f.view(np.uint32)
    assert not np.any(bits & np.uint32(0xFFFF)), "value not exactly representable in bf16"
    return (bits >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns (for printing / integer checks in tests)."""
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def uniform_f16(seed: int, stream: int, n: int, scale: float = 1.0) -> np.ndarray:
    """n binary16 bit patterns (uint16): uniform[-scale, scale) fp32 draws converted by numpy."""
    return (uniform_f32(seed, stream, n) * np.float32(scale)).astype(np.float16).view(np.uint16)


def uniform_i32(seed: int, stream: int, n: int, lo: int = -(1 << 31), hi: int = (1 << 31) - 1) -> np.ndarray:
    """n int32 values uniform on {lo..hi} (full range by default, so sums and products wrap)."""
    return rng(seed, stream).integers(lo, hi + 1, int(n), dtype=np.int64).astype(np.int32)


def np_dtype(dtype_code: int):
    """Storage dtype of a buffer holding elements of the given ABI dtype code
    (0 fp32, 1 bf16 bits, 2 binary16 bits, 3 int32)."""
    return {0: np.float32, 1: np.uint16, 2: np.uint16, 3: np.int32}[dtype_code]
