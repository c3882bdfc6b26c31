"""Counter-based generator: value i of stream s under seed z is a pure function of (z, s, i).

The mixing function is the published splitmix64 finaliser. Everything downstream is exact
integer arithmetic followed by at most one int->float32 conversion and one float32
multiply, so the numpy implementation (CPU) and the torch implementation (CPU or GPU)
produce identical bytes; tests check that.
"""
from __future__ import annotations

import numpy as np

_GOLDEN = 0x9E3779B97F4A7C15
_M1 = 0xBF58476D1CE4E5B9
_M2 = 0x94D049BB133111EB
_MASK64 = (1 << 64) - 1


def _mix_int(x: int) -> int:
    x &= _MASK64
    x ^= x >> 30
    x = (x * _M1) & _MASK64
    x ^= x >> 27
    x = (x * _M2) & _MASK64
    x ^= x >> 31
    return x


def stream_base(seed: int, stream: int) -> int:
    """64-bit offset added to the element counter for one (seed, stream) pair."""
    return _mix_int(_mix_int(seed) + ((stream + 1) * _GOLDEN))


def hash_u64(seed: int, stream: int, start: int, count: int) -> np.ndarray:
    """uint64[count]: mixed values for counters start .. start+count-1."""
    with np.errstate(over="ignore"):
        x = np.arange(start, start + count, dtype=np.uint64)
        x += np.uint64(stream_base(seed, stream))
        x ^= x >> np.uint64(30)
        x *= np.uint64(_M1)
        x ^= x >> np.uint64(27)
        x *= np.uint64(_M2)
        x ^= x >> np.uint64(31)
    return x


def uniform_tokens(seed: int, stream: int, start: int, count: int, vocab: int) -> np.ndarray:
    """int32[count] uniform over [0, vocab) (multiply-shift on the top 32 hash bits)."""
    h = hash_u64(seed, stream, start, count)
    return (((h >> np.uint64(32)) * np.uint64(vocab)) >> np.uint64(32)).astype(np.int32)


def uniform_unit(seed: int, stream: int, start: int, count: int) -> np.ndarray:
    """float64[count] uniform over [0, 1) with 53 random bits."""
    h = hash_u64(seed, stream, start, count)
    return (h >> np.uint64(11)).astype(np.float64) * (1.0 / (1 << 53))


# Sum of the four 16-bit fields of one hash word: Irwin-Hall(4), centred.  Its standard
# deviation is sqrt(4 * (65536^2 - 1) / 12); dividing by it gives a bell-shaped variate
# of unit variance supported on about +-3.46 sigma (excess kurtosis -0.3).
_IH4_STD = float(np.sqrt(4.0 * (65536.0 ** 2 - 1.0) / 12.0))


def _ih4_int(h: np.ndarray) -> np.ndarray:
    m = np.uint64(0xFFFF)
    s = (h & m) + ((h >> np.uint64(16)) & m) + ((h >> np.uint64(32)) & m) + (h >> np.uint64(48))
    return s.astype(np.int64) - 131070


def approx_normal_f32(seed: int, stream: int, start: int, count: int, std: float,
                      mean: float = 0.0) -> np.ndarray:
    """float32[count]: mean + std * (centred Irwin-Hall(4) variate of unit variance)."""
    s = _ih4_int(hash_u64(seed, stream, start, count)).astype(np.float32)
    out = s * np.float32(std / _IH4_STD)
    if mean != 0.0:
        out = out + np.float32(mean)
    return out


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of float32 values rounded to bfloat16 (nearest, ties to even)."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def round_to_bf16_f32(x: np.ndarray) -> np.ndarray:
    """float32 array holding exactly the bfloat16-rounded values of x."""
    return (bf16_bits(x).astype(np.uint32) << np.uint32(16)).view(np.float32).reshape(np.shape(x))


# ---------------------------------------------------------------------------------------
# torch twin (used to materialise multi-GB weight sets directly in device memory)
# ---------------------------------------------------------------------------------------

def _s64(c: int) -> int:
    return c - (1 << 64) if c >= (1 << 63) else c


def torch_hash_i64(seed: int, stream: int, start: int, count: int, device):
    """int64 tensor whose bit patterns equal hash_u64(seed, stream, start, count)."""
    import torch

    def lsr(t, s):
        return (t >> s) & ((1 << (64 - s)) - 1)

    x = torch.arange(start, start + count, dtype=torch.int64, device=device)
    x += _s64(stream_base(seed, stream))
    x ^= lsr(x, 30)
    x *= _s64(_M1)
    x ^= lsr(x, 27)
    x *= _s64(_M2)
    x ^= lsr(x, 31)
    return x


def torch_approx_normal(seed: int, stream: int, start: int, count: int, std: float,
                        mean: float = 0.0, device="cpu"):
    """float32 tensor equal, bit for bit, to approx_normal_f32(...)."""
    import torch

    h = torch_hash_i64(seed, stream, start, count, device)
    s = (h & 0xFFFF) + ((h >> 16) & 0xFFFF) + ((h >> 32) & 0xFFFF) + ((h >> 48) & 0xFFFF) - 131070
    out = s.to(torch.float32) * float(np.float32(std / _IH4_STD))
    if mean != 0.0:
        out = out + float(np.float32(mean))
    return out
