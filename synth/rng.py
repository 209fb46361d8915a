"""Counter-based random draws: value i of stream (seed, stream) depends on (seed, stream, i) only.

The generator is the SplitMix64 output function (Steele, Lea, Flood 2014: add the golden-gamma
constant, then two xor-shift-multiply rounds and a final xor-shift) applied to a counter, so
any element can be produced on its own, in any order, by numpy here or by any other
implementation of the same three lines.  Nothing depends on numpy's or torch's own generators.
"""
import numpy as np

_GAMMA = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)


def splitmix64(x):
    """SplitMix64 finaliser of the uint64 array ``x`` (wrapping arithmetic)."""
    with np.errstate(over="ignore"):
        z = (np.asarray(x, dtype=np.uint64) + _GAMMA)
        z = (z ^ (z >> np.uint64(30))) * _M1
        z = (z ^ (z >> np.uint64(27))) * _M2
        return z ^ (z >> np.uint64(31))


def _raw(seed, stream, count, offset=0):
    """uint64 draws for counters offset .. offset+count-1 of stream (seed, stream)."""
    with np.errstate(over="ignore"):
        key = splitmix64(np.uint64(seed) * np.uint64(0x100000001B3) + np.uint64(stream))
        ctr = np.arange(offset, offset + count, dtype=np.uint64)
        return splitmix64(key + ctr * _GAMMA)


def uniform_pm1(seed, stream, shape):
    """float32 i.i.d. uniform on [-1, 1): top 24 bits of each draw, so every value is exact."""
    n = int(np.prod(shape, dtype=np.int64))
    u24 = (_raw(seed, stream, n) >> np.uint64(40)).astype(np.float64)
    return (u24 * (2.0 / 16777216.0) - 1.0).astype(np.float32).reshape(shape)


def normal(seed, stream, shape, sigma=1.0):
    """float32 i.i.d. N(0, sigma^2): Box-Muller in float64 on pairs of draws, rounded once."""
    n = int(np.prod(shape, dtype=np.int64))
    m = (n + 1) // 2
    r = _raw(seed, stream, 2 * m)
    # u1 in (0, 1], u2 in [0, 1): 53-bit fractions
    u1 = ((r[0::2] >> np.uint64(11)).astype(np.float64) + 1.0) * (1.0 / 9007199254740992.0)
    u2 = (r[1::2] >> np.uint64(11)).astype(np.float64) * (1.0 / 9007199254740992.0)
    rad = np.sqrt(-2.0 * np.log(u1))
    z = np.empty(2 * m, dtype=np.float64)
    z[0::2] = rad * np.cos(2.0 * np.pi * u2)
    z[1::2] = rad * np.sin(2.0 * np.pi * u2)
    return (z[:n] * float(sigma)).astype(np.float32).reshape(shape)


def small_ints(seed, stream, shape, lo=-3, hi=3):
    """float32 array of i.i.d. integers in [lo, hi]; sums of products of these stay exact in
    fp32 as long as (reduction length) * max|a| * max|b| < 2**24."""
    n = int(np.prod(shape, dtype=np.int64))
    span = np.uint64(hi - lo + 1)
    v = (_raw(seed, stream, n) >> np.uint64(33)) % span
    return (v.astype(np.int64) + lo).astype(np.float32).reshape(shape)


def to_bf16_bits(x):
    """Round float32 to bfloat16 (round to nearest, ties to even); returns the uint16 patterns.
    Inputs are finite, so no NaN handling is needed."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounding = np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))
    return ((b + rounding) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits):
    """Widen bfloat16 patterns exactly to float32."""
    return (np.asarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)
