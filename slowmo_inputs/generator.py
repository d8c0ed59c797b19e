"""Counter-based seeded input generator (host side, NumPy).

The stochastic gradients of Section 2 (Eq. (1): worker i draws a sample and
evaluates its gradient) are replaced by synthetic values: the hot path only
moves and combines them, so any reproducible stream of the right scale does.

A value is a pure function of (seed, worker, step, global element index):

    key   = mix64( mix64(seed + G*(worker+1)) ^ (S*(step+1)) )
    w_l   = mix64( key + G*(3*index + l + 1) ),  l = 0, 1, 2
    k_0..k_11 = the twelve 16-bit fields of (w_0, w_1, w_2)
    n     = (sum k_r - 393210) / 65536           (393210 = 12 * 32767.5)

mix64 is the SplitMix64 output function.  n is an Irwin-Hall(12) variate:
mean 0, variance 1 - 2**-32, support (-6, 6).  The integer sum is below 2**24
and the divisor is a power of two, so n is exactly representable in fp32 and
is the same bit pattern on every platform: no transcendental function is
evaluated.  A gradient is the single fp32 product sigma * n; a bf16 gradient
is that product rounded to nearest-even by integer arithmetic.

The device generator (csrc/gradgen.hip) evaluates the same function; the two
are compared bit for bit by the tests.  This module holds none of the
optimizer's arithmetic.
"""
from __future__ import annotations

import numpy as np

_G = np.uint64(0x9E3779B97F4A7C15)      # 2**64 / golden ratio (SplitMix64 increment)
_S = np.uint64(0xD1342543DE82EF95)      # odd multiplier separating steps
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_IH_OFFSET = 393210                     # 12 * (65535 / 2)
PARAM_SEED_XOR = 0x5EED


def mix64(z):
    """SplitMix64 output function on uint64 (array or scalar), wrapping."""
    z = np.asarray(z, dtype=np.uint64)
    with np.errstate(over="ignore"):
        z = (z ^ (z >> np.uint64(30))) * _M1
        z = (z ^ (z >> np.uint64(27))) * _M2
        z = z ^ (z >> np.uint64(31))
    return z


def stream_key(seed: int, worker: int, step: int) -> np.uint64:
    with np.errstate(over="ignore"):
        a = mix64(np.uint64(seed) + _G * np.uint64(worker + 1))
        return mix64(a ^ (_S * np.uint64(step + 1)))[()]


def unit_normal(seed: int, worker: int, step: int, index) -> np.ndarray:
    """n(seed, worker, step, index) as float32, for an int64 index array."""
    idx = np.asarray(index, dtype=np.int64).astype(np.uint64)
    key = stream_key(seed, worker, step)
    total = np.zeros(idx.shape, dtype=np.int64)
    mask = np.uint64(0xFFFF)
    with np.errstate(over="ignore"):
        for lane in range(3):
            w = mix64(key + _G * (np.uint64(3) * idx + np.uint64(lane + 1)))
            for sh in (0, 16, 32, 48):
                total += ((w >> np.uint64(sh)) & mask).astype(np.int64)
    return ((total - _IH_OFFSET).astype(np.float32) / np.float32(65536.0)).astype(np.float32)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16, returned as uint16 bit patterns.
    Inputs here are finite, so NaN handling is not needed."""
    u = np.asarray(x, dtype=np.float32).view(np.uint32)
    r = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening bf16 -> fp32."""
    return (np.asarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def gradient(seed: int, worker: int, step: int, index, sigma: float,
             bf16: bool = False) -> np.ndarray:
    """Gradient values at the given global element indices, as float32.
    With bf16=True the values are bf16-representable (already rounded)."""
    g = (np.float32(sigma) * unit_normal(seed, worker, step, index)).astype(np.float32)
    if bf16:
        g = bf16_bits_to_f32(f32_to_bf16_bits(g))
    return g


def initial_params(seed: int, index, scale: float = 0.01) -> np.ndarray:
    """x_{0,0}: scale * n(seed ^ 0x5eed, worker 0, step 0, index), float32."""
    return (np.float32(scale) *
            unit_normal(seed ^ PARAM_SEED_XOR, 0, 0, index)).astype(np.float32)
