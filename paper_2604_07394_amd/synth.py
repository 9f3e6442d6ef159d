"""Seeded synthetic inputs for the Flux Attention hot path (test and bench infrastructure).

This module holds no attention or router arithmetic.  It is a counter-based
random generator: every element of every synthetic tensor is a pure function of
``(seed, stream, counter)``, so any row of a tensor far too large for host
memory (a 137 GB KV cache) can be regenerated on the host on demand.

The same generator exists twice, bit for bit:

* here, in NumPy (host side, feeds the CPU oracle and small GPU cases);
* in ``csrc/synth_fill.hip`` (device side, fills large tensors in place).

To make the two agree bit-exactly the transform from hash bits to a Gaussian
uses only operations that IEEE-754 fixes completely and that every
implementation rounds alike: integer arithmetic, int->float conversion of
values below 2**24, and single fp32 ``+ - *`` roundings in a fixed order (no
fused multiply-add, no division, no ``sqrt``, no library ``log``/``cos``: a GPU
may round those differently in the last bit).  ``ln`` is evaluated with the
atanh series on a reduced mantissa, its reciprocal and the square root with
Newton iterations from fixed starting values, and ``cos`` with a Taylor
polynomial on one quadrant; all are accurate to a few 1e-7, far below the bf16
rounding applied afterwards.

Distribution: ``hash -> (u1, u2)`` two 24-bit uniforms, Box-Muller
``z = sqrt(-2 ln u1) * cos(2 pi u2)`` (one normal per counter).
"""
from __future__ import annotations

import numpy as np

_MASK64 = (1 << 64) - 1
_GOLDEN = 0x9E3779B97F4A7C15
_MIX1 = 0xBF58476D1CE4E5B9
_MIX2 = 0x94D049BB133111EB

f32 = np.float32

# atanh-series coefficients for ln(m) = s * (2 + 2/3 s^2 + 2/5 s^4 + 2/7 s^6 + 2/9 s^8)
_LN_C = [f32(2.0 / 9.0), f32(2.0 / 7.0), f32(2.0 / 5.0), f32(2.0 / 3.0), f32(2.0)]
_LN2 = f32(0.6931471805599453)
_SQRT2 = f32(1.4142135623730951)
# Taylor coefficients in theta^2 on [0, pi/2)
_SIN_C = [f32(-1.0 / 39916800.0), f32(1.0 / 362880.0), f32(-1.0 / 5040.0),
          f32(1.0 / 120.0), f32(-1.0 / 6.0), f32(1.0)]
_COS_C = [f32(1.0 / 479001600.0), f32(-1.0 / 3628800.0), f32(1.0 / 40320.0),
          f32(-1.0 / 720.0), f32(1.0 / 24.0), f32(-0.5), f32(1.0)]
_QUARTER_TURN = f32(1.5707963267948966 / 4194304.0)  # (pi/2) / 2**22
_TWO_M24 = f32(1.0 / 16777216.0)


def _mix_int(z: int) -> int:
    z &= _MASK64
    z = ((z ^ (z >> 30)) * _MIX1) & _MASK64
    z = ((z ^ (z >> 27)) * _MIX2) & _MASK64
    return z ^ (z >> 31)


def stream_key(seed: int, stream: int) -> int:
    """64-bit key of one tensor: a splitmix64 finalisation of ``seed:stream``."""
    return _mix_int(((int(seed) & 0xFFFFFFFF) << 32) | (int(stream) & 0xFFFFFFFF))


def hash_u64(seed: int, stream: int, counter) -> np.ndarray:
    """splitmix64 output number ``counter`` of the sequence started at ``stream_key``."""
    c = np.asarray(counter, dtype=np.uint64)
    with np.errstate(over="ignore"):
        z = c * np.uint64(_GOLDEN) + np.uint64(stream_key(seed, stream))
        z = (z ^ (z >> np.uint64(30))) * np.uint64(_MIX1)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(_MIX2)
        z = z ^ (z >> np.uint64(31))
    return z


def _horner(coeffs, x):
    acc = np.full_like(x, coeffs[0])
    for c in coeffs[1:]:
        acc = acc * x          # one fp32 rounding
        acc = acc + c          # one fp32 rounding
    return acc


def _recip_1p7_2p5(d):
    """1/d for d in (1.7, 2.5) by Newton's iteration on d/4 (multiplies and adds only)."""
    dq = d * f32(0.25)
    y = f32(48.0 / 17.0) - f32(32.0 / 17.0) * dq
    for _ in range(4):
        e = f32(1.0) - dq * y
        y = y + y * e
    return y * f32(0.25)


def _sqrt_newton(x):
    """sqrt(x) for x >= 0 as x * rsqrt(x): bit-level first guess, four Newton steps on rsqrt."""
    xb = np.ascontiguousarray(x, dtype=f32).view(np.uint32)
    y = (np.uint32(0x5F3759DF) - (xb >> np.uint32(1))).view(f32)
    for _ in range(4):
        t = x * y
        t = t * y
        t = f32(1.5) - f32(0.5) * t
        y = y * t
    return x * y


def uniform_f32(seed: int, stream: int, counter, lo: float = 0.0, hi: float = 1.0) -> np.ndarray:
    """``lo + (hi-lo) * k/2**24`` with ``k`` the top 24 hash bits (fp32, two roundings)."""
    h = hash_u64(seed, stream, counter)
    k = (h >> np.uint64(40)).astype(np.uint32).astype(f32)
    u = k * _TWO_M24
    return f32(lo) + (f32(hi) - f32(lo)) * u


def normal_f32(seed: int, stream: int, counter) -> np.ndarray:
    """Standard normal samples (fp32) for the given counters."""
    h = hash_u64(seed, stream, counter)
    k1 = (h >> np.uint64(40)).astype(np.uint32)                       # 24 bits
    k2 = ((h >> np.uint64(16)) & np.uint64(0xFFFFFF)).astype(np.uint32)  # 24 bits

    # ---- -ln(u1), u1 = (k1+1) / 2**24 in (0, 1]
    x = (k1 + np.uint32(1)).astype(f32)                 # exact: <= 2**24
    bits = x.view(np.uint32)
    e = (bits >> np.uint32(23)).astype(np.int32) - np.int32(127)
    m = ((bits & np.uint32(0x7FFFFF)) | np.uint32(0x3F800000)).view(f32)   # [1, 2)
    big = m > _SQRT2
    m = np.where(big, m * f32(0.5), m)                  # (sqrt(.5), sqrt(2)]
    e = e + big.astype(np.int32)
    s = (m - f32(1.0)) * _recip_1p7_2p5(m + f32(1.0))
    s2 = s * s
    ln_m = s * _horner(_LN_C, s2)
    neg_ln = (np.int32(24) - e).astype(f32) * _LN2 - ln_m
    neg_ln = np.maximum(neg_ln, f32(0.0))
    r = _sqrt_newton(neg_ln + neg_ln)

    # ---- cos(2 pi u2), u2 = k2 / 2**24: quadrant from the top two bits
    quad = k2 >> np.uint32(22)
    theta = (k2 & np.uint32(0x3FFFFF)).astype(f32) * _QUARTER_TURN     # [0, pi/2)
    t2 = theta * theta
    sin_t = theta * _horner(_SIN_C, t2)
    cos_t = _horner(_COS_C, t2)
    c = np.where(quad == 0, cos_t, np.where(quad == 1, -sin_t, np.where(quad == 2, -cos_t, sin_t)))
    return (r * c).astype(f32)


def f32_to_bf16_bits(x) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16, returned as uint16 bit patterns."""
    b = np.ascontiguousarray(x, dtype=f32).view(np.uint32)
    b = b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))
    return (b >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b) -> np.ndarray:
    return (np.asarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(f32)


def normal_bf16(seed: int, stream: int, shape, scale=None, scale_axis: int | None = None,
                counter0: int = 0) -> np.ndarray:
    """A whole tensor of N(0,1) (times an optional per-index scale), as bf16 bit patterns.

    The counter of an element is ``counter0`` + its row-major flat index in
    ``shape``.  ``scale`` (fp32, length ``shape[scale_axis]``) multiplies the
    fp32 sample once before the bf16 rounding.
    """
    shape = tuple(int(s) for s in shape)
    n = int(np.prod(shape, dtype=np.int64)) if shape else 1
    z = normal_f32(seed, stream, np.arange(n, dtype=np.uint64) + np.uint64(counter0)).reshape(shape)
    if scale is not None:
        sc = np.asarray(scale, dtype=f32)
        bshape = [1] * len(shape)
        bshape[scale_axis] = shape[scale_axis]
        z = z * sc.reshape(bshape)
    return f32_to_bf16_bits(z).reshape(shape)


def normal_bf16_rows(seed: int, stream: int, logical_shape, lead_index, row0: int, row1: int,
                     scale: float | None = None) -> np.ndarray:
    """Rows ``row0:row1`` of the 2-D slab ``tensor[lead_index]`` of a tensor of ``logical_shape``.

    ``logical_shape = (*lead, n_rows, width)``; ``lead_index`` indexes the
    leading axes.  Used to regenerate one (batch, kv-head) stretch of a cache
    without materialising the rest.
    """
    *lead, n_rows, width = (int(s) for s in logical_shape)
    flat = 0
    for dim, idx in zip(lead, lead_index):
        flat = flat * dim + int(idx)
    base = (flat * n_rows + int(row0)) * width
    n = (int(row1) - int(row0)) * width
    z = normal_f32(seed, stream, np.arange(n, dtype=np.uint64) + np.uint64(base))
    if scale is not None:
        z = z * f32(scale)
    return f32_to_bf16_bits(z).reshape(int(row1) - int(row0), width)


def head_scales(seed: int, stream: int, n: int, lo: float = 0.5, hi: float = 2.0) -> np.ndarray:
    """``n`` per-head scale factors ~ U(lo, hi), fp32."""
    return uniform_f32(seed, stream, np.arange(n, dtype=np.uint64), lo, hi)


# Stream ids: one per synthetic tensor family; the layer (and decode step) is folded in.
STREAM_Q, STREAM_K, STREAM_V = 1, 2, 3
STREAM_QSCALE, STREAM_KSCALE, STREAM_VSCALE = 4, 5, 6
STREAM_X, STREAM_W1, STREAM_W2, STREAM_B1, STREAM_B2 = 7, 8, 9, 10, 11
STREAM_MASK = 12
STREAM_QDEC, STREAM_KDEC, STREAM_VDEC = 13, 14, 15


def stream_id(kind: int, layer: int = 0, step: int = 0) -> int:
    """Pack (tensor family, layer, decode step) into the 32-bit stream id."""
    return (int(kind) << 24) | ((int(layer) & 0xFF) << 16) | (int(step) & 0xFFFF)


def random_layer_mask(seed: int, n_layers: int, n_sa: int) -> np.ndarray:
    """uint8[n_layers], 1 = FA, 0 = SA, with exactly ``n_sa`` SA layers chosen uniformly.

    The layers with the ``n_sa`` smallest hash values become SA.
    """
    h = hash_u64(seed, stream_id(STREAM_MASK), np.arange(n_layers, dtype=np.uint64))
    order = np.argsort(h, kind="stable")
    mask = np.ones(n_layers, dtype=np.uint8)
    mask[order[:n_sa]] = 0
    return mask
