"""MXFP8 rounding for the oracle (test infrastructure, not a product path).

The paper names 8-bit multiplication only as a future direction (Section 9.1); it fixes no format.  This
build's reduced-precision mode for the prefix feed-forward GEMMs uses the public OCP Microscaling
format MXFP8: elements in FP8 E4M3 (OCP "e4m3fn": bias 7, no infinities, one NaN mantissa, largest
finite value 448), one shared power-of-two scale (E8M0, bias 127) per 32 consecutive elements of
the contraction axis.  This file is that definition written out in numpy: it shares no code with
the HIP library.  Only tests, the smoke check and the benchmark's CPU leg may import it.

Quantisation rule (OCP MX v1.0, Section 6.3): shared exponent = floor(log2(max |x|)) - 8 (8 is the
exponent of E4M3's largest power of two), elements = x / 2^shared_exponent rounded to nearest even
in E4M3, magnitudes beyond 448 saturate to 448.  A block of zeros takes the smallest scale.
"""
from __future__ import annotations

import numpy as np

E4M3_MAX = 448.0
BLOCK = 32


def e4m3_decode(codes: np.ndarray) -> np.ndarray:
    """Value of E4M3 bit patterns (uint8) as float32; 0x7f / 0xff are NaN."""
    c = codes.astype(np.int32)
    sign = np.where(c & 0x80, -1.0, 1.0)
    e = (c >> 3) & 15
    m = c & 7
    sub = np.ldexp(m.astype(np.float64), -9)                   # exponent field 0: m * 2^-9
    nor = np.ldexp(1.0 + m / 8.0, e - 7)
    v = np.where(e == 0, sub, nor)
    v = np.where((e == 15) & (m == 7), np.nan, v)
    return (sign * v).astype(np.float32)


def e4m3_encode(x: np.ndarray) -> np.ndarray:
    """Nearest E4M3 bit pattern of finite values, ties to the even mantissa, saturating at +-448."""
    x = np.asarray(x, dtype=np.float64)
    a = np.minimum(np.abs(x), E4M3_MAX)
    sign = np.where(np.signbit(x), 0x80, 0).astype(np.int32)
    # subnormal range (below 2^-6): multiples of 2^-9; the count 8 is the smallest normal, code 0x08
    q_sub = np.rint(a * 512.0).astype(np.int32)
    with np.errstate(divide="ignore"):
        e = np.floor(np.log2(np.where(a > 0, a, 1.0))).astype(np.int32)
    e = np.clip(e, -6, 8)
    m = np.rint((a / np.ldexp(1.0, e) - 1.0) * 8.0).astype(np.int32)
    carry = m == 8
    e = np.where(carry, e + 1, e)
    m = np.where(carry, 0, m)
    q_nor = ((e + 7) << 3) | m
    code = np.where(a < 2.0 ** -6, q_sub, q_nor)
    return (sign | code).astype(np.uint8)


def mx_quantize(x: np.ndarray):
    """Blocks of 32 along the last axis -> (E4M3 codes uint8 of x's shape, E8M0 scale codes uint8 [..., n/32])."""
    x = np.asarray(x, dtype=np.float64)
    assert x.shape[-1] % BLOCK == 0
    xb = x.reshape(x.shape[:-1] + (x.shape[-1] // BLOCK, BLOCK))
    amax = np.abs(xb).max(axis=-1)
    with np.errstate(divide="ignore"):
        se = np.floor(np.log2(np.where(amax > 0, amax, 1.0))).astype(np.int32) - 8
    se = np.where(amax > 0, np.clip(se, -127, 127), -127)
    codes = e4m3_encode(xb / np.ldexp(1.0, se)[..., None]).reshape(x.shape)
    return codes, (se + 127).astype(np.uint8)


def mx_dequantize(codes: np.ndarray, scales: np.ndarray, dtype=np.float32) -> np.ndarray:
    v = e4m3_decode(codes).astype(np.float64)
    vb = v.reshape(v.shape[:-1] + (v.shape[-1] // BLOCK, BLOCK))
    out = vb * np.ldexp(1.0, scales.astype(np.int32) - 127)[..., None]
    return out.reshape(v.shape).astype(dtype)


def mx_round(x: np.ndarray, dtype=None) -> np.ndarray:
    """x rounded through MXFP8 along its last axis (what a GEMM operand holds after quantisation)."""
    codes, scales = mx_quantize(x)
    return mx_dequantize(codes, scales, dtype or np.asarray(x).dtype)
