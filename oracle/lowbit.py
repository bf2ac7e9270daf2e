"""Meaning of the stored numbers of a low-bit target model (Sec. 4.3 sweeps 16-, 8- and 4-bit targets).

TEST INFRASTRUCTURE ONLY, like the rest of oracle/: the float64 matrices decoded here are what the
CPU oracle multiplies with when the HIP library is given 8-bit or 4-bit weights.  Nothing here is
shared with or imported by the product package; the decoders are written from the published
format definitions (OCP 8-bit floating point, OCP microscaling formats), not from the kernels.

  FP8 E4M3   1 sign bit, 4 exponent bits (bias 7), 3 mantissa bits, no infinities:
             exponent field 0 is subnormal, value = (-1)^s * (m / 8) * 2^-6;
             otherwise        value = (-1)^s * (1 + m / 8) * 2^(e - 7);
             the all-ones pattern S.1111.111 is NaN (the model's weights must not hold it).
  FP4 E2M1   1 sign bit, 2 exponent bits (bias 1), 1 mantissa bit:
             exponent field 0: value = (-1)^s * (m / 2);  otherwise (-1)^s * (1 + m / 2) * 2^(e - 1),
             i.e. magnitudes 0, 0.5, 1, 1.5, 2, 3, 4, 6.
  E8M0       a scale byte e stands for 2^(e - 127); 255 is NaN.
  MXFP4      FP4 E2M1 elements in blocks of 32 along the input axis, one E8M0 scale per block.

Pins (tests/test_oracle_lowbit.py): every one of the 256 FP8 bytes against torch's float8_e4m3fn
widening (a library routine that shares nothing with this file), the sixteen FP4 codes and sample
scale bytes against the values the format documents print (tests/golden/ocp_lowbit_formats.txt).
"""
from __future__ import annotations

import numpy as np


def decode_fp8_e4m3(b: np.ndarray) -> np.ndarray:
    """uint8 bytes -> float64 values of OCP FP8 E4M3 (NaN for the two all-ones patterns)."""
    b = np.asarray(b, dtype=np.uint8).astype(np.int64)
    sign = np.where(b & 0x80, -1.0, 1.0)
    e = (b >> 3) & 0xF
    m = (b & 0x7).astype(np.float64)
    sub = m / 8.0 * 2.0 ** -6
    nor = (1.0 + m / 8.0) * np.ldexp(1.0, (e - 7).astype(np.int64))
    v = sign * np.where(e == 0, sub, nor)
    return np.where((b & 0x7F) == 0x7F, np.nan, v)


def decode_fp4_e2m1(c: np.ndarray) -> np.ndarray:
    """4-bit codes (0..15, bit 3 = sign) -> float64 values of OCP FP4 E2M1."""
    c = np.asarray(c).astype(np.int64)
    sign = np.where(c & 0x8, -1.0, 1.0)
    e = (c >> 1) & 0x3
    m = (c & 0x1).astype(np.float64)
    return sign * np.where(e == 0, m / 2.0, (1.0 + m / 2.0) * np.ldexp(1.0, (e - 1).astype(np.int64)))


def decode_e8m0(e: np.ndarray) -> np.ndarray:
    """scale bytes -> 2^(e - 127) as float64 (NaN for 255)."""
    e = np.asarray(e, dtype=np.uint8).astype(np.int64)
    return np.where(e == 255, np.nan, np.ldexp(1.0, e - 127))


def dequant_fp8_rows(q_bytes: np.ndarray, row_scale: np.ndarray) -> np.ndarray:
    """W[n, k] = fp8(q_bytes[n, k]) * row_scale[n]: weight-only FP8 with one scale per output row."""
    return decode_fp8_e4m3(q_bytes) * np.asarray(row_scale, dtype=np.float64)[:, None]


def dequant_mxfp4(packed: np.ndarray, scale_bytes: np.ndarray) -> np.ndarray:
    """packed[n, K/2]: two codes per byte, the even input index in the low nibble; scale_bytes[n, K/32].
    W[n, k] = fp4(code[n, k]) * 2^(scale_bytes[n, k // 32] - 127)."""
    packed = np.asarray(packed, dtype=np.uint8)
    n, half = packed.shape
    codes = np.empty((n, 2 * half), dtype=np.uint8)
    codes[:, 0::2] = packed & 0xF
    codes[:, 1::2] = packed >> 4
    vals = decode_fp4_e2m1(codes).reshape(n, -1, 32)
    return (vals * decode_e8m0(scale_bytes)[:, :, None]).reshape(n, 2 * half)
