"""Storage formats -> fp64, from the formats' definitions (oracle side).

bf16 is the upper half of an IEEE binary32.  fp8 e4m3fn is the OCP 8-bit format
with 1 sign, 4 exponent (bias 7) and 3 mantissa bits, no infinities, the single
NaN mantissa-exponent pattern S.1111.111, and a largest finite value of 448.
"""
import numpy as np


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    u = np.asarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    with np.errstate(invalid="ignore"):          # signalling-NaN patterns are data here
        return u.view(np.float32).astype(np.float64)


def _e4m3_value(byte: int) -> float:
    sign = -1.0 if byte & 0x80 else 1.0
    exp = (byte >> 3) & 0xF
    man = byte & 0x7
    if exp == 0xF and man == 0x7:
        return float("nan")
    if exp == 0:
        return sign * (man / 8.0) * 2.0 ** (-6)
    return sign * (1.0 + man / 8.0) * 2.0 ** (exp - 7)


E4M3_TABLE = np.array([_e4m3_value(b) for b in range(256)], dtype=np.float64)


def e4m3_bytes_to_f64(b: np.ndarray) -> np.ndarray:
    return E4M3_TABLE[np.asarray(b, dtype=np.uint8)]
