"""Exact widening of the stored number formats to fp64 (oracle side).

bf16: the upper 16 bits of an IEEE-754 binary32.
e4m3: OCP 8-bit float "E4M3" (finite-only variant): 1 sign bit, 4 exponent bits
with bias 7, 3 mantissa bits; exponent field 0 is subnormal (value m/8 * 2^-6);
codes 0x7F and 0xFF are NaN; the largest finite magnitude is 448.

Pins: tests/test_oracle_formats.py checks bf16 widening against struct packing,
hand-written e4m3 landmark values fixed by the format's definition, and every
e4m3 code against torch's independent float8_e4m3fn cast.
"""
import numpy as np


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    b = np.ascontiguousarray(bits).astype(np.uint32) << np.uint32(16)
    return b.view(np.float32).astype(np.float64)


def _e4m3_table() -> np.ndarray:
    t = np.empty(256, dtype=np.float64)
    for code in range(256):
        sign = -1.0 if code & 0x80 else 1.0
        e = (code >> 3) & 0xF
        m = code & 0x7
        if e == 0xF and m == 0x7:
            t[code] = np.nan
        elif e == 0:
            t[code] = sign * (m / 8.0) * 2.0 ** (-6)
        else:
            t[code] = sign * (1.0 + m / 8.0) * 2.0 ** (e - 7)
    return t


E4M3_TABLE = _e4m3_table()


def e4m3_codes_to_f64(codes: np.ndarray) -> np.ndarray:
    return E4M3_TABLE[np.ascontiguousarray(codes).astype(np.int64)]
