"""Storage formats decoded in software, from their definitions.

bf16: the upper 16 bits of an IEEE-754 binary32.
e4m3 (OCP 8-bit float, "fn" flavour): 1 sign, 4 exponent bits with bias 7, 3 mantissa
bits; exponent field 0 is subnormal (mantissa/8 * 2^-6); no infinities; 0x7F and 0xFF are
NaN; largest finite magnitude 448.
"""
import numpy as np


def decode_bf16(bits):
    """uint16 bit patterns -> float64 values."""
    b = np.asarray(bits, dtype=np.uint16)
    with np.errstate(invalid="ignore"):      # signalling-NaN patterns are only ever decoded by the format tests
        return (b.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def encode_bf16_rne(x32):
    """float32 -> bf16 bits, round to nearest, ties to even (finite inputs)."""
    x32 = np.ascontiguousarray(x32, dtype=np.float32)
    u = x32.view(np.uint32).astype(np.uint64)
    low = u & np.uint64(0xFFFF)
    hi = u >> np.uint64(16)
    up = (low > np.uint64(0x8000)) | ((low == np.uint64(0x8000)) & ((hi & np.uint64(1)) == np.uint64(1)))
    return (hi + up.astype(np.uint64)).astype(np.uint16)


def _e4m3_table():
    t = np.empty(256, dtype=np.float64)
    for code in range(256):
        s = -1.0 if code & 0x80 else 1.0
        e = (code >> 3) & 0xF
        m = code & 0x7
        if e == 0xF and m == 0x7:
            v = float("nan")
        elif e == 0:
            v = s * (m / 8.0) * 2.0 ** -6
        else:
            v = s * (1.0 + m / 8.0) * 2.0 ** (e - 7)
        t[code] = v
    return t


E4M3_TABLE = _e4m3_table()


def decode_e4m3(codes):
    """uint8 e4m3 codes -> float64 values."""
    return E4M3_TABLE[np.asarray(codes, dtype=np.uint8)]


def decode(bits, dtype):
    if dtype == "bf16":
        return decode_bf16(bits)
    if dtype == "e4m3":
        return decode_e4m3(bits)
    raise ValueError(dtype)
