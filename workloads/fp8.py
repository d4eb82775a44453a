"""One-byte weights for the seeded workloads: the OCP e4m3 grid (sign, 4 exponent bits of bias 7, 3 mantissa
bits, no infinities, largest finite value 448) with one float32 scale per output row.  Input preparation only (no
arithmetic of the method): the harness quantises a seeded matrix once, uploads codes and scales to the library
and hands the SAME dequantised values to the oracle."""
import numpy as np


def e4m3_table():
    """float32 value of every code (the two not-a-number codes 0x7f / 0xff map to nan)."""
    c = np.arange(256, dtype=np.int64)
    s = np.where(c & 0x80, -1.0, 1.0)
    e = (c >> 3) & 0xF
    m = c & 7
    v = np.where(e == 0, m * 2.0 ** -9, (1.0 + m / 8.0) * 2.0 ** (e.astype(np.float64) - 7.0))
    v = np.where((c & 0x7F) == 0x7F, np.nan, v)
    return (s * v).astype(np.float32)


_TABLE = e4m3_table()


def encode_rne(x):
    """float32 -> nearest e4m3 code (ties to the even mantissa), saturating at +-448."""
    x = np.asarray(x, np.float32)
    a = np.minimum(np.abs(x), np.float32(448.0))
    b = a.view(np.uint32).astype(np.uint64)
    r = b + np.uint64(0x7FFFF) + ((b >> np.uint64(20)) & np.uint64(1))       # round to 3 mantissa bits
    e = (r >> np.uint64(23)).astype(np.int64) - 127 + 7
    m = ((r >> np.uint64(20)) & np.uint64(7)).astype(np.int64)
    normal = (e << 3) | m
    sub = np.rint(a.astype(np.float64) * 512.0).astype(np.int64)             # below 2^-6: spacing 2^-9
    code = np.where(a >= np.float32(2.0 ** -6), normal, sub)
    code = np.where(np.signbit(x), code | 0x80, code)
    return code.astype(np.uint8)


def quantize_rows(w):
    """w float32 [out][in] -> (codes uint8 [out][in], scale float32 [out], dequantised float32 [out][in]):
    scale = max |row| / 448, code = nearest e4m3 of fl32(w / scale), value = fl32(table[code] * scale)."""
    w = np.asarray(w, np.float32)
    amax = np.abs(w).max(axis=1)
    scale = np.where(amax > 0, amax / np.float32(448.0), np.float32(1.0)).astype(np.float32)
    codes = encode_rne(w / scale[:, None])
    deq = (_TABLE[codes] * scale[:, None]).astype(np.float32)
    return codes, scale, deq
