"""Four-bit weights for the seeded workloads: the OCP microscaling format MXFP4.  Elements are E2M1 codes (sign,
two exponent bits of bias 1, one mantissa bit: magnitudes 0, 0.5, 1, 1.5, 2, 3, 4, 6); every block of 32 consecutive
inputs of an output row shares a power-of-two scale stored as an E8M0 byte (2^(e - 127)).  Input preparation only (no
arithmetic of the method): the harness quantises a seeded matrix once, uploads codes and scales to the library and
hands the SAME dequantised values to the oracle.

Scale rule (the one the format's specification recommends): shared exponent = floor(log2(max |block|)) - 2, where 2
is the exponent of the largest E2M1 magnitude (6 = 1.5 * 2^2); elements are rounded to the nearest code, ties to the
code with an even mantissa bit, and saturate at +-6."""
import numpy as np

BLOCK = 32
_MAGNITUDES = np.array([0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0], np.float32)


def e2m1_table():
    """float32 value of every 4-bit code (bit 3 = sign)."""
    return np.concatenate([_MAGNITUDES, -_MAGNITUDES]).astype(np.float32)


_TABLE = e2m1_table()


def encode_rne(x):
    """float32 -> nearest E2M1 code, ties to the even mantissa bit, saturating at +-6."""
    x = np.asarray(x, np.float32)
    a = np.abs(x).astype(np.float64)
    # midpoints between neighbouring magnitudes; at a tie the neighbour with mantissa bit 0 wins: codes 0, 2, 4, 6
    # have mantissa 0, so the tie at the midpoint of (m_i, m_{i+1}) goes up when i is odd and down when i is even
    mids = (_MAGNITUDES[:-1].astype(np.float64) + _MAGNITUDES[1:]) / 2.0
    idx = np.zeros(a.shape, np.int64)
    for i, mid in enumerate(mids):
        idx += (a > mid) if i % 2 == 0 else (a >= mid)
    code = idx | (np.signbit(x).astype(np.int64) << 3)
    return code.astype(np.uint8)


def quantize_blocks(w):
    """w float32 [out][in], in a multiple of 32 -> (codes uint8 [out][in/2], column c in the low nibble of byte c/2 for
    even c; scales uint8 [out][in/32], E8M0; dequantised float32 [out][in])."""
    w = np.asarray(w, np.float32)
    n, k = w.shape
    assert k % BLOCK == 0
    blocks = w.reshape(n, k // BLOCK, BLOCK)
    amax = np.abs(blocks).max(axis=2).astype(np.float64)
    exp = np.where(amax > 0, np.floor(np.log2(np.where(amax > 0, amax, 1.0))) - 2.0, 0.0)
    exp = np.clip(exp, -126.0, 127.0)                       # (E8M0 byte 1 .. 254; 255 is not-a-number)
    scales = (exp + 127.0).astype(np.uint8)
    s = np.exp2(exp).astype(np.float32)                     # powers of two: exact
    codes4 = encode_rne(blocks / s[:, :, None])             # division by a power of two: exact
    deq = (_TABLE[codes4] * s[:, :, None]).astype(np.float32).reshape(n, k)
    flat = codes4.reshape(n, k)
    packed = (flat[:, 0::2] | (flat[:, 1::2] << 4)).astype(np.uint8)
    return packed, scales, deq
