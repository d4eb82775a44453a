"""The MXFP4 helpers that prepare four-bit weights for both sides (workloads/fp4.py), against the published format:
OCP microscaling formats, MXFP4 = E2M1 elements (magnitudes 0, 0.5, 1, 1.5, 2, 3, 4, 6) in blocks of 32 that share
an E8M0 power-of-two scale."""
import numpy as np

from workloads.fp4 import e2m1_table, encode_rne, quantize_blocks


def test_e2m1_grid_and_block_scales():
    t = e2m1_table()
    # the format's value table: code = sign, two exponent bits (bias 1), one mantissa bit
    for code in range(16):
        s, e, m = code >> 3, (code >> 1) & 3, code & 1
        v = (m * 0.5) if e == 0 else (1.0 + 0.5 * m) * 2.0 ** (e - 1)
        assert t[code] == (-v if s else v)
    assert (encode_rne(t[:8]) == np.arange(8)).all() and (encode_rne(t[9:]) == np.arange(9, 16)).all()
    # nearest value, ties to the even mantissa bit, saturation at 6
    x = np.array([0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0, 0.26, 0.74, 2.6, 100.0, -5.0, -7.0], np.float32)
    want = np.array([0.0, 1.0, 1.0, 2.0, 2.0, 4.0, 4.0, 0.5, 0.5, 3.0, 6.0, -4.0, -6.0], np.float32)
    assert (t[encode_rne(x)] == want).all()
    rng = np.random.default_rng(0)
    w = (rng.standard_normal((24, 256)) * 0.02).astype(np.float32)
    w[3, 32:64] = 0.0                                           # an all-zero block
    codes, scales, deq = quantize_blocks(w)
    assert codes.shape == (24, 128) and scales.shape == (24, 8) and deq.shape == w.shape
    amax = np.abs(w.reshape(24, 8, 32)).max(axis=2)
    nz = amax > 0
    # shared exponent = floor(log2(block maximum)) - 2: the block maximum lands in [4, 8) scale units, so it is
    # represented by 4 or 6 and nothing in the block overflows by more than the step at the top
    s = np.exp2(scales.astype(np.float64) - 127.0)
    assert (amax[nz] / s[nz] >= 4.0).all() and (amax[nz] / s[nz] < 8.0).all()
    assert (deq[3, 32:64] == 0).all()
    # every element within half a step of its block's grid (the step is at most 2 scale units; saturation at 6
    # can cost up to 2 more for block maxima in (6, 8) scale units)
    err = np.abs(deq - w).reshape(24, 8, 32)
    assert (err <= 2.0 * s[:, :, None] + 1e-12).all()
    assert (err[np.abs(w.reshape(24, 8, 32)) <= 6.0 * s[:, :, None]] <= 1.0 * np.broadcast_to(s[:, :, None], err.shape)[np.abs(w.reshape(24, 8, 32)) <= 6.0 * s[:, :, None]] + 1e-12).all()
    # packing: column c in the low nibble of byte c / 2 for even c
    c4 = encode_rne(w.reshape(24, 8, 32) / s[:, :, None].astype(np.float32)).reshape(24, 256)
    assert ((codes & 0xF) == c4[:, 0::2]).all() and ((codes >> 4) == c4[:, 1::2]).all()
    assert (deq == (t[c4].reshape(24, 8, 32) * s[:, :, None].astype(np.float32)).reshape(24, 256)).all()
