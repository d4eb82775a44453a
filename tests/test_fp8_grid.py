"""The e4m3 grid helpers that prepare one-byte weights for both sides (workloads/fp8.py), against the published
format: OCP 8-bit floating point, E4M3 variant (bias 7, no infinities, largest finite value 448)."""
import numpy as np

from workloads.fp8 import e4m3_table, encode_rne, quantize_rows


def test_e4m3_grid_helpers():
    """Every code decodes to sign * (1 + m/8) *
    2^(e-7), subnormals m * 2^-9, largest 448; encoding is the nearest code with ties to the even mantissa."""
    t = e4m3_table()
    assert t[0x38] == 1.0 and t[0x7E] == 448.0 and t[0x01] == 2.0 ** -9 and t[0x08] == 2.0 ** -6 and np.isnan(t[0x7F])
    ok = ~np.isnan(t)
    assert (encode_rne(t[ok]) == np.arange(256, dtype=np.uint8)[ok]).all()
    assert encode_rne(np.float32(1.0625)) == 0x38 and encode_rne(np.float32(1.1875)) == 0x3A     # ties to even
    assert encode_rne(np.float32(1e9)) == 0x7E and encode_rne(np.float32(-1e9)) == 0xFE          # saturation
    rng = np.random.default_rng(0)
    w = (rng.standard_normal((32, 512)) * 0.02).astype(np.float32)
    codes, scale, deq = quantize_rows(w)
    assert np.abs(deq - w).max() <= np.abs(w).max(axis=1).max() / 448 * 16 + 1e-9               # half a step at the top binade
    assert np.allclose(np.abs(deq).max(axis=1), np.abs(w).max(axis=1), rtol=1e-6, atol=0)        # the row maximum maps to 448


