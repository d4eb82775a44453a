"""Philox4x32-10 counter-based generator (Salmon et al., "Parallel random numbers: as easy as
1, 2, 3", SC'11), vectorised over counters with numpy.

Harness code: it only manufactures seeded inputs (uniforms in [0,1) on the 2^-24 grid) that are handed
identically to the CPU oracle and to the HIP library.  It holds none of the method's arithmetic.
"""
import numpy as np

_M0 = np.uint64(0xD2511F53)
_M1 = np.uint64(0xCD9E8D57)
_W0 = 0x9E3779B9
_W1 = 0xBB67AE85
_MASK = np.uint64(0xFFFFFFFF)


def philox4x32_10(counter, key):
    """counter: uint32 array [..., 4]; key: (k0, k1) python ints. Returns uint32 array [..., 4]."""
    c = np.asarray(counter, dtype=np.uint32).astype(np.uint64)
    c0, c1, c2, c3 = c[..., 0], c[..., 1], c[..., 2], c[..., 3]
    k0, k1 = int(key[0]) & 0xFFFFFFFF, int(key[1]) & 0xFFFFFFFF
    for _ in range(10):
        p0 = _M0 * c0
        p1 = _M1 * c2
        hi0, lo0 = p0 >> np.uint64(32), p0 & _MASK
        hi1, lo1 = p1 >> np.uint64(32), p1 & _MASK
        c0, c1, c2, c3 = (hi1 ^ c1 ^ np.uint64(k0), lo1, hi0 ^ c3 ^ np.uint64(k1), lo0)
        k0 = (k0 + _W0) & 0xFFFFFFFF
        k1 = (k1 + _W1) & 0xFFFFFFFF
    return np.stack([c0, c1, c2, c3], axis=-1).astype(np.uint32)


def uniform24(seed, shape, stream=0):
    """Seeded uniforms u = m * 2^-24, m a 24-bit integer, as float32 (exactly representable).

    Element i of the flattened result is word (i % 4) of block (i // 4) with counter
    (i // 4, 0, stream, 0) and key (seed, 0x5EED): consumed by index, never "next from stream".
    """
    n = int(np.prod(shape)) if len(shape) else 1
    nb = (n + 3) // 4
    ctr = np.zeros((nb, 4), dtype=np.uint32)
    ctr[:, 0] = np.arange(nb, dtype=np.uint64).astype(np.uint32)
    ctr[:, 2] = np.uint32(stream)
    words = philox4x32_10(ctr, (seed, 0x5EED)).reshape(-1)[:n]
    m = (words >> np.uint32(8)).astype(np.float32)
    return (m * np.float32(2.0 ** -24)).reshape(shape)
