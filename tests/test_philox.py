"""The counter-based generator of the uniforms: the harness's host version against the published known answers
(no GPU), and the library's device version against the host version, bit for bit."""
import numpy as np
import pytest

import workloads as wl


def _hex(c, k):
    return " ".join("%08x" % x for x in wl.philox4x32_10(np.array(c, dtype=np.uint32), k))


def test_host_philox_matches_the_published_known_answers():
    # Philox4x32-10 known-answer vectors distributed with the generator's reference implementation
    # (Salmon et al., SC'11): zero, all-ones and the digits-of-pi counter / key
    assert _hex([0, 0, 0, 0], (0, 0)) == "6627e8d5 e169c58d bc57ac4c 9b00dbd8"
    assert _hex([0xFFFFFFFF] * 4, (0xFFFFFFFF, 0xFFFFFFFF)) == "408f276d 41c83b0e a20bc7c6 6d5451fd"
    assert _hex([0x243F6A88, 0x85A308D3, 0x13198A2E, 0x03707344], (0xA4093822, 0x299F31D0)) == \
        "d16cfe09 94fdcceb 5001e420 24126ea1"


def test_uniforms_are_on_the_24_bit_grid_and_indexed():
    u = wl.uniform24(7, (3, 5))
    assert u.dtype == np.float32 and (u >= 0).all() and (u < 1).all()
    assert np.array_equal(u * 2 ** 24, np.floor(u * 2 ** 24))
    # element i depends on (seed, stream, i) only: a longer draw starts with the shorter one
    assert np.array_equal(wl.uniform24(7, (40,))[:15], u.reshape(-1))
    assert not np.array_equal(wl.uniform24(7, (15,), stream=1), u.reshape(-1))


@pytest.mark.gpu
@pytest.mark.parametrize("seed,stream,n", [(0, 0, 1), (3001, 0, 5), (4004, 1, 4099), (0xFFFFFFFF, 7, 1 << 20), (12, 3, 0)])
def test_device_philox_equals_the_host_generator(seed, stream, n):
    import paper_2406_18200_amd as sv
    got = sv.uniform_philox(seed, (n,), stream=stream).cpu().numpy()
    want = wl.uniform24(seed, (n,), stream=stream)
    assert got.dtype == np.float32 and np.array_equal(got, want)
