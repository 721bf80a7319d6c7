"""Pins for oracle/philox.py (CPU only)."""
import numpy as np
from scipy import stats

from oracle import philox


def test_generic_rounds_match_numpy_philox4x64():
    # numpy.random.Philox is an independent Philox-4x64-10; it advances the counter
    # by one before producing each block of four words.
    rng = np.random.default_rng(7)
    for _ in range(5):
        ctr = [int(v) for v in rng.integers(0, 2**63, size=4, dtype=np.uint64)]
        key = [int(v) for v in rng.integers(0, 2**63, size=2, dtype=np.uint64)]
        bg = np.random.Philox(counter=np.array(ctr, dtype=np.uint64), key=np.array(key, dtype=np.uint64))
        got = [int(v) for v in bg.random_raw(8)]
        c1 = [ctr[0] + 1, ctr[1], ctr[2], ctr[3]]
        c2 = [ctr[0] + 2, ctr[1], ctr[2], ctr[3]]
        want = list(philox.philox4_scalar(c1, key, W=64)) + list(philox.philox4_scalar(c2, key, W=64))
        assert got == want


def test_vectorised_matches_generic_w32():
    rng = np.random.default_rng(11)
    c = rng.integers(0, 2**32, size=(64, 4), dtype=np.uint64)
    k0, k1 = 0x9ABCDEF0, 0x12345678
    out = philox.philox4x32(c[:, 0], c[:, 1], c[:, 2], c[:, 3], k0, k1)
    for i in range(64):
        want = philox.philox4_scalar([int(v) for v in c[i]], [k0, k1], W=32)
        assert tuple(int(o[i]) for o in out) == want


def test_round_count_and_key_matter():
    a = philox.philox4_scalar([1, 2, 3, 4], [5, 6], W=32, rounds=10)
    assert a != philox.philox4_scalar([1, 2, 3, 4], [5, 6], W=32, rounds=9)
    assert a != philox.philox4_scalar([1, 2, 3, 4], [5, 7], W=32, rounds=10)
    assert a != philox.philox4_scalar([1, 2, 4, 3], [5, 6], W=32, rounds=10)


def test_word_layout_of_stream():
    w = philox.uint32_words(0x1234567890ABCDEF, philox.STREAM_STEP, 17, 3, 10)
    b0 = philox.philox4_scalar([0, 3, 17, philox.STREAM_STEP], [0x90ABCDEF, 0x12345678], W=32)
    b2 = philox.philox4_scalar([2, 3, 17, philox.STREAM_STEP], [0x90ABCDEF, 0x12345678], W=32)
    assert tuple(int(v) for v in w[:4]) == b0
    assert tuple(int(v) for v in w[8:10]) == b2[:2]


def test_uniform_bits():
    w = philox.uint32_words(99, philox.STREAM_INIT, 0, 0, 1 << 18)
    bits = np.unpackbits(w.view(np.uint8))
    assert abs(bits.mean() - 0.5) < 3e-3
    # every one of the 32 bit positions is balanced
    per_bit = [(w >> np.uint32(b)) & np.uint32(1) for b in range(32)]
    assert max(abs(float(p.mean()) - 0.5) for p in per_bit) < 6e-3


def test_normals_moments_and_ks():
    z = philox.normals(12345, philox.STREAM_STEP, 5, 2, 1 << 18)
    n = len(z)
    assert abs(z.mean()) < 5.0 / np.sqrt(n)
    assert abs(z.var() - 1.0) < 5.0 * np.sqrt(2.0 / n)
    assert abs(stats.skew(z)) < 0.03
    assert abs(stats.kurtosis(z)) < 0.06
    assert stats.kstest(z, "norm").pvalue > 1e-3
    # the four Box-Muller lanes are individually normal and mutually uncorrelated
    q = z.reshape(-1, 4)
    cc = np.corrcoef(q.T)
    assert np.max(np.abs(cc - np.eye(4))) < 0.02
    for lane in range(4):
        assert stats.kstest(q[:, lane], "norm").pvalue > 1e-3


def test_streams_are_distinct_and_keyed_by_original_id():
    a = philox.normals(1, philox.STREAM_STEP, 3, 0, 64)
    assert not np.allclose(a, philox.normals(1, philox.STREAM_STEP, 4, 0, 64))
    assert not np.allclose(a, philox.normals(1, philox.STREAM_STEP, 3, 1, 64))
    assert not np.allclose(a, philox.normals(1, philox.STREAM_INIT, 3, 0, 64))
    assert not np.allclose(a, philox.normals(2, philox.STREAM_STEP, 3, 0, 64))
    np.testing.assert_array_equal(a[:10], philox.normals(1, philox.STREAM_STEP, 3, 0, 10))


# ---- the 32-bit constants ----
def test_weyl_increments_have_their_closed_form():
    # the key schedule adds the fractional parts of the golden ratio and of sqrt(3) - 1, scaled to the
    # word width and truncated (SC'11 paper, the paragraph on the Weyl sequence): exact integer arithmetic
    from math import isqrt
    for W in (32, 64):
        c = philox._CONST[W]
        golden = (isqrt(5 << (2 * W + 8)) - (1 << (W + 4))) >> 5        # floor(2^W (sqrt(5) - 1) / 2)
        root3 = isqrt(3 << (2 * W)) - (1 << W)                         # floor(2^W (sqrt(3) - 1))
        assert c["W0"] == golden and c["W1"] == root3


def _vendor_philox_constants():
    """The four 32-bit constants as the GPU vendor's random-number library states them in the header it
    installs (an independent statement of the generator's published constants)."""
    import os
    import re
    path = "/opt/rocm/include/rocrand/rocrand_philox4x32_10.h"
    if not os.path.exists(path):
        return None
    text = open(path).read()
    out = {}
    for ours, theirs in (("M0", "ROCRAND_PHILOX_M4x32_0"), ("M1", "ROCRAND_PHILOX_M4x32_1"),
                         ("W0", "ROCRAND_PHILOX_W32_0"), ("W1", "ROCRAND_PHILOX_W32_1")):
        m = re.search(r"#define\s+" + theirs + r"\s+(0[xX][0-9a-fA-F]+)", text)
        assert m, theirs
        out[ours] = int(m.group(1), 16)
    return out


def test_w32_constants_match_the_vendor_header():
    import pytest
    vendor = _vendor_philox_constants()
    if vendor is None:
        pytest.skip("vendor random-number header not installed")
    assert philox._CONST[32] == vendor


def test_kernel_header_states_the_same_constants():
    # the HIP side keeps its own copy (the two share no code): both must state the published values
    import os
    import re
    import pytest
    vendor = _vendor_philox_constants()
    if vendor is None:
        pytest.skip("vendor random-number header not installed")
    here = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    text = open(os.path.join(here, "paper_2512_15347_amd", "csrc", "philox.hpp")).read()
    for name in ("M0", "M1", "W0", "W1"):
        m = re.search(r"PHILOX_" + name + r"\s*=\s*(0[xX][0-9a-fA-F]+)", text)
        assert m and int(m.group(1), 16) == vendor[name]
