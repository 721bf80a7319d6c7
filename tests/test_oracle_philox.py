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
