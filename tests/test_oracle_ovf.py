"""Pins for oracle/ovf.py (CPU only): brute force over all k-subsets (Eq. 10),
the two-extremes property, the variance guarantees, and the advantage invariants
(Eq. 5, Eq. 8, Eq. 18)."""
import itertools
import math
import numpy as np
import pytest

from oracle import ovf
from paper_2512_15347_amd import workloads


def _mask_to_idx(mask):
    return [i for i in range(64) if (int(mask) >> i) & 1]


def test_matches_bruteforce_on_tie_free_inputs():
    rng = np.random.default_rng(0)
    for n in range(2, 12):
        for k in range(1, n + 1):
            for trial in range(3):
                r = rng.standard_normal(n).astype(np.float32)
                if trial == 1:
                    r = (r * 0.05 + 23.0).astype(np.float32)      # reward-model scale, clustered
                mask, idx, j = ovf.ovf_select(r, k)
                best, best_set = ovf.ovf_bruteforce(r, k)
                assert len(idx) == k and idx == _mask_to_idx(mask)
                got = ovf.population_variance(r[idx])
                assert got == pytest.approx(best, rel=1e-12, abs=1e-300)
                if k > 1 and len(set(r.tolist())) == n:
                    assert tuple(idx) == best_set


def test_ties_reach_the_optimal_value():
    rng = np.random.default_rng(1)
    for n in (4, 7, 10):
        for k in range(1, n + 1):
            r = rng.integers(-2, 3, size=n).astype(np.float32)    # many equal values
            _, idx, _ = ovf.ovf_select(r, k)
            best, _ = ovf.ovf_bruteforce(r, k)
            assert ovf.population_variance(r[idx]) == pytest.approx(best, rel=1e-12, abs=1e-15)


def test_tie_rules():
    # all equal: every split scores 0 -> j = 0 -> the k highest ranks = the k largest indices
    mask, idx, j = ovf.ovf_select(np.ones(6, np.float32), 3)
    assert j == 0 and idx == [3, 4, 5]
    # k = 1: every score is 0 -> the single largest reward
    mask, idx, j = ovf.ovf_select(np.array([0.1, 0.9, -0.5, 0.3], np.float32), 1)
    assert idx == [1] and j == 0
    # k = n keeps all
    mask, idx, j = ovf.ovf_select(np.array([3, 1, 2], np.float32), 3)
    assert idx == [0, 1, 2] and mask == 0b111
    # symmetric input: j=1 (low + 2 high) and j=2 (2 low + high) tie -> smaller j
    mask, idx, j = ovf.ovf_select(np.array([-2, -1, 0, 1, 2], np.float32), 3)
    assert j == 1 and idx == [0, 3, 4]
    # -0.0 and +0.0 are the same value: index breaks the tie
    a = ovf.ovf_select(np.array([-0.0, 0.0, 1.0, -1.0], np.float32), 3)
    b = ovf.ovf_select(np.array([0.0, -0.0, 1.0, -1.0], np.float32), 3)
    assert a == b


def test_contains_both_extremes_and_is_extreme_split():
    rng = np.random.default_rng(2)
    for _ in range(200):
        n = int(rng.integers(2, 65)); k = int(rng.integers(2, n + 1))
        r = rng.standard_normal(n).astype(np.float32)
        _, idx, j = ovf.ovf_select(r, k)
        assert int(np.argmin(r)) in idx and int(np.argmax(r)) in idx
        order = np.argsort(r, kind="stable")
        assert sorted(order[:j].tolist() + order[n - (k - j):].tolist()) == idx


def test_variance_dominates_random_subsets_and_full_group_bound():
    rng = np.random.default_rng(3)
    r = workloads.stress_rewards(50, 64)
    for g in range(50):
        _, idx, _ = ovf.ovf_select(r[g], 16)
        v = ovf.population_variance(r[g][idx])
        for _ in range(20):
            sub = rng.choice(64, 16, replace=False)
            assert v >= ovf.population_variance(r[g][sub]) - 1e-15
        # the mean over all k-subsets of the unbiased variance equals the unbiased
        # variance of the full group, so the best subset is at least that large
        n, k = 64, 16
        assert v >= (k - 1) * n / (k * (n - 1)) * ovf.population_variance(r[g]) - 1e-15


def test_doubling_scan_is_a_prefix_sum():
    rng = np.random.default_rng(4)
    a = rng.standard_normal(64)
    s = ovf._doubling_scan(a)
    np.testing.assert_allclose(s, np.cumsum(a), rtol=1e-13, atol=1e-13)
    ints = rng.integers(-1000, 1000, 64).astype(np.float64)        # exact in fp64
    np.testing.assert_array_equal(ovf._doubling_scan(ints), np.cumsum(ints))


def test_rejects_bad_input():
    with pytest.raises(FloatingPointError):
        ovf.ovf_select(np.array([0.0, np.nan, 1.0], np.float32), 2)
    with pytest.raises(FloatingPointError):
        ovf.ovf_select(np.array([0.0, np.inf, 1.0], np.float32), 2)
    with pytest.raises(ValueError):
        ovf.ovf_select(np.zeros(3, np.float32), 4)
    with pytest.raises(ValueError):
        ovf.ovf_select(np.zeros(3, np.float32), 0)
    with pytest.raises(ValueError):
        ovf.ovf_select(np.zeros(1025, np.float32), 4)
    with pytest.raises(ValueError):
        ovf.ovf_groups(np.zeros(65, np.float32), [0, 65], [4])


def test_groups_above_64_members():
    """Generalisation beyond the paper's group sizes.  Pins: the chosen set beats every "j lowest + k-j highest"
    candidate evaluated in exact rational arithmetic (an arithmetic path of its own), no single swap with an
    unselected member raises the variance (necessary for the optimum of Eq. 10), and up to 64 members the
    result is what the 64-slot routine gave before."""
    from fractions import Fraction
    rng = np.random.default_rng(12)
    for n, k in ((65, 7), (100, 50), (200, 77), (513, 40), (1024, 512)):
        r = (rng.standard_normal(n) * np.where(rng.random(n) < 0.8, 0.05, 1.0)).astype(np.float32)
        mask, idx, j = ovf.ovf_select(r, k)
        assert len(idx) == k and bin(mask).count("1") == k and idx == sorted(idx)
        fr = sorted(Fraction(float(v)) for v in r)
        def score(jj):
            sub = fr[:jj] + fr[n - (k - jj):]
            s1 = sum(sub); s2 = sum(v * v for v in sub)
            return k * s2 - s1 * s1
        best = max(range(k + 1), key=lambda jj: (score(jj), -jj))
        chosen = sorted(Fraction(float(r[i])) for i in idx)
        assert chosen == fr[:best] + fr[n - (k - best):]
        var_sel = np.var(r[idx].astype(np.float64))
        inside = set(idx)
        outside = [i for i in range(n) if i not in inside]
        for _ in range(300):
            a = idx[rng.integers(k)]; b = outside[rng.integers(n - k)]
            trial = [i for i in idx if i != a] + [b]
            assert np.var(r[trial].astype(np.float64)) <= var_sel * (1 + 1e-12)
    masks, sel, off = ovf.ovf_groups_large(np.arange(300, dtype=np.float32), [0, 100, 300], [3, 130], 4)
    assert masks.shape == (2, 4) and off.tolist() == [0, 3, 133]
    assert sum(bin(int(w)).count("1") for w in masks[1]) == 130 and int(masks[0, 2]) == 0
    assert sel[:3].tolist() in ([0, 98, 99], [0, 1, 99])


def test_groups_compaction_and_schedule_counts():
    rng = np.random.default_rng(5)
    sizes = [48, 48, 17, 64, 1, 48]
    ks = [32, 48, 5, 16, 1, 16]
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    r = rng.standard_normal(off[-1]).astype(np.float32)
    masks, sel, new_off = ovf.ovf_groups(r, off, ks)
    assert new_off.tolist() == np.concatenate([[0], np.cumsum(ks)]).tolist()
    assert len(sel) == sum(ks) and np.all(np.diff(sel) > 0)         # (group, ascending slot) order
    for g in range(len(sizes)):
        assert bin(int(masks[g])).count("1") == ks[g]
        seg = sel[new_off[g]:new_off[g + 1]] - off[g]
        assert seg.tolist() == _mask_to_idx(masks[g])
    assert _mask_to_idx(masks[1]) == list(range(48))                # k = N is the identity
    payload = rng.standard_normal((off[-1], 3))
    np.testing.assert_array_equal(ovf.compact(payload, sel), payload[sel])


def test_advantages_invariants():
    rng = np.random.default_rng(6)
    sizes = [16, 12, 4, 1, 8]
    off = np.concatenate([[0], np.cumsum(sizes)])
    r = rng.standard_normal(off[-1]) * 0.3 + 22.0
    r[off[4]:off[5]] = 1.25                                         # a constant group
    eps = 1e-6
    a = ovf.group_advantages(r, off, eps)
    for g in range(len(sizes)):
        seg, rs = a[off[g]:off[g + 1]], r[off[g]:off[g + 1]]
        sigma = math.sqrt(np.mean((rs - rs.mean()) ** 2))           # population (1/K)
        assert abs(seg.mean()) < 1e-9
        assert seg.std() == pytest.approx(sigma / (sigma + eps), rel=1e-9, abs=1e-12)
    assert np.all(a[off[3]:off[5]] == 0.0)                          # sigma = 0 -> 0
    # worked example: rewards 1, 2, 3, 4 -> mu 2.5, sigma sqrt(1.25)
    a = ovf.group_advantages(np.array([1.0, 2.0, 3.0, 4.0]), [0, 4], 0.0)
    np.testing.assert_allclose(a, np.array([-1.5, -0.5, 0.5, 1.5]) / math.sqrt(1.25), rtol=1e-15)


def test_advantage_bound_on_clustered_region():
    rng = np.random.default_rng(7)
    for delta in (0.25, 0.5, 1.0):
        r = workloads.stress_rewards(20, 24, seed=9).astype(np.float64)
        for g in range(20):
            a = ovf.group_advantages(r[g], [0, 24], 1e-6)
            c = ovf.clustered_region(r[g], delta)
            assert np.all(np.abs(a[c]) <= delta)
