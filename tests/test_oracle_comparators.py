"""Pins of the comparison arms (uniform k-subset, static OVF) and the group diagnostics
(sigma_G, clustered share of Eq. 7)."""
import itertools
import math

import numpy as np
import pytest

from oracle import comparators as cmp, ovf, philox
from paper_2512_15347_amd import workloads


def test_uniform_subset_is_the_k_smallest_keys_of_the_scalar_generator():
    seed, draw, g, n, k = 0x1234_5678_9ABC_DEF0, 3, 5, 11, 4
    keys = [philox.philox4_scalar((j, draw, g, cmp.STREAM_SUBSAMPLE), (seed & 0xFFFFFFFF, seed >> 32))[0]
            for j in range(n)]
    want = sorted(sorted(range(n), key=lambda j: (keys[j], j))[:k])
    mask, idx = cmp.uniform_subset(seed, draw, g, n, k)
    assert idx == want
    assert mask == sum(1 << j for j in want)
    assert bin(mask).count("1") == k


def test_uniform_subset_edges():
    assert cmp.uniform_subset(1, 0, 0, 1, 1) == (1, [0])
    m, idx = cmp.uniform_subset(1, 0, 0, 64, 64)
    assert m == (1 << 64) - 1 and idx == list(range(64))
    with pytest.raises(ValueError):
        cmp.uniform_subset(1, 0, 0, 8, 9)
    with pytest.raises(ValueError):
        cmp.uniform_subset(1, 0, 0, 8, 0)
    # other draw, other group, other seed: other keys
    base = cmp.subset_keys(7, 0, 0, 16)
    assert not np.array_equal(base, cmp.subset_keys(7, 1, 0, 16))
    assert not np.array_equal(base, cmp.subset_keys(7, 0, 1, 16))
    assert not np.array_equal(base, cmp.subset_keys(8, 0, 0, 16))
    # and not the words the step noise of trajectory 0 uses
    assert not np.array_equal(base, philox.philox4x32(np.arange(16), 0, 0, philox.STREAM_STEP, 7, 0)[0])


def test_every_subset_is_equally_likely():
    """3 of 8: 56 subsets; 28000 draws give 500 expected per subset.  Chi-square with 55 degrees of
    freedom stays below 100 with overwhelming probability (p ~ 2e-4 of exceeding)."""
    n, k, draws = 8, 3, 28000
    counts = {}
    for g in range(draws):
        m, _ = cmp.uniform_subset(99, 0, g, n, k)
        counts[m] = counts.get(m, 0) + 1
    assert len(counts) == math.comb(n, k)
    exp = draws / math.comb(n, k)
    chi2 = sum((c - exp) ** 2 / exp for c in counts.values())
    assert chi2 < 100.0
    incl = np.zeros(n)
    for m, c in counts.items():
        for j in range(n):
            if (m >> j) & 1:
                incl[j] += c
    np.testing.assert_allclose(incl / draws, k / n, atol=0.012)


def test_uniform_subsampling_keeps_the_variance_in_expectation():
    """Sec. 4.1: a random k-subset does not raise the variance in expectation.  Exactly: the unbiased
    sample variance of a simple random sample without replacement has expectation S^2 of the group, i.e.
    E[sigma_sub^2] = sigma_G^2 * (k - 1) / k * n / (n - 1) <= sigma_G^2."""
    r = workloads.stress_rewards(1, 24)[0].astype(np.float64)
    n, k = 24, 12
    sig2 = np.var(r)
    acc = 0.0
    draws = 6000
    for d in range(draws):
        _, idx = cmp.uniform_subset(5, d, 0, n, k)
        acc += np.var(r[idx])
    want = sig2 * (k - 1) / k * n / (n - 1)
    assert abs(acc / draws - want) < 0.03 * want
    assert want < sig2


def test_ovf_sigma_dominates_every_drawn_subset_and_the_full_group():
    r = workloads.stress_rewards(6, 24)
    offs = np.arange(0, 7 * 24, 24)
    kk = [12] * 6
    s_full, _ = cmp.group_stats(r.reshape(-1), offs, 1.0)
    o = cmp.select_final(r.reshape(-1), offs, kk, cmp.MODE_OVF)
    s_ovf, _ = cmp.group_stats(o["rewards"], o["offsets"], 1.0)
    assert np.all(s_ovf >= s_full)
    for d in range(50):
        u = cmp.select_final(r.reshape(-1), offs, kk, cmp.MODE_UNIFORM, seed=3, draw=d)
        s_uni, _ = cmp.group_stats(u["rewards"], u["offsets"], 1.0)
        assert np.all(s_ovf >= s_uni - 1e-12)
        assert list(u["offsets"]) == list(range(0, 73, 12))
        # advantages of the kept members: zero mean, unit population std (up to eps)
        for g in range(6):
            a = u["adv"][12 * g:12 * g + 12]
            assert abs(a.mean()) < 1e-9 and abs(a.std() - 1.0) < 1e-4


def test_select_final_gathers_in_group_then_slot_order():
    r = np.arange(20, dtype=np.float32)[::-1].copy()
    offs = np.array([0, 8, 20])
    out = cmp.select_final(r, offs, [3, 5], cmp.MODE_UNIFORM, seed=11, draw=2)
    sel = out["sel_idx"]
    assert np.all(np.diff(sel) > 0) and np.all(sel[:3] < 8) and np.all(sel[3:] >= 8)
    np.testing.assert_array_equal(out["rewards"], r[sel])
    for g, (b, e) in enumerate([(0, 8), (8, 20)]):
        m = int(out["masks"][g])
        assert [b + j for j in range(e - b) if (m >> j) & 1] == list(sel[out["offsets"][g]:out["offsets"][g + 1]])


def test_group_stats_against_numpy_and_a_hand_example():
    # hand example: rewards 0,0,0,0,10 -> mu 2, sigma 4; |R - mu| = 2,2,2,2,8
    sig, frac = cmp.group_stats([0, 0, 0, 0, 10], [0, 5], 0.5)
    assert sig[0] == 4.0 and frac[0] == 0.8            # 2 <= 0.5 * 4 holds with equality
    sig, frac = cmp.group_stats([0, 0, 0, 0, 10], [0, 5], 0.49)
    assert frac[0] == 0.0
    sig, frac = cmp.group_stats([0, 0, 0, 0, 10], [0, 5], 2.0)
    assert frac[0] == 1.0
    r = workloads.stress_rewards(5, 17).reshape(-1).astype(np.float64)
    offs = [0, 17, 34, 34, 60, 85]                      # ragged, one empty group
    sig, frac = cmp.group_stats(r, offs, 1.0)
    for g in range(5):
        b, e = offs[g], offs[g + 1]
        if e == b:
            assert sig[g] == 0 and frac[g] == 0
            continue
        assert abs(sig[g] - np.std(r[b:e])) < 1e-15
        idx = ovf.clustered_region(r[b:e], 1.0)
        assert frac[g] == len(idx) / (e - b)
    # the clustered stress input: most members sit inside one sigma (the phenomenon of Sec. 4.1)
    assert np.mean(frac[[0, 1, 3, 4]]) > 0.7


def test_static_ovf_equals_brute_force_on_small_groups():
    rng = np.random.default_rng(5)
    r = rng.normal(size=(4, 9)).astype(np.float32)
    offs = np.arange(0, 45, 9)
    out = cmp.select_final(r.reshape(-1), offs, [4] * 4, cmp.MODE_OVF)
    for g in range(4):
        best = max(itertools.combinations(range(9), 4), key=lambda s: np.var(r[g, list(s)].astype(np.float64)))
        got = out["rewards"][4 * g:4 * g + 4]
        assert abs(np.var(got) - np.var(r[g, list(best)].astype(np.float64))) < 1e-12
