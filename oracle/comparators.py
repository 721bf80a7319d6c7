"""Comparison arms of the paper's motivation study and the group diagnostics they
are judged by, fp64 (test infrastructure only).

Sec. 4.1 measures how rewards of a group cluster around the group mean (Eq. 7:
the set C_delta within delta standard deviations of the mean) and argues that a
uniformly random k-subset does not raise the within-group variance; Sec. 4.2
applies Optimal Variance Filtering once, after sampling, to the final rewards
("static" OVF) and compares the within-group standard deviation sigma_G of
three arms: the full group, a uniform k-subset, the OVF k-subset.

* ``group_stats``     sigma_G (population, 1/G) and |C_delta| / G per ragged group.
* ``uniform_subset``  the uniform k-subset.  The paper does not say how it is
  drawn.  Reading used here (shared with the library, which implements the same
  published generator on its own): slot j of group g draws one 32-bit key, word
  0 of the Philox-4x32-10 block with counter (j, draw, g, STREAM_SUBSAMPLE) and
  the run's seed as key; the k slots with the smallest (key, slot) are kept.
  Sorting i.i.d. keys and keeping the first k is a uniform draw over k-subsets.
* ``select_final``    one arm applied to a finished sampling run: select on the
  final rewards, gather the survivors, recompute Eq. 18 on them.

Pins (tests/test_oracle_comparators.py): subset size and order; agreement with a
sort of keys from the scalar Philox routine; every 3-subset of 8 equally likely
(chi-square); the sample-variance identity E[s^2_subset] = s^2_group behind the
paper's remark that subsampling leaves the variance unchanged in expectation;
OVF's sigma_G is never below any drawn subset's; sigma_G against numpy.std and a
hand-worked C_delta example.
"""
import numpy as np

from . import philox, ovf

STREAM_SUBSAMPLE = 2     # fourth counter word of the subset keys (0, 1: initial latents, step noise)

MODE_OVF = 0
MODE_UNIFORM = 1


def subset_keys(seed, draw, group, n):
    """The n 32-bit keys of one group's draw."""
    w = philox.philox4x32(np.arange(n, dtype=np.uint64), draw, group, STREAM_SUBSAMPLE,
                          seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF)
    return w[0]


def uniform_subset(seed, draw, group, n, k):
    """(mask, ascending slot indices) of the k slots with the smallest (key, slot)."""
    if not (1 <= k <= n <= 64):
        raise ValueError("need 1 <= k <= n <= 64")
    keys = subset_keys(seed, draw, group, n)
    order = sorted(range(n), key=lambda j: (int(keys[j]), j))
    idx = sorted(order[:k])
    mask = 0
    for j in idx:
        mask |= 1 << j
    return mask, idx


def uniform_groups(seed, draw, group_offsets, k_per_group):
    """Uniform subsets over ragged groups; same return convention as ovf.ovf_groups."""
    P = len(k_per_group)
    masks = np.zeros(P, dtype=np.uint64)
    sel = []
    new_off = np.zeros(P + 1, dtype=np.int32)
    for g in range(P):
        b, e = int(group_offsets[g]), int(group_offsets[g + 1])
        m, idx = uniform_subset(seed, draw, g, e - b, int(k_per_group[g]))
        masks[g] = np.uint64(m)
        sel.extend(b + i for i in idx)
        new_off[g + 1] = new_off[g] + len(idx)
    return masks, np.asarray(sel, dtype=np.int32), new_off


def group_stats(rewards, group_offsets, delta):
    """Per ragged group: population standard deviation sigma_G and the share of
    members inside the clustered region of Eq. 7, |R - mu| <= delta * sigma_G.
    An empty group reports (0, 0)."""
    r = np.asarray(rewards, dtype=np.float64)
    P = len(group_offsets) - 1
    sigma = np.zeros(P)
    frac = np.zeros(P)
    for g in range(P):
        b, e = int(group_offsets[g]), int(group_offsets[g + 1])
        if e == b:
            continue
        mu = np.mean(r[b:e])
        sigma[g] = np.sqrt(np.mean((r[b:e] - mu) ** 2))
        frac[g] = np.count_nonzero(np.abs(r[b:e] - mu) <= delta * sigma[g]) / (e - b)
    return sigma, frac


def select_final(rewards, group_offsets, k_per_group, mode, seed=0, draw=0, eps=1e-6):
    """One comparison arm on the final rewards of a finished run.

    Returns dict(masks, sel_idx, offsets, rewards, adv): the selection, the packed
    positions of the kept members, and Eq. 18 recomputed on them."""
    r = np.asarray(rewards, dtype=np.float64)
    if mode == MODE_OVF:
        masks, sel, new_off = ovf.ovf_groups(np.asarray(rewards, dtype=np.float32), group_offsets, k_per_group)
    elif mode == MODE_UNIFORM:
        masks, sel, new_off = uniform_groups(seed, draw, group_offsets, k_per_group)
    else:
        raise ValueError("mode")
    kept = ovf.compact(r, sel)
    return dict(masks=masks, sel_idx=sel, offsets=new_off, rewards=kept,
                adv=ovf.group_advantages(kept, new_off, eps))
