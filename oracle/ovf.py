"""Optimal Variance Filtering, compaction and group-relative advantages, fp64
(test infrastructure only).

OVF (Sec. 4.2, Eq. 10; in-loop form in Sec. 5.1, the arg-max after Eq. 16): of
G rewards keep the k-subset with the largest population variance.  The paper
gives the definition only, so

* ``ovf_bruteforce`` IS the definition: enumerate every k-subset.
* ``ovf_select`` is the exact fast routine.  Structure used: for fixed other
  members the variance is a convex quadratic in one member's value, so some
  optimum is "the j smallest and the k-j largest" for a j in 0..k; only k+1
  candidates need scoring.  Pinned by ``ovf_bruteforce`` on small G.

Evaluation order of ``ovf_select`` (fixed so that an index set is reproducible
bit for bit by any implementation that follows the same order):
  1. non-finite rewards are an error; -0.0 equals +0.0;
  2. rank by (value ascending, original index ascending);
  3. fp64 prefix sums of y and y*y from the bottom (lo, lo2) and from the top
     (hi, hi2), each by the doubling recurrence over 64 zero-padded slots
     (groups above 64 members, a generalisation beyond the paper's group sizes:
     the next power of two)
     (a[i] += a[i-d] for d = 1, 2, 4, ..., 32, all i updated from the values of
     the previous pass);
  4. score D_j = k*(lo2[j] + hi2[k-j]) - (lo[j] + hi[k-j])^2  (= k^2 * variance),
     every operation rounded separately (no fused multiply-add);
  5. largest D_j wins, ties go to the smallest j;
  6. the result is a 64-bit mask over original slots and the selected original
     indices in ascending order.

Advantages (Eq. 5, Eq. 18): population mean and standard deviation (1/K) of the
survivors' rewards, A = (R - mu) / (sigma + eps).
Pins: zero mean, std sigma/(sigma+eps), the bound of Eq. 8 on the clustered set
of Eq. 7, sigma = 0 gives 0.
"""
import itertools
import numpy as np

WAVE = 64


def population_variance(values):
    v = np.asarray(values, dtype=np.float64)
    return float(np.mean((v - np.mean(v)) ** 2))


def ovf_bruteforce(rewards, k):
    """Eq. 10 verbatim: (best variance, sorted index tuple) over all k-subsets."""
    r = np.asarray(rewards, dtype=np.float64)
    best, best_set = -1.0, None
    for comb in itertools.combinations(range(len(r)), k):
        v = population_variance(r[list(comb)])
        if v > best:
            best, best_set = v, comb
    return best, best_set


MAX_GROUP = 1024


def scan_slots(n):
    """Slots of the prefix-sum recurrence for a group of n: 64 up to 64 members (the
    sampling loop's case), else the next power of two."""
    s = WAVE
    while s < n:
        s *= 2
    return s


def _doubling_scan(a):
    """Inclusive prefix sum of len(a) (a power of two) fp64 slots by the doubling recurrence."""
    a = np.array(a, dtype=np.float64)
    d = 1
    while d < len(a):
        prev = a.copy()
        a[d:] = prev[d:] + prev[:-d]
        d *= 2
    return a


def ovf_select(rewards, k):
    """Exact variance-maximising k-subset of up to MAX_GROUP fp32 rewards (the paper's
    groups have at most 64 members; larger groups are a generalisation and use
    scan_slots(n) zero-padded slots in step 3).

    Returns (mask as Python int, ascending list of selected original indices,
    j = how many were taken from the low end)."""
    r = np.asarray(rewards, dtype=np.float32)
    n = len(r)
    if not (1 <= k <= n <= MAX_GROUP):
        raise ValueError("need 1 <= k <= n <= %d" % MAX_GROUP)
    S = scan_slots(n)
    if not np.all(np.isfinite(r)):
        raise FloatingPointError("non-finite reward")
    r = r + np.float32(0.0)                                   # -0.0 -> +0.0
    order = sorted(range(n), key=lambda i: (float(r[i]), i))   # step 2
    y = np.zeros(S); z = np.zeros(S)
    for rank, i in enumerate(order):
        y[rank] = float(r[i])                                  # ascending
        z[n - 1 - rank] = float(r[i])                          # descending
    lo = np.concatenate([[0.0], _doubling_scan(y)])            # lo[j] = sum of j smallest
    lo2 = np.concatenate([[0.0], _doubling_scan(y * y)])
    hi = np.concatenate([[0.0], _doubling_scan(z)])            # hi[m] = sum of m largest
    hi2 = np.concatenate([[0.0], _doubling_scan(z * z)])
    best_j, best_d = 0, None
    kk = np.float64(k)
    for j in range(k + 1):
        s1 = np.float64(lo[j]) + np.float64(hi[k - j])
        s2 = np.float64(lo2[j]) + np.float64(hi2[k - j])
        dj = kk * s2 - s1 * s1                                 # numpy scalars: no fma
        if best_d is None or dj > best_d:
            best_j, best_d = j, dj
    chosen = order[:best_j] + order[n - (k - best_j):]
    idx = sorted(chosen)
    mask = 0
    for i in idx:
        mask |= 1 << i
    return mask, idx, best_j


def ovf_groups(rewards, group_offsets, k_per_group):
    """OVF over ragged groups of a packed reward vector.

    Returns (masks uint64[P], sel_idx int32 = packed positions of the survivors
    in (group, ascending slot) order, new_offsets int32[P+1])."""
    P = len(k_per_group)
    masks = np.zeros(P, dtype=np.uint64)
    sel = []
    new_off = np.zeros(P + 1, dtype=np.int32)
    for g in range(P):
        b, e = int(group_offsets[g]), int(group_offsets[g + 1])
        if e - b > WAVE:
            raise ValueError("groups above 64 members need ovf_groups_large")
        m, idx, _ = ovf_select(rewards[b:e], int(k_per_group[g]))
        masks[g] = np.uint64(m)
        sel.extend(b + i for i in idx)
        new_off[g + 1] = new_off[g] + len(idx)
    return masks, np.asarray(sel, dtype=np.int32), new_off


def ovf_groups_large(rewards, group_offsets, k_per_group, mask_words):
    """As ovf_groups for groups of up to MAX_GROUP members: masks is uint64[P, mask_words],
    bit i of word w = slot 64 w + i."""
    P = len(k_per_group)
    masks = np.zeros((P, mask_words), dtype=np.uint64)
    sel = []
    new_off = np.zeros(P + 1, dtype=np.int32)
    for g in range(P):
        b, e = int(group_offsets[g]), int(group_offsets[g + 1])
        if e - b > 64 * mask_words:
            raise ValueError("group does not fit the mask")
        m, idx, _ = ovf_select(rewards[b:e], int(k_per_group[g]))
        for w in range(mask_words):
            masks[g, w] = np.uint64((m >> (64 * w)) & 0xFFFFFFFFFFFFFFFF)
        sel.extend(b + i for i in idx)
        new_off[g + 1] = new_off[g] + len(idx)
    return masks, np.asarray(sel, dtype=np.int32), new_off


def compact(array, sel_idx):
    """Ragged gather of the survivors (Sec. 5.1: only the selected trajectories
    continue): row r of the result is row sel_idx[r] of the input."""
    return np.asarray(array)[np.asarray(sel_idx, dtype=np.int64)].copy()


def group_advantages(rewards, group_offsets, eps):
    """Eq. 18 / Eq. 5 per ragged group, population statistics."""
    r = np.asarray(rewards, dtype=np.float64)
    out = np.zeros_like(r)
    for g in range(len(group_offsets) - 1):
        b, e = int(group_offsets[g]), int(group_offsets[g + 1])
        if e == b:
            continue
        mu = np.mean(r[b:e])
        sigma = np.sqrt(np.mean((r[b:e] - mu) ** 2))
        out[b:e] = (r[b:e] - mu) / (sigma + eps)
    return out


def clustered_region(rewards, delta):
    """Eq. 7: indices within delta population-sigmas of the group mean."""
    r = np.asarray(rewards, dtype=np.float64)
    mu = np.mean(r)
    sigma = np.sqrt(np.mean((r - mu) ** 2))
    return np.nonzero(np.abs(r - mu) <= delta * sigma)[0]
