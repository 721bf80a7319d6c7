"""The selection entry point that allocates nothing (its scan scratch is a device array inside the library)
against the entry point that takes a scratch buffer: identical outputs, on two calls in a row, the second
smaller than the first (the built-in array keeps the first call's contents)."""
import numpy as np
import pytest
import torch

from oracle import ovf
from paper_2512_15347_amd import workloads

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _ragged_case(n_groups, seed):
    rng = np.random.default_rng([workloads.MASTER_SEED, 7000, seed])
    sizes = rng.integers(1, 65, size=n_groups)
    offs = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    k = np.array([int(rng.integers(1, n + 1)) for n in sizes], dtype=np.int32)
    r = workloads.stress_rewards(n_groups, 64, seed=workloads.MASTER_SEED + seed).reshape(-1)[:offs[-1]].copy()
    return r, offs, k


def _select(lib, fn_name, r, offs, k):
    n_groups = len(k)
    rd = torch.from_numpy(r).to(DEV)
    od = torch.from_numpy(offs).to(DEV)
    kd = torch.from_numpy(k).to(DEV)
    masks = torch.full((n_groups,), -1, dtype=torch.int64, device=DEV)
    sel = torch.full((int(k.sum()),), -1, dtype=torch.int32, device=DEV)
    noffs = torch.full((n_groups + 1,), -1, dtype=torch.int32, device=DEV)
    status = torch.zeros(4, dtype=torch.int32, device=DEV)
    if fn_name == "pg_ovf_select":
        scratch = torch.zeros(lib.pg_ovf_scratch_ints(n_groups), dtype=torch.int32, device=DEV)
        lib.pg_ovf_select(rd, od, kd, n_groups, masks, sel, noffs, status, scratch)
    else:
        lib.pg_ovf_select_noalloc(rd, od, kd, n_groups, masks, sel, noffs, status)
    torch.cuda.synchronize()
    assert int(status[0]) == 0
    return masks.cpu().numpy().view(np.uint64), sel.cpu().numpy(), noffs.cpu().numpy()


def test_noalloc_selection_equals_the_scratch_taking_one(lib):
    # 20 000 ragged groups span ten scan blocks; the second call (700 groups) fits in one
    for n_groups, seed in ((20000, 1), (700, 2)):
        print(f"no-alloc selection, {n_groups} ragged groups", flush=True)
        r, offs, k = _ragged_case(n_groups, seed)
        want = _select(lib, "pg_ovf_select", r, offs, k)
        got = _select(lib, "pg_ovf_select_noalloc", r, offs, k)
        for a, b in zip(got, want):
            np.testing.assert_array_equal(a, b)
        if n_groups <= 1000:                          # and both equal the oracle's selection
            m, s, no = ovf.ovf_groups(r, offs, k)
            np.testing.assert_array_equal(got[0], m)
            np.testing.assert_array_equal(got[1], s)
            np.testing.assert_array_equal(got[2], no)


def test_noalloc_selection_rejects_what_its_scratch_cannot_hold(lib):
    one = torch.zeros(4, dtype=torch.int32, device=DEV)
    with pytest.raises(lib.PgError) as e:
        lib.pg_ovf_select_noalloc(one, one, one, lib.PG_OVF_NOALLOC_MAX_GROUPS + 1, one, one, one, one)
    assert e.value.status == lib.PG_ESHAPE and "at most" in str(e.value)
    with pytest.raises(lib.PgError):
        lib.pg_ovf_select_noalloc(None, one, one, 1, one, one, one, one)
    lib.pg_ovf_select_noalloc(None, None, None, 0, None, None, None, None)      # nothing to do
