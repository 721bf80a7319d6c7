"""GPU parity of the kernel-level entry points against the oracle (through the C ABI)."""
import math
import numpy as np
import pytest
import torch

from oracle import philox, sampler, ovf
from paper_2512_15347_amd import workloads

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a))
    return (t.to(dtype) if dtype else t).to(DEV)


def say(msg):
    print(msg, flush=True)


# ------------------------------------------------------------------ initial latents / Philox
@pytest.mark.parametrize("n,d", [(3, 1024), (2, 4100), (5, 16384)])
def test_init_latents_matches_oracle(lib, n, d):
    say(f"init_latents n={n} d={d}")
    ids = np.array([7, 0, 123456, 5, 9][:n], dtype=np.int32)
    x = torch.zeros(n, d, device=DEV)
    seed = 0x1234567890ABCDEF
    lib.pg_init_latents(x, dev(ids), seed)
    torch.cuda.synchronize()
    want = np.stack([philox.normals(seed, philox.STREAM_INIT, int(i), 0, d) for i in ids])
    got = x.cpu().numpy().astype(np.float64)
    # fp32 hardware log2 / sin / cos / sqrt against the fp64 transform
    assert np.max(np.abs(got - want)) < 2e-5
    assert abs(got.mean()) < 5 / math.sqrt(got.size) and abs(got.var() - 1) < 0.05


def test_init_latents_empty_and_bad_shape(lib):
    x = torch.zeros(0, 64, device=DEV)
    lib.pg_init_latents(x, torch.zeros(0, dtype=torch.int32, device=DEV), 1)
    with pytest.raises(lib.PgError):
        lib.pg_init_latents(torch.zeros(2, 6, device=DEV), torch.zeros(2, dtype=torch.int32, device=DEV), 1)


# ------------------------------------------------------------------ fused update + log-prob
def _step_case(lib, n, d, seed, step, A, B, Cc, src=None, ids=None):
    x, u = workloads.stress_latents(n, d, seed=seed)
    ids = np.arange(n, dtype=np.int32) * 3 + 1 if ids is None else ids
    n_out = n if src is None else len(src)
    ids_out = ids if src is None else ids[src]
    xo = torch.zeros(n_out, d, device=DEV)
    logp = torch.zeros(n_out, device=DEV)
    hist = torch.full((int(ids.max()) + 1,), float("nan"), device=DEV)
    lsum = torch.ones(int(ids.max()) + 1, device=DEV)
    part = torch.zeros(lib.pg_step_scratch_floats(n_out, d), device=DEV)
    lib.pg_sde_step_logprob(dev(x), dev(u), xo, logp, hist, lsum, None if src is None else dev(src.astype(np.int32)),
                            dev(ids_out.astype(np.int32)), n_out, d, A, B, Cc, seed, step, part)
    torch.cuda.synchronize()
    rows = np.arange(n) if src is None else src
    xi = np.stack([philox.normals(seed, philox.STREAM_STEP, int(i), step, d) for i in ids_out])
    want_x, mean = sampler.sde_step(x[rows].astype(np.float64), u[rows].astype(np.float64), A, B, Cc, xi)
    want_lp = sampler.gaussian_logprob(want_x, mean, Cc)
    got_x = xo.cpu().numpy().astype(np.float64)
    assert np.max(np.abs(got_x - want_x)) < 1e-5 * max(1.0, np.max(np.abs(want_x)))
    got_lp = logp.cpu().numpy().astype(np.float64)
    np.testing.assert_allclose(got_lp, want_lp, rtol=2e-5)          # bar: 1e-3 relative
    h = hist.cpu().numpy()
    np.testing.assert_array_equal(h[ids_out], logp.cpu().numpy())
    assert np.isnan(np.delete(h, ids_out)).all()
    np.testing.assert_allclose(lsum.cpu().numpy()[ids_out], 1.0 + logp.cpu().numpy(), rtol=1e-6)


@pytest.mark.parametrize("n,d", [(4, 1024), (3, 4096 * 2 + 520), (2, 65536)])
def test_sde_step_logprob_matches_oracle(lib, n, d):
    say(f"sde_step n={n} d={d}")
    t = sampler.flow_sde_tables(10, 0.7)
    _step_case(lib, n, d, seed=42, step=3, A=t["A"][3], B=t["B"][3], Cc=t["C"][3])


def test_sde_step_with_gather_on_read(lib):
    say("sde_step gather")
    src = np.array([0, 2, 3, 7, 8, 11])
    _step_case(lib, 12, 4096 + 256, seed=9, step=5, A=0.93, B=-0.21, Cc=0.31, src=src)


@pytest.mark.parametrize("n,d,gather", [(4, 1024, False), (3, 4096 * 2 + 520, False), (12, 4096 + 256, True)])
def test_sde_step_bf16_storage_matches_oracle(lib, n, d, gather):
    """Storage variant: bf16 latents and network output in, bf16 latents out.  The oracle takes the same
    bf16-representable inputs; the result may differ from the exactly rounded one by the fp32 arithmetic, i.e.
    by at most one bf16 rounding step; the log-prob is that of the fp32 call."""
    say(f"sde_step bf16 n={n} d={d}")
    seed, step, A, B, Cc = 17, 2, 0.93, -0.21, 0.31
    x, u = workloads.stress_latents(n, d, seed=seed)
    x = workloads.bf16_round(x); u = workloads.bf16_round(u)
    src = np.array([0, 2, 3, 7, 8, 11]) if gather else None
    ids = np.arange(n, dtype=np.int32) * 2 + 5
    rows = np.arange(n) if src is None else src
    ids_out = ids[rows]
    n_out = len(rows)
    bits = lambda a: torch.from_numpy(workloads.bf16_bits(a).view(np.int16)).to(DEV)
    xo = torch.zeros(n_out, d, dtype=torch.int16, device=DEV)
    logp = torch.zeros(n_out, device=DEV)
    part = torch.zeros(lib.pg_step_scratch_floats(n_out, d), device=DEV)
    lib.pg_sde_step_logprob_bf16(bits(x), bits(u), xo, logp, None, None, None if src is None else dev(src.astype(np.int32)),
                                 dev(ids_out.astype(np.int32)), n_out, d, A, B, Cc, seed, step, part)
    torch.cuda.synchronize()
    xi = np.stack([philox.normals(seed, philox.STREAM_STEP, int(i), step, d) for i in ids_out])
    want_x, mean = sampler.sde_step(x[rows].astype(np.float64), u[rows].astype(np.float64), A, B, Cc, xi)
    got = (xo.cpu().numpy().view(np.uint16).astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    # half a bf16 step is 2^-9 of the value's power of two (<= 2^-8 relative); allow the fp32 arithmetic on top
    assert np.all(np.abs(got - want_x) <= 2.0 ** -8 * np.abs(want_x) * 1.02 + 1e-30 + 2e-6)
    exact = workloads.bf16_round(want_x.astype(np.float32)).astype(np.float64)
    assert np.mean(got == exact) > 0.995                             # rounding decisions differ only near ties
    np.testing.assert_allclose(logp.cpu().numpy().astype(np.float64), sampler.gaussian_logprob(want_x, mean, Cc), rtol=2e-5)
    with pytest.raises(lib.PgError):
        lib.pg_sde_step_logprob_bf16(bits(x), bits(u), xo, logp, None, None, None, dev(ids_out.astype(np.int32)), n_out, 1028, A, B,
                                     Cc, seed, step, part)


def test_sde_step_rejects_bad_arguments(lib):
    x = torch.zeros(2, 64, device=DEV); o = torch.zeros(2, 64, device=DEV)
    ids = torch.zeros(2, dtype=torch.int32, device=DEV); part = torch.zeros(2, device=DEV)
    with pytest.raises(lib.PgError):                                  # C = 0: no density
        lib.pg_sde_step_logprob(x, x, o, None, None, None, None, ids, 2, 64, 1.0, 1.0, 0.0, 1, 0, part)
    with pytest.raises(lib.PgError):                                  # in-place gather would race
        lib.pg_sde_step_logprob(x, x, x, None, None, None, None, ids, 2, 64, 1.0, 1.0, 0.5, 1, 0, part)
    lib.pg_sde_step_logprob(x, x, o, None, None, None, None, ids, 0, 64, 1.0, 1.0, 0.5, 1, 0, part)   # empty: no-op


# ------------------------------------------------------------------ preview + reward, gather
@pytest.mark.parametrize("n,d,with_u", [(5, 1024, True), (3, 16384 + 64, True), (4, 4096, False)])
def test_preview_reward_matches_oracle(lib, n, d, with_u):
    say(f"preview_reward n={n} d={d} u={with_u}")
    x, u = workloads.stress_latents(n, d, seed=5)
    w = np.random.default_rng(1).standard_normal(d).astype(np.float32) / math.sqrt(d)
    Pc, Qc, bias = (1.3, -0.6, 0.25) if with_u else (1.0, 0.0, -0.5)
    r = torch.zeros(n, device=DEV)
    part = torch.zeros(lib.pg_step_scratch_floats(n, d), device=DEV)
    lib.pg_preview_reward(dev(x), dev(u) if with_u else None, dev(w), r, n, d, Pc, Qc, bias, part)
    torch.cuda.synchronize()
    want = sampler.linear_reward(sampler.preview(x.astype(np.float64), u.astype(np.float64), Pc, Qc),
                                 w.astype(np.float64), bias)
    np.testing.assert_allclose(r.cpu().numpy(), want, rtol=0, atol=1e-5)      # bar: 1e-3 of sigma_R ~ 1


def test_compact_gather_is_bit_exact(lib):
    say("compact_gather")
    rng = np.random.default_rng(2)
    for n, d in ((16, 1024), (9, 4096 * 3 + 4)):
        x = rng.standard_normal((n, d), dtype=np.float32)
        x.view(np.uint32)[0, :4] = [0x7FC00001, 0x80000000, 0x00000001, 0xFF800000]   # NaN payload, -0, denormal, -inf
        src = np.sort(rng.choice(n, n // 2, replace=False)).astype(np.int32)
        out = torch.zeros(len(src), d, device=DEV)
        lib.pg_compact_gather(dev(x), out, dev(src), len(src), d)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(out.cpu().numpy().view(np.uint32), ovf.compact(x, src).view(np.uint32))
    lib.pg_compact_gather(dev(x), out, dev(src), 0, d)                   # empty


# ------------------------------------------------------------------ OVF
def _run_ovf(lib, rewards, offsets, ks):
    P = len(ks)
    total = int(np.sum(np.maximum(ks, 0)))          # a negative count reserves no slots
    masks = torch.zeros(P, dtype=torch.int64, device=DEV)
    sel = torch.full((max(total, 1),), -1, dtype=torch.int32, device=DEV)
    newoff = torch.zeros(P + 1, dtype=torch.int32, device=DEV)
    status = torch.zeros(4, dtype=torch.int32, device=DEV)
    scratch = torch.zeros(max(lib.pg_ovf_scratch_ints(P), 1), dtype=torch.int32, device=DEV)
    lib.pg_ovf_select(dev(rewards.astype(np.float32)), dev(np.asarray(offsets, np.int32)), dev(np.asarray(ks, np.int32)),
                      P, masks, sel, newoff, status, scratch)
    torch.cuda.synchronize()
    return (masks.cpu().numpy().view(np.uint64), sel.cpu().numpy()[:total], newoff.cpu().numpy(),
            int(status.cpu()[0]))


def test_ovf_stress_config_bit_exact(lib):
    say("ovf 4096 x 64 -> 16")
    for offset in (0.0, 23.0):
        r = workloads.stress_rewards(4096, 64, offset=offset)
        off = np.arange(4097) * 64
        ks = np.full(4096, 16)
        masks, sel, newoff, status = _run_ovf(lib, r.reshape(-1), off, ks)
        w_masks, w_sel, w_off = ovf.ovf_groups(r.reshape(-1), off, ks)
        assert status == 0
        np.testing.assert_array_equal(masks, w_masks)
        np.testing.assert_array_equal(sel, w_sel)
        np.testing.assert_array_equal(newoff, w_off)


def test_ovf_ragged_groups_ties_and_degenerate_k(lib):
    say("ovf ragged")
    rng = np.random.default_rng(8)
    sizes = [48, 48, 32, 17, 64, 1, 2, 64, 33, 5, 48, 64]
    ks =    [32, 48, 16, 5, 16, 1, 1, 64, 32, 5, 1, 63]
    off = np.concatenate([[0], np.cumsum(sizes)])
    r = rng.standard_normal(off[-1]).astype(np.float32)
    r[off[2]:off[3]] = np.round(r[off[2]:off[3]] * 2) / 2        # many exact ties
    r[off[8]:off[9]] = 0.75                                       # all equal
    r[off[4]] = -0.0; r[off[4] + 1] = 0.0
    masks, sel, newoff, status = _run_ovf(lib, r, off, ks)
    w_masks, w_sel, w_off = ovf.ovf_groups(r, off, ks)
    assert status == 0
    np.testing.assert_array_equal(masks, w_masks)
    np.testing.assert_array_equal(sel, w_sel)
    np.testing.assert_array_equal(newoff, w_off)


def test_ovf_groups_above_64_members(lib):
    """Groups of up to 1024 members (one workgroup per group), ragged, with ties, bit for bit against the
    oracle; groups of at most 64 members must get the 64-slot routine's answer."""
    say("ovf large groups")
    rng = np.random.default_rng(21)
    sizes = [1024, 65, 100, 513, 64, 48, 1, 777, 200, 1000, 129, 2]
    ks =    [512, 7, 50, 40, 16, 24, 1, 776, 200, 1, 64, 1]
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    r = (rng.standard_normal(off[-1]) * np.where(rng.random(off[-1]) < 0.8, 0.05, 1.0)).astype(np.float32)
    r[off[2]:off[3]] = np.round(r[off[2]:off[3]] * 4) / 4         # many exact ties
    r[off[10]:off[11]] = -1.5                                      # all equal
    words = 16
    w_masks, w_sel, w_off = ovf.ovf_groups_large(r, off, ks, words)
    P = len(sizes)
    masks = torch.full((P, words), -1, dtype=torch.int64, device=DEV)
    sel = torch.full((int(np.sum(ks)),), -1, dtype=torch.int32, device=DEV)
    noff = torch.zeros(P + 1, dtype=torch.int32, device=DEV)
    status = torch.zeros(4, dtype=torch.int32, device=DEV)
    scratch = torch.zeros(lib.pg_ovf_scratch_ints(P), dtype=torch.int32, device=DEV)
    lib.pg_ovf_select_large(torch.from_numpy(r).to(DEV), torch.from_numpy(off).to(DEV),
                            torch.tensor(ks, dtype=torch.int32, device=DEV), P, words, masks, sel, noff, status, scratch)
    torch.cuda.synchronize()
    assert status[0].item() == 0
    np.testing.assert_array_equal(masks.cpu().numpy().view(np.uint64), w_masks)
    np.testing.assert_array_equal(noff.cpu().numpy(), w_off)
    np.testing.assert_array_equal(sel.cpu().numpy(), w_sel)
    # the small groups agree with the one-wave kernel
    for g in (4, 5, 6, 11):
        m64, _, _ = ovf.ovf_groups(r[off[g]:off[g + 1]], [0, sizes[g]], [ks[g]])
        assert int(w_masks[g, 0]) == int(m64[0])
    # a group that does not fit the mask, a bad k and a non-finite reward are flagged
    off2 = torch.tensor([0, 200, 210, 300], dtype=torch.int32, device=DEV)
    k2 = torch.tensor([5, 11, 3], dtype=torch.int32, device=DEV)
    r2 = torch.from_numpy(r[:300].copy()).to(DEV); r2[250] = float("inf")
    masks2 = torch.full((3, 2), -1, dtype=torch.int64, device=DEV)
    sel2 = torch.full((19,), -1, dtype=torch.int32, device=DEV)
    status.zero_()
    lib.pg_ovf_select_large(r2, off2, k2, 3, 2, masks2, sel2, noff[:4], status, scratch)
    torch.cuda.synchronize()
    assert status[0].item() == 3
    m2 = masks2.cpu().numpy().view(np.uint64)
    assert not m2[0].any() and not m2[1].any() and int(m2[2, 0]) == 0b111
    assert sel2.cpu().numpy()[16:].tolist() == [210, 211, 212]


def test_ovf_many_groups_and_schedule_sizes(lib):
    say("ovf 20000 groups")
    rng = np.random.default_rng(9)
    sizes = rng.choice([24, 32, 48, 64], size=20000)
    ks = np.array([{24: 12, 32: 16, 48: 32, 64: 8}[int(s)] for s in sizes])
    off = np.concatenate([[0], np.cumsum(sizes)])
    r = (rng.standard_normal(off[-1]) * 0.3 + 22.0).astype(np.float32)
    masks, sel, newoff, status = _run_ovf(lib, r, off, ks)
    w_masks, w_sel, w_off = ovf.ovf_groups(r, off, ks)
    assert status == 0
    np.testing.assert_array_equal(masks, w_masks)
    np.testing.assert_array_equal(sel, w_sel)
    np.testing.assert_array_equal(newoff, w_off)


def test_ovf_flags_non_finite_and_bad_counts(lib):
    say("ovf error flags")
    r = np.array([0.1, np.nan, 0.3, 0.4, 1.0, 2.0, 3.0, 4.0], dtype=np.float32)
    masks, sel, newoff, status = _run_ovf(lib, r, [0, 4, 8], [2, 2])
    assert status & 1
    assert masks[1] == np.uint64(ovf.ovf_select(r[4:], 2)[0])    # the clean group is still selected
    assert set(sel[:2].tolist()) <= {0, 1, 2, 3}                  # indices stay inside the group
    r[1] = np.inf
    assert _run_ovf(lib, r, [0, 4, 8], [2, 2])[3] & 1
    r[1] = 0.2
    masks, sel, newoff, status = _run_ovf(lib, r, [0, 4, 8], [5, 2])   # k > n
    assert status & 2 and masks[0] == 0
    # the five slots reserved for the bad group hold rows of that group, and the clean group behind it is intact
    assert newoff.tolist() == [0, 5, 7] and set(sel[:5].tolist()) <= {0, 1, 2, 3}
    assert sel[5:7].tolist() == [4 + i for i in range(4) if (int(masks[1]) >> i) & 1]
    # a negative count reserves nothing: the groups behind it keep non-negative offsets
    masks, sel, newoff, status = _run_ovf(lib, r, [0, 4, 8], [-3, 2])
    assert status & 2 and masks[0] == 0 and newoff.tolist() == [0, 0, 2]
    assert masks[1] == np.uint64(ovf.ovf_select(r[4:], 2)[0])
    masks, sel, newoff, status = _run_ovf(lib, r, [0, 0, 8], [0, 3])   # an empty group is fine
    assert status == 0 and masks[0] == 0 and newoff.tolist() == [0, 0, 3]


# ------------------------------------------------------------------ advantages
def test_group_advantages_match_oracle(lib):
    say("advantages")
    rng = np.random.default_rng(3)
    sizes = [16, 12, 4, 1, 8, 64, 16]
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    r = (rng.standard_normal(off[-1]) * 0.3 + 22.0).astype(np.float32)
    r[off[4]:off[5]] = 1.25
    adv = torch.zeros(int(off[-1]), device=DEV)
    for eps in (1e-6, 1e-2):
        lib.pg_group_advantages(dev(r), dev(off), len(sizes), eps, adv)
        torch.cuda.synchronize()
        want = ovf.group_advantages(r.astype(np.float64), off, eps)
        np.testing.assert_allclose(adv.cpu().numpy(), want, rtol=1e-5, atol=1e-6)
    a = adv.cpu().numpy()
    assert np.all(a[off[3]:off[5]] == 0)
