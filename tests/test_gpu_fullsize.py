"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times: sampled
outputs the oracle can compute one by one, plus properties that hold at any size."""
import math
import numpy as np
import pytest
import torch

from oracle import dit, philox, sampler, ovf
from paper_2512_15347_amd import workloads
from pg_progress import say            # not captured: these tests run for minutes

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


# ------------------------------------------------------------------ config 5: stress shapes
def test_cfg5_fused_update_logprob_full_size(lib):
    n, d = 1024, 16 * 128 * 128
    say(f"cfg5b fused update + log-prob {n} x {d}")
    x = torch.empty(n, d, device=DEV); u = torch.empty(n, d, device=DEV)
    for b in range(0, n, 128):
        rows = list(range(b, b + 128))
        x[b:b + 128] = torch.from_numpy(workloads.stress_latent_rows(rows, d, stream=4100)).to(DEV)
        u[b:b + 128] = torch.from_numpy(workloads.stress_latent_rows(rows, d, stream=4200)).to(DEV)
        say(f"  uploaded rows {b + 128}")
    t = sampler.flow_sde_tables(10, 0.7)
    A, B, Cc, step, seed = t["A"][3], t["B"][3], t["C"][3], 3, workloads.MASTER_SEED
    ids = torch.arange(n, dtype=torch.int32, device=DEV)
    xo = torch.empty(n, d, device=DEV)
    logp = torch.zeros(n, device=DEV)
    part = torch.zeros(lib.pg_step_scratch_floats(n, d), device=DEV)
    lib.pg_sde_step_logprob(x, u, xo, logp, None, None, None, ids, n, d, A, B, Cc, seed, step, part)
    torch.cuda.synchronize()
    lp = logp.cpu().numpy().astype(np.float64)
    for r in (0, 511, 1023):
        xr = workloads.stress_latent_rows([r], d, stream=4100)[0].astype(np.float64)
        ur = workloads.stress_latent_rows([r], d, stream=4200)[0].astype(np.float64)
        xi = philox.normals(seed, philox.STREAM_STEP, r, step, d)
        want, mean = sampler.sde_step(xr, ur, A, B, Cc, xi)
        got = xo[r].cpu().numpy().astype(np.float64)
        assert np.max(np.abs(got - want)) < 1e-5 * np.max(np.abs(want))
        assert abs(lp[r] - sampler.gaussian_logprob(want, mean, Cc)) < 2e-5 * abs(lp[r])
    # every trajectory: -1/2 chi^2_d - d (ln C + 1/2 ln 2 pi): mean -d/2, standard deviation sqrt(d/2)
    core = lp + d * (math.log(Cc) + 0.5 * math.log(2 * math.pi))
    assert np.all(np.abs(core + d / 2) < 6 * math.sqrt(d / 2))
    assert abs(core.mean() + d / 2) < 5 * math.sqrt(d / 2 / n)
    # compaction 1024 -> 512 (every other trajectory) on the same tensor, bit for bit
    say("cfg5b compaction 1024 -> 512")
    src = torch.arange(0, n, 2, dtype=torch.int32, device=DEV)
    out = torch.empty(n // 2, d, device=DEV)
    lib.pg_compact_gather(xo, out, src, n // 2, d)
    torch.cuda.synchronize()
    for r in (0, 255, 511):
        np.testing.assert_array_equal(out[r].cpu().numpy().view(np.uint32),
                                      ovf.compact(xo[2 * r:2 * r + 1].cpu().numpy(), [0])[0].view(np.uint32))
    assert torch.equal(out.view(torch.int32), xo.view(torch.int32)[::2])


# ------------------------------------------------------------------ configs 2-4: the network at full width
def _full(lib, name, keep_history=False):
    cfg = workloads.get_config(name)
    say(f"  {name}: drawing weights")
    w = workloads.make_weights(cfg)
    inp = workloads.make_inputs(cfg, w)
    c, keep = lib.make_config(cfg, probe_bias=inp["probe_b"])
    ctx = lib.pg_create(c)
    say(f"  {name}: packing {lib.pg_weights_numel(ctx) / 1e6:.0f} M weights, workspace {lib.pg_workspace_bytes(ctx) / 2**30:.2f} GiB")
    buf = lib.Buffers(ctx, cfg, inputs=inp, weights_flat=lib.pack_weights(ctx, cfg, w), keep_history=keep_history)
    lib.pg_bind(ctx, buf)
    s = cfg["sampler"]
    tables = (sampler.flow_sde_tables(cfg["T"], s["a"]) if s["kind"] == "flow"
              else sampler.ddim_sde_tables(cfg["T"], s["eta"], s["beta0"], s["beta1"], s["T_train"]))
    return cfg, w, inp, tables, ctx, buf


def _sampled_first_step(lib, cfg, w, inp, tables, ctx, buf, seed, sample_ids):
    """Oracle follows the sampled trajectories through step 0 from the seed alone."""
    d, N = cfg["d"], cfg["N"]
    lib.pg_init_group(ctx, seed)
    lib.pg_net_forward(ctx, 0)
    torch.cuda.synchronize()
    u_gpu = {i: buf.u[i].cpu().numpy().astype(np.float64) for i in sample_ids}
    lib.pg_step(ctx, 0)
    torch.cuda.synchronize()
    st = lib.pg_state(ctx, cfg["P"])
    for i in sample_ids:
        g = i // N
        say(f"  oracle forward for trajectory {i} (group {g})")
        x0 = philox.normals(seed, philox.STREAM_INIT, i, 0, d)[None]
        ctx_tok = inp["ctx"][g] if inp.get("ctx") is not None else None
        u = dit.forward(w, cfg, x0, tables["t_in"][0], inp["y"][g], ctx_tok)
        err = np.max(np.abs(u_gpu[i] - u[0])) / np.max(np.abs(u[0]))
        say(f"    u: max err / max|u| = {err:.2e}")
        assert err < 2e-2
        xi = philox.normals(seed, philox.STREAM_STEP, i, 0, d)
        x1, mean = sampler.sde_step(x0, u, tables["A"][0], tables["B"][0], tables["C"][0], xi[None])
        got = buf.x[st["cur_x"]][i].cpu().numpy().astype(np.float64)
        assert np.max(np.abs(got - x1[0])) < 2e-2 * np.max(np.abs(x1[0]))
        lp = float(buf.logp_hist[0, i].cpu())
        assert abs(lp - sampler.gaussian_logprob(x1, mean, tables["C"][0])[0]) < 1e-3 * abs(lp)


def _free_run(lib, cfg, ctx, buf, seed):
    """The whole loop as bench.py runs it, one call per stage.  At every checkpoint the selection the library
    made from ITS OWN proxy rewards is held, bit for bit and for every group, to the oracle's selection on those
    same fp32 rewards (masks, packed survivor positions, new offsets): a near-tie that bf16 network noise
    decides differently from a free-running fp64 loop cannot hide a selection error, nor cause a false one.
    Returns what the float comparisons below need, keyed by original trajectory id."""
    P, N, T = cfg["P"], cfg["N"], cfg["T"]
    lib.pg_init_group(ctx, seed)
    sizes = [N] * P
    rec = dict(proxy={}, sigma={}, u0=None)
    for s in range(T):
        lib.pg_net_forward(ctx, s)
        if s == 0:
            rec["u0"] = buf.u.clone()
        ks = [dict(cfg["schedule"][g]).get(s) for g in range(P)]
        if any(k is not None for k in ks):
            st0 = lib.pg_state(ctx, P)
            off_before = np.asarray(st0["offsets"])
            ids_before = buf.orig_id[st0["cur_id"]].cpu().numpy()[:st0["M"]]
            lib.pg_prune(ctx, s)
            torch.cuda.synchronize()
            r = buf.rewards.cpu().numpy()[:st0["M"]]
            k_g = np.array([ks[g] if ks[g] is not None else sizes[g] for g in range(P)])
            want_masks, want_sel, want_off = ovf.ovf_groups(r, off_before, k_g)
            np.testing.assert_array_equal(buf.masks.cpu().numpy().view(np.uint64)[:P], want_masks)
            np.testing.assert_array_equal(buf.sel_idx.cpu().numpy()[:int(want_off[-1])], want_sel)
            np.testing.assert_array_equal(buf.group_offsets.cpu().numpy(), want_off)
            assert lib.pg_state(ctx, P)["offsets"] == want_off.tolist()
            rec["proxy"][s] = dict(zip(ids_before.tolist(), r.astype(np.float64).tolist()))
            rec["sigma"][s] = [float(np.std(r[off_before[g]:off_before[g + 1]].astype(np.float64))) for g in range(P)]
            sizes = k_g.tolist()
            say(f"  step {s}: selection of all {P} groups equals the oracle's on the same rewards, kept {sizes}")
        lib.pg_step(ctx, s)
    lib.pg_advantages(ctx)
    lib.pg_check(ctx)
    st = lib.pg_state(ctx, P)
    assert st["evals"] == workloads.network_evals(cfg)
    assert st["offsets"] == np.concatenate([[0], np.cumsum(sizes)]).tolist()
    M = st["M"]
    ids = buf.orig_id[st["cur_id"]].cpu().numpy()[:M]
    assert np.all(np.diff(ids) > 0)
    x = buf.x[st["cur_x"]][:M]
    assert torch.isfinite(x).all()
    hist = buf.logp_hist.cpu().numpy()
    surv = np.zeros(P * N, bool); surv[ids] = True
    assert np.isfinite(hist[:, surv]).all() and np.isnan(hist[-1, ~surv]).all()
    adv = buf.adv.cpu().numpy()[:M].astype(np.float64)
    rew = buf.rewards.cpu().numpy()[:M].astype(np.float64)
    for g in range(P):
        b, e = st["offsets"][g], st["offsets"][g + 1]
        assert np.all(ids[b:e] // N == g)
        assert abs(adv[b:e].mean()) < 1e-5 and abs(adv[b:e].std() - 1) < 1e-3
    np.testing.assert_allclose(adv, ovf.group_advantages(rew, st["offsets"], 1e-6), rtol=1e-4, atol=1e-5)
    rec.update(ids=ids, st=st, rewards=rew, logp_hist=hist.astype(np.float64), logp_hist32=hist.copy(),
               logp_sum=buf.logp_sum.cpu().numpy().astype(np.float64))
    return rec


def _follow_in_oracle(cfg, w, inp, tables, seed, ids):
    """The oracle takes the trajectories `ids` (original ids, all of one prompt) from the seed through all T
    steps in fp64: trajectories are independent given that they survive, so no other member of the group is
    needed.  Network output of step 0, proxy reward at the prompt's checkpoints, per-step log-prob, final latent
    and final reward."""
    d, N, T = cfg["d"], cfg["N"], cfg["T"]
    g = ids[0] // N
    assert all(i // N == g for i in ids)
    ctx_tok = inp["ctx"][g] if inp.get("ctx") is not None else None
    x = np.stack([philox.normals(seed, philox.STREAM_INIT, i, 0, d) for i in ids])
    out = dict(proxy={}, logp=np.zeros((T, len(ids))))
    checkpoints = {s for sched in cfg["schedule"] for (s, _) in sched}
    for s in range(T):
        u = dit.forward(w, cfg, x, tables["t_in"][s], inp["y"][g], ctx_tok)
        if s == 0:
            out["u0"] = u
        if s in checkpoints:
            out["proxy"][s] = sampler.linear_reward(sampler.preview(x, u, tables["P"][s], tables["Q"][s]),
                                                    inp["probe_w"], inp["probe_b"])
        xi = np.stack([philox.normals(seed, philox.STREAM_STEP, i, s, d) for i in ids])
        x, mean = sampler.sde_step(x, u, tables["A"][s], tables["B"][s], tables["C"][s], xi)
        out["logp"][s] = sampler.gaussian_logprob(x, mean, tables["C"][s])
        say(f"    oracle step {s} done")
    out["x"] = x
    out["reward"] = sampler.linear_reward(x, inp["probe_w"], inp["probe_b"])
    return out


def _compare_followed(cfg, inp, buf, rec, want, ids):
    """Library against the oracle on the followed trajectories, at the stated tolerances: network output 2e-2 of
    its maximum, every step's log-prob 1e-3 relative, final latent 2e-2 of its maximum.  Rewards: the reward the
    library computes FROM ITS OWN latent is held to 1e-3 of max(|R|, sigma of the group) against the fp64 dot
    product of that latent.  Against the oracle's own trajectory the proxy and final rewards are a unit-norm
    linear functional of latents and network outputs that went through the bf16 network, so they carry the
    latents' tolerance, 2e-2 of max(|R|, sigma_group); what is observed (about 1e-3) is printed."""
    N = cfg["N"]
    g = ids[0] // N
    pos = {int(i): p for p, i in enumerate(rec["ids"])}
    x_gpu = buf.x[rec["st"]["cur_x"]]
    final_sigma = float(np.std(rec["rewards"][rec["st"]["offsets"][g]:rec["st"]["offsets"][g + 1]]))
    for j, i in enumerate(ids):
        u = rec["u0"][i].cpu().numpy().astype(np.float64)
        err_u = np.max(np.abs(u - want["u0"][j])) / np.max(np.abs(want["u0"][j]))
        assert err_u < 2e-2, err_u
        lp = rec["logp_hist"][:, i]
        err_lp = np.max(np.abs(lp - want["logp"][:, j]) / np.abs(want["logp"][:, j]))
        assert err_lp < 1e-3, err_lp
        assert abs(rec["logp_sum"][i] - want["logp"][:, j].sum()) < 1e-3 * abs(want["logp"][:, j].sum())
        err_p = 0.0
        for s, r in want["proxy"].items():
            scale = max(abs(r[j]), rec["sigma"][s][g])
            err_p = max(err_p, abs(rec["proxy"][s][i] - r[j]) / scale)
        got = x_gpu[pos[i]].cpu().numpy().astype(np.float64)
        err_x = np.max(np.abs(got - want["x"][j])) / np.max(np.abs(want["x"][j]))
        err_r = abs(rec["rewards"][pos[i]] - want["reward"][j]) / max(abs(want["reward"][j]), final_sigma)
        # the library's reward of ITS final latent, against the fp64 dot product of that same latent
        own = abs(rec["rewards"][pos[i]] - sampler.linear_reward(got, inp["probe_w"].astype(np.float64), inp["probe_b"]))
        say(f"  trajectory {i}: u {err_u:.1e}, log-prob {err_lp:.1e}, proxy reward {err_p:.1e}, final latent {err_x:.1e}, "
            f"final reward {err_r:.1e} (of max(|R|, sigma_group)), reward of own latent {own:.1e}")
        assert err_x < 2e-2
        assert err_p < 2e-2 and err_r < 2e-2 and own < 1e-3 * max(abs(want["reward"][j]), final_sigma)


def _one_call_loop_is_the_stepwise_loop(lib, cfg, ctx, buf, rec, seed):
    """pg_sample_group, the call bench.py times, against the stage-by-stage run above: same launches in the same order,
    so every output is bit-identical."""
    M = rec["st"]["M"]
    x_step = buf.x[rec["st"]["cur_x"]][:M].clone()
    adv_step = buf.adv[:M].clone()
    lib.pg_sample_group(ctx, seed)
    lib.pg_check(ctx)
    st = lib.pg_state(ctx, cfg["P"])
    assert st["M"] == M and st["offsets"] == rec["st"]["offsets"] and st["evals"] == rec["st"]["evals"]
    assert torch.equal(buf.orig_id[st["cur_id"]][:M].cpu(), torch.from_numpy(rec["ids"]))
    assert torch.equal(buf.x[st["cur_x"]][:M], x_step)
    assert torch.equal(buf.adv[:M], adv_step)
    np.testing.assert_array_equal(buf.logp_hist.cpu().numpy().view(np.uint32), rec["logp_hist32"].view(np.uint32))
    say("  pg_sample_group reproduces the stage-by-stage loop bit for bit")


def _same_weights_log_ratio(lib, cfg, tables, ctx, buf, rec):
    """Eq. 19 at full width with the weights that sampled: every log-ratio is 0 up to the fp32 rounding of the
    stored states, |log r| <~ sqrt(d) ulp(x) / C_s."""
    T, M0, d = cfg["T"], cfg["P"] * cfg["N"], cfg["d"]
    logp_new = torch.zeros(T, M0, device=DEV); ratio = torch.zeros(T, M0, device=DEV); J = torch.zeros(cfg["P"], device=DEV)
    lib.pg_policy_ratio(ctx, buf.weights, 0.2, logp_new, ratio, J)
    lib.pg_check(ctx)
    r = ratio.cpu().numpy().astype(np.float64)
    ids = rec["ids"]
    assert np.isnan(np.delete(r, ids, axis=1)).all()
    worst = 0.0
    for s in range(T):
        xmax = float(buf.x_hist[s + 1][torch.from_numpy(ids.astype(np.int64)).to(DEV)].abs().max())
        bound = 8 * np.sqrt(d) * 2.0 ** -23 * xmax / tables["C"][s]
        got = float(np.max(np.abs(np.log(r[s, ids]))))
        worst = max(worst, got / bound)
        assert got < bound, (s, got, bound)
    say(f"  same-weights log-ratio: at most {worst:.2f} of 8 sqrt(d) ulp(x) / C over {T} steps x {len(ids)} survivors")
    np.testing.assert_allclose(logp_new.cpu().numpy()[:, ids], buf.logp_hist.cpu().numpy()[:, ids], rtol=1e-4)
    assert np.max(np.abs(J.cpu().numpy())) < 1e-2


@pytest.mark.timeout(900)
def test_cfg2_full_size(lib):
    say("cfg2 full size")
    cfg, w, inp, tables, ctx, buf = _full(lib, "cfg2")
    seed = workloads.MASTER_SEED
    rec = _free_run(lib, cfg, ctx, buf, seed)
    ids = [int(rec["ids"][0]), int(rec["ids"][-1])]           # two survivors, through all 20 steps
    say(f"  oracle follows trajectories {ids}")
    want = _follow_in_oracle(cfg, w, inp, tables, seed, ids)
    _compare_followed(cfg, inp, buf, rec, want, ids)
    _one_call_loop_is_the_stepwise_loop(lib, cfg, ctx, buf, rec, seed)
    lib.pg_destroy(ctx)


@pytest.mark.timeout(900)
def test_cfg3_full_size(lib):
    say("cfg3 full size")
    cfg, w, inp, tables, ctx, buf = _full(lib, "cfg3", keep_history=True)
    seed = workloads.MASTER_SEED
    rec = _free_run(lib, cfg, ctx, buf, seed)
    ids = [int(rec["ids"][-1])]                               # a survivor of both prunes, through all 10 steps
    say(f"  oracle follows trajectory {ids}")
    want = _follow_in_oracle(cfg, w, inp, tables, seed, ids)
    _compare_followed(cfg, inp, buf, rec, want, ids)
    _same_weights_log_ratio(lib, cfg, tables, ctx, buf, rec)
    _one_call_loop_is_the_stepwise_loop(lib, cfg, ctx, buf, rec, seed)
    lib.pg_destroy(ctx)


@pytest.mark.timeout(600)
def test_cfg3_dual_stream_full_size(lib):
    say("cfg3 network with dual-stream blocks, full size")
    cfg, w, inp, tables, ctx, buf = _full(lib, "cfg3_mmdit")
    _sampled_first_step(lib, cfg, w, inp, tables, ctx, buf, workloads.MASTER_SEED, [31])
    _free_run(lib, cfg, ctx, buf, workloads.MASTER_SEED)
    lib.pg_destroy(ctx)


@pytest.mark.timeout(900)
def test_cfg4_full_size(lib):
    say("cfg4 full size (8 groups, ragged, one unpruned)")
    cfg, w, inp, tables, ctx, buf = _full(lib, "cfg4")
    seed = workloads.MASTER_SEED
    rec = _free_run(lib, cfg, ctx, buf, seed)
    st = rec["st"]
    assert st["offsets"] == [0, 16, 32, 48, 64, 80, 96, 112, 160] and st["M"] == 160
    ids = [int(rec["ids"][5])]                                # a survivor of the first (twice pruned) group
    say(f"  oracle follows trajectory {ids}")
    want = _follow_in_oracle(cfg, w, inp, tables, seed, ids)
    _compare_followed(cfg, inp, buf, rec, want, ids)
    _one_call_loop_is_the_stepwise_loop(lib, cfg, ctx, buf, rec, seed)
    lib.pg_destroy(ctx)
