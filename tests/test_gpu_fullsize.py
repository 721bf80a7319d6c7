"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times: sampled
outputs the oracle can compute one by one, plus properties that hold at any size."""
import math
import numpy as np
import pytest
import torch

from oracle import dit, philox, sampler, ovf
from paper_2512_15347_amd import workloads

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def say(msg):
    print(msg, flush=True)


def _check_mask_is_variance_optimal_split(r, mask, k):
    """Properties of the OVF result that hold for any input: k members, the members are the j lowest
    and k-j highest under the (value, slot) order for some j, and no other split has a larger variance."""
    n = len(r)
    idx = [i for i in range(n) if (int(mask) >> i) & 1]
    assert len(idx) == k and int(mask) >> n == 0
    order = sorted(range(n), key=lambda i: (float(r[i]), i))
    r64 = np.asarray(r, np.float64)
    var = lambda sel: float(np.var(r64[sel])) if len(sel) else 0.0
    splits = [sorted(order[:j] + order[n - (k - j):]) for j in range(k + 1)]
    assert idx in splits
    best = max(var(s) for s in splits)
    assert var(idx) >= best * (1 - 1e-12) - 1e-300


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
def _full(lib, name):
    cfg = workloads.get_config(name)
    say(f"  {name}: drawing weights")
    w = workloads.make_weights(cfg)
    inp = workloads.make_inputs(cfg, w)
    c, keep = lib.make_config(cfg, probe_bias=inp["probe_b"])
    ctx = lib.pg_create(c)
    say(f"  {name}: packing {lib.pg_weights_numel(ctx) / 1e6:.0f} M weights, workspace {lib.pg_workspace_bytes(ctx) / 2**30:.2f} GiB")
    buf = lib.Buffers(ctx, cfg, inputs=inp, weights_flat=lib.pack_weights(ctx, cfg, w))
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


def _free_run_properties(lib, cfg, ctx, buf, seed):
    """Whole loop as bench.py runs it; everything checked holds at any size."""
    P, N, T = cfg["P"], cfg["N"], cfg["T"]
    lib.pg_init_group(ctx, seed)
    sizes = [N] * P
    for s in range(T):
        lib.pg_net_forward(ctx, s)
        ks = [dict(cfg["schedule"][g]).get(s) for g in range(P)]
        if any(k is not None for k in ks):
            off_before = lib.pg_state(ctx, P)["offsets"]
            lib.pg_prune(ctx, s)
            torch.cuda.synchronize()
            r = buf.rewards.cpu().numpy()
            masks = buf.masks.cpu().numpy().view(np.uint64)
            sel = buf.sel_idx.cpu().numpy()
            pos = 0
            for g in range(P):
                k = ks[g] if ks[g] is not None else sizes[g]
                rg = r[off_before[g]:off_before[g + 1]]
                _check_mask_is_variance_optimal_split(rg, masks[g], k)
                want_sel = [off_before[g] + i for i in range(sizes[g]) if (int(masks[g]) >> i) & 1]
                assert sel[pos:pos + k].tolist() == want_sel
                pos += k
                sizes[g] = k
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
    d, Cs = cfg["d"], None
    adv = buf.adv.cpu().numpy()[:M].astype(np.float64)
    rew = buf.rewards.cpu().numpy()[:M].astype(np.float64)
    for g in range(P):
        b, e = st["offsets"][g], st["offsets"][g + 1]
        assert np.all(ids[b:e] // N == g)
        assert abs(adv[b:e].mean()) < 1e-5 and abs(adv[b:e].std() - 1) < 1e-3
    np.testing.assert_allclose(adv, ovf.group_advantages(rew, st["offsets"], 1e-6), rtol=1e-4, atol=1e-5)
    # final reward of a sampled survivor from the final latent (fp64 dot product)
    xr = x[0].cpu().numpy().astype(np.float64)
    return xr, rew[0]


def test_cfg2_full_size(lib):
    say("cfg2 full size")
    cfg, w, inp, tables, ctx, buf = _full(lib, "cfg2")
    _sampled_first_step(lib, cfg, w, inp, tables, ctx, buf, workloads.MASTER_SEED, [0, 23])
    xr, r0 = _free_run_properties(lib, cfg, ctx, buf, workloads.MASTER_SEED)
    assert abs(r0 - sampler.linear_reward(xr, inp["probe_w"].astype(np.float64), inp["probe_b"])) < 1e-3
    lib.pg_destroy(ctx)


@pytest.mark.timeout(600)
def test_cfg3_full_size(lib):
    say("cfg3 full size")
    cfg, w, inp, tables, ctx, buf = _full(lib, "cfg3")
    _sampled_first_step(lib, cfg, w, inp, tables, ctx, buf, workloads.MASTER_SEED, [47])
    xr, r0 = _free_run_properties(lib, cfg, ctx, buf, workloads.MASTER_SEED)
    assert abs(r0 - sampler.linear_reward(xr, inp["probe_w"].astype(np.float64), inp["probe_b"])) < 1e-3
    lib.pg_destroy(ctx)


@pytest.mark.timeout(600)
def test_cfg3_dual_stream_full_size(lib):
    say("cfg3 network with dual-stream blocks, full size")
    cfg, w, inp, tables, ctx, buf = _full(lib, "cfg3_mmdit")
    _sampled_first_step(lib, cfg, w, inp, tables, ctx, buf, workloads.MASTER_SEED, [31])
    xr, r0 = _free_run_properties(lib, cfg, ctx, buf, workloads.MASTER_SEED)
    assert abs(r0 - sampler.linear_reward(xr, inp["probe_w"].astype(np.float64), inp["probe_b"])) < 1e-3
    lib.pg_destroy(ctx)


@pytest.mark.timeout(600)
def test_cfg4_full_size(lib):
    say("cfg4 full size (8 groups, ragged, one unpruned)")
    cfg, w, inp, tables, ctx, buf = _full(lib, "cfg4")
    _sampled_first_step(lib, cfg, w, inp, tables, ctx, buf, workloads.MASTER_SEED, [7 * 48 + 5])
    _free_run_properties(lib, cfg, ctx, buf, workloads.MASTER_SEED)
    st = lib.pg_state(ctx, cfg["P"])
    assert st["offsets"] == [0, 16, 32, 48, 64, 80, 96, 112, 160] and st["M"] == 160
    lib.pg_destroy(ctx)
