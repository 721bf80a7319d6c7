"""GPU parity of the sampling loop (init group, prune, step, advantages) through the C ABI.

The first block drives the loop with the network output taken from the oracle run (written into
the library's `u` buffer before each prune / step), which isolates every non-network stage at the
loop level; the second block runs the library's own network."""
import numpy as np
import pytest
import torch

from oracle import loop, sampler, ovf
from paper_2512_15347_amd import workloads

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def say(msg):
    print(msg, flush=True)


def _oracle(name, seed, **kw):
    cfg = workloads.get_config(name)
    w = workloads.make_weights(cfg)
    inp = workloads.make_inputs(cfg, w)
    s = cfg["sampler"]
    tables = (sampler.flow_sde_tables(cfg["T"], s["a"]) if s["kind"] == "flow"
              else sampler.ddim_sde_tables(cfg["T"], s["eta"], s["beta0"], s["beta1"], s["T_train"]))
    rec = loop.run(cfg, tables, inp, seed, wts=w, keep_u_steps=range(cfg["T"]), **kw)
    return cfg, w, inp, tables, rec


def _compare_final(lib, ctx, buf, cfg, rec, x_tol, lp_rtol=1e-3):
    st = lib.pg_state(ctx, cfg["P"])
    M = st["M"]
    assert st["offsets"] == rec["offsets"].tolist()
    assert st["evals"] == rec["evals"] and st["updates"] == rec["updates"]
    ids = buf.orig_id[st["cur_id"]].cpu().numpy()[:M]
    np.testing.assert_array_equal(ids, rec["orig_id"])
    np.testing.assert_array_equal(buf.group_offsets.cpu().numpy(), rec["offsets"])
    gof = buf.group_of.cpu().numpy()[:M]
    for g in range(cfg["P"]):
        assert np.all(gof[rec["offsets"][g]:rec["offsets"][g + 1]] == g)
    x = buf.x[st["cur_x"]].cpu().numpy()[:M].astype(np.float64)
    for r in range(M):                                   # max error relative to the trajectory's largest entry
        assert np.max(np.abs(x[r] - rec["x"][r])) <= x_tol * np.max(np.abs(rec["x"][r])), r
    hist = buf.logp_hist.cpu().numpy().astype(np.float64)
    want = rec["logp_hist"]
    assert np.array_equal(np.isnan(hist), np.isnan(want))
    ok = ~np.isnan(want)
    np.testing.assert_allclose(hist[ok], want[ok], rtol=lp_rtol)
    lsum = buf.logp_sum.cpu().numpy().astype(np.float64)
    np.testing.assert_allclose(lsum, rec["logp_sum"], rtol=lp_rtol, atol=lp_rtol * np.max(np.abs(want[ok])))
    rew = buf.rewards.cpu().numpy()[:M].astype(np.float64)
    for g in range(cfg["P"]):
        b, e = rec["offsets"][g], rec["offsets"][g + 1]
        scale = max(np.max(np.abs(rec["rewards"][b:e])), np.std(rec["rewards"][b:e]))
        assert np.max(np.abs(rew[b:e] - rec["rewards"][b:e])) <= 1e-3 * scale
    return x, rew


@pytest.mark.parametrize("name", ["cfg1", "cfg4_small", "cfg2_small"])
def test_loop_with_injected_network_output(lib, name):
    say(f"loop (oracle u injected) {name}")
    seed = workloads.MASTER_SEED
    cfg, w, inp, tables, rec = _oracle(name, seed)
    c, keep = lib.make_config(cfg, probe_bias=inp["probe_b"], net=False)
    ctx = lib.pg_create(c)
    buf = lib.Buffers(ctx, cfg, inputs=inp)
    lib.pg_bind(ctx, buf)
    lib.pg_init_group(ctx, seed)
    assert np.max(np.abs(buf.x[0].cpu().numpy().astype(np.float64) - rec["x_init"])) < 2e-5
    for s in range(cfg["T"]):
        ids_s, u_s = rec["u"][s]
        M = lib.pg_state(ctx, cfg["P"])["M"]
        assert M == len(ids_s)
        buf.u[:M].copy_(torch.from_numpy(u_s.astype(np.float32)))
        lib.pg_net_forward(ctx, s)                       # network kind NONE: marks u as supplied
        if s in rec["ovf_masks"]:
            lib.pg_prune(ctx, s)
            torch.cuda.synchronize()
            np.testing.assert_array_equal(buf.masks.cpu().numpy().view(np.uint64), rec["ovf_masks"][s])
            pr = buf.rewards.cpu().numpy()[:M].astype(np.float64)
            assert np.max(np.abs(pr - rec["proxy"][s][1])) <= 1e-3 * max(1.0, np.std(rec["proxy"][s][1]))
        lib.pg_step(ctx, s)
        ids_a, x_a = rec["x_after"][s]
        st = lib.pg_state(ctx, cfg["P"])
        got = buf.x[st["cur_x"]].cpu().numpy()[:st["M"]].astype(np.float64)
        assert np.max(np.abs(got - x_a)) <= 2e-5 * np.max(np.abs(x_a)), s
    lib.pg_advantages(ctx)
    lib.pg_check(ctx)
    _compare_final(lib, ctx, buf, cfg, rec, x_tol=2e-5, lp_rtol=2e-5)
    M = lib.pg_state(ctx, cfg["P"])["M"]
    adv = buf.adv.cpu().numpy()[:M].astype(np.float64)
    np.testing.assert_allclose(adv, rec["adv"], rtol=2e-3, atol=2e-3)
    lib.pg_destroy(ctx)


def test_loop_call_order_is_enforced(lib):
    cfg = workloads.get_config("cfg1")
    c, keep = lib.make_config(cfg, net=False)
    ctx = lib.pg_create(c)
    buf = lib.Buffers(ctx, cfg)
    with pytest.raises(lib.PgError):
        lib.pg_init_group(ctx, 1)                        # not bound yet
    lib.pg_bind(ctx, buf)
    with pytest.raises(lib.PgError):
        lib.pg_step(ctx, 0)                              # not initialised
    lib.pg_init_group(ctx, 1)
    with pytest.raises(lib.PgError) as e:
        lib.pg_step(ctx, 0)                              # no network evaluation yet
    assert e.value.status == lib.PG_ESCHED
    with pytest.raises(lib.PgError) as e:
        lib.pg_net_forward(ctx, 1)                       # the network is evaluated at the step that comes next
    assert e.value.status == lib.PG_ESCHED
    lib.pg_net_forward(ctx, 0)
    with pytest.raises(lib.PgError):
        lib.pg_prune(ctx, 0)                             # step 0 is not a checkpoint
    lib.pg_step(ctx, 0)
    with pytest.raises(lib.PgError) as e:
        lib.pg_advantages(ctx)                           # Eq. 18 is on the final latents: 1 of 10 steps taken
    assert e.value.status == lib.PG_ESCHED
    for s in range(1, 5):
        lib.pg_net_forward(ctx, s)
        if s == 3:
            with pytest.raises(lib.PgError) as e:
                lib.pg_prune(ctx, 4)                     # a prune belongs to the step whose evaluation it uses
            assert e.value.status == lib.PG_ESCHED
        if s == 4:
            with pytest.raises(lib.PgError) as e:
                lib.pg_step(ctx, 4)                      # the schedule prunes here: the funnel must be followed
            assert e.value.status == lib.PG_ESCHED
            lib.pg_prune(ctx, 4)
            with pytest.raises(lib.PgError):
                lib.pg_net_forward(ctx, 5)               # the prune must be consumed by its step first
            with pytest.raises(lib.PgError):
                lib.pg_advantages(ctx)
        lib.pg_step(ctx, s)
    assert lib.pg_state(ctx, 1)["M"] == 4
    with pytest.raises(lib.PgError):
        lib.pg_prune_forced(ctx, 5, [0b10000])           # u is stale
    lib.pg_net_forward(ctx, 5)
    with pytest.raises(lib.PgError):
        lib.pg_prune_forced(ctx, 5, [0b10000])           # names a slot beyond the 4 members
    with pytest.raises(lib.PgError):
        lib.pg_prune_forced(ctx, 5, [0])                 # empty
    lib.pg_check(ctx)
    small = lib.Buffers(ctx, cfg)
    small.c.workspace_bytes = 16
    with pytest.raises(lib.PgError) as e:
        lib.pg_bind(ctx, small)
    assert e.value.status == lib.PG_EWORKSPACE
    lib.pg_destroy(ctx)


def test_nan_reward_is_reported(lib):
    cfg = workloads.get_config("cfg1")
    c, keep = lib.make_config(cfg, net=False)
    ctx = lib.pg_create(c)
    inp = dict(probe_w=np.ones(cfg["d"], np.float32))
    buf = lib.Buffers(ctx, cfg, inputs=inp)
    lib.pg_bind(ctx, buf)
    lib.pg_init_group(ctx, 3)
    for s in range(5):
        buf.u.zero_()
        if s == 4:
            buf.u[2, 7] = float("nan")
        lib.pg_net_forward(ctx, s)
        if s == 4:
            lib.pg_prune(ctx, s)
        lib.pg_step(ctx, s)
    with pytest.raises(lib.PgError) as e:
        lib.pg_check(ctx)
    assert e.value.status == lib.PG_ENAN
    assert lib.pg_state(ctx, 1)["M"] == 4                # the loop itself stayed in bounds
    lib.pg_destroy(ctx)


# ------------------------------------------------------------------ the library's own network
def _gpu_ctx(lib, cfg, w, inp):
    c, keep = lib.make_config(cfg, probe_bias=inp["probe_b"])
    ctx = lib.pg_create(c)
    buf = lib.Buffers(ctx, cfg, inputs=inp, weights_flat=lib.pack_weights(ctx, cfg, w))
    lib.pg_bind(ctx, buf)
    return ctx, buf


@pytest.mark.parametrize("name", ["cfg1", "cfg2_small", "cfg3_small", "cfg4_small", "cfg3_mmdit_small"])
def test_network_output_at_step_0(lib, name):
    say(f"network forward {name}")
    seed = workloads.MASTER_SEED
    cfg, w, inp, tables, rec = _oracle(name, seed)
    ctx, buf = _gpu_ctx(lib, cfg, w, inp)
    lib.pg_init_group(ctx, seed)
    lib.pg_net_forward(ctx, 0)
    torch.cuda.synchronize()
    u = buf.u.cpu().numpy().astype(np.float64)
    want = rec["u"][0][1]
    err = np.max(np.abs(u - want)) / np.max(np.abs(want))
    rms = np.sqrt(np.mean((u - want) ** 2)) / np.sqrt(np.mean(want ** 2))
    say(f"  u: max err / max|u| = {err:.2e}, rms rel = {rms:.2e}")
    assert err < 2e-2 and rms < 1e-2
    lib.pg_destroy(ctx)


@pytest.mark.parametrize("P,N,tile_rows", [(5, 51, 192), (5, 42, 160), (6, 49, 224)])
def test_network_output_with_every_tile_height_of_the_projection(lib, P, N, tile_rows):
    """The fused query / key / value projection stages its value channels through LDS in groups of two 32-row
    slabs; tiles of 192, 160 and 224 rows end in a single slab.  Row counts P * N * 64 chosen so that the
    launcher picks that height for the 768-column projection (255, 252 and 252 tiles for 256 compute units);
    sampled trajectories (first, last, and two whose rows straddle tile boundaries) against the oracle."""
    from oracle import dit, philox
    say(f"network forward with {P * N * 64} rows ({tile_rows}-row tiles in the projection)")
    seed = workloads.MASTER_SEED
    cfg = workloads.get_config("cfg1")
    cfg.update(P=P, N=N, D=256, heads=4, T=2, schedule=[[] for _ in range(P)])
    w = workloads.make_weights(cfg)
    inp = workloads.make_inputs(cfg, w)
    tables = sampler.flow_sde_tables(cfg["T"], cfg["sampler"]["a"])
    ctx, buf = _gpu_ctx(lib, cfg, w, inp)
    lib.pg_init_group(ctx, seed)
    lib.pg_net_forward(ctx, 0)
    torch.cuda.synchronize()
    u_gpu = buf.u.cpu().numpy().astype(np.float64)
    M = P * N
    for i in sorted({0, 2, tile_rows // 64, M // 2, M - 1}):  # trajectory tile_rows // 64 holds the first tile boundary
        x0 = philox.normals(seed, philox.STREAM_INIT, i, 0, cfg["d"])[None]
        u = dit.forward(w, cfg, x0, tables["t_in"][0], inp["y"][i // N], None)
        err = np.max(np.abs(u_gpu[i].reshape(-1) - u[0].reshape(-1))) / np.max(np.abs(u[0]))
        say(f"  trajectory {i}: max err / max|u| = {err:.2e}")
        assert err < 2e-2
    lib.pg_destroy(ctx)


@pytest.mark.parametrize("name", ["cfg1", "cfg2_small", "cfg3_small", "cfg4_small", "cfg3_mmdit_small"])
def test_full_loop_with_own_network(lib, name):
    """Free-running library loop against the free-running oracle: the survivor sets must be the
    oracle's (the seeds used here leave no near-tie), floats within the stated tolerances."""
    say(f"full loop {name}")
    seed = workloads.MASTER_SEED
    cfg, w, inp, tables, rec = _oracle(name, seed)
    ctx, buf = _gpu_ctx(lib, cfg, w, inp)
    lib.pg_sample_group(ctx, seed)
    lib.pg_check(ctx)
    x, rew = _compare_final(lib, ctx, buf, cfg, rec, x_tol=2e-2)
    M = lib.pg_state(ctx, cfg["P"])["M"]
    adv = buf.adv.cpu().numpy()[:M].astype(np.float64)
    np.testing.assert_allclose(adv, ovf.group_advantages(rew, rec["offsets"], 1e-6), rtol=1e-4, atol=1e-5)
    for g in range(cfg["P"]):
        a = adv[rec["offsets"][g]:rec["offsets"][g + 1]]
        assert abs(a.mean()) < 1e-5 and abs(a.std() - 1) < 1e-3
    lib.pg_destroy(ctx)


def test_forced_masks_follow_the_oracle(lib):
    """Survivors imposed from the oracle run (test hook): the library still reports its own OVF
    decision for the proxy rewards it computed, and that decision is the oracle's."""
    name, seed = "cfg3_small", 99
    say(f"forced loop {name}")
    cfg, w, inp, tables, rec = _oracle(name, seed)
    ctx, buf = _gpu_ctx(lib, cfg, w, inp)
    shadow = torch.zeros(cfg["P"], dtype=torch.int64, device=DEV)
    lib.pg_init_group(ctx, seed)
    for s in range(cfg["T"]):
        lib.pg_net_forward(ctx, s)
        if s in rec["used_masks"]:
            lib.pg_prune_forced(ctx, s, rec["used_masks"][s], shadow)
            torch.cuda.synchronize()
            np.testing.assert_array_equal(shadow.cpu().numpy().view(np.uint64), rec["ovf_masks"][s])
            np.testing.assert_array_equal(buf.masks.cpu().numpy().view(np.uint64), rec["used_masks"][s])
        lib.pg_step(ctx, s)
    lib.pg_advantages(ctx)
    lib.pg_check(ctx)
    _compare_final(lib, ctx, buf, cfg, rec, x_tol=2e-2)
    lib.pg_destroy(ctx)


PAPER_SCHEDULES = {
    "paper_std_small": [48] * 6 + [24] * 2 + [12] * 2,
    "paper_flash_small": [24] * 6 + [16] * 2 + [12] * 2,
    "paper_diffusion_small": [48] * 31 + [32] * 10 + [8] * 9,
    "paper_ablation32_small": [32] * 6 + [16] * 2 + [8] * 2,
    "paper_ablation48_small": [48] * 6 + [24] * 2 + [8] * 2,
    "paper_ablation64_small": [64] * 6 + [32] * 2 + [8] * 2,
}


@pytest.mark.parametrize("name", sorted(PAPER_SCHEDULES))
def test_paper_schedules(lib, name):
    """The paper's own schedules (Sec. 6.1: 48 -> 24 -> 12 at steps 5 and 7 of T = 10, the 24 -> 16 -> 12
    efficiency variant, 48 -> 32 -> 8 at steps 30 and 40 of T = 50 for the diffusion model; Sec. 6.3: 32, 48
    and 64 pruned to 8) on small networks: free-running library against the free-running oracle."""
    seed = 2512
    say(f"full loop {name}")
    cfg, w, inp, tables, rec = _oracle(name, seed)
    assert rec["active"] == PAPER_SCHEDULES[name]
    ctx, buf = _gpu_ctx(lib, cfg, w, inp)
    lib.pg_sample_group(ctx, seed)
    lib.pg_check(ctx)
    _compare_final(lib, ctx, buf, cfg, rec, x_tol=2e-2)
    lib.pg_destroy(ctx)


def test_full_width_group_of_64_and_explicit_tables(lib):
    """Largest group the selection takes (64, the paper's largest G_max), caller-supplied step tables,
    a latent whose size is not a multiple of the streaming chunk."""
    cfg = workloads.get_config("cfg1")
    cfg.update(N=64, C=5, H=18, W=14, T=4, schedule=[[(1, 33), (2, 7)]])
    cfg["d"] = 5 * 18 * 14
    cfg["Li"] = 9 * 7
    say("loop N=64 with explicit tables")
    seed = 77
    w = workloads.make_weights(cfg); inp = workloads.make_inputs(cfg, w)
    tables = sampler.flow_sde_tables(4, 0.35)
    rec = loop.run(cfg, tables, inp, seed, wts=w)
    c, keep = lib.make_config(cfg, probe_bias=inp["probe_b"], tables=tables)
    ctx = lib.pg_create(c)
    buf = lib.Buffers(ctx, cfg, inputs=inp, weights_flat=lib.pack_weights(ctx, cfg, w))
    lib.pg_bind(ctx, buf)
    lib.pg_sample_group(ctx, seed)
    lib.pg_check(ctx)
    _compare_final(lib, ctx, buf, cfg, rec, x_tol=2e-2)
    assert lib.pg_state(ctx, 1)["M"] == 7
    lib.pg_destroy(ctx)


def test_sample_group_is_repeatable_and_seed_dependent(lib):
    cfg = workloads.get_config("cfg3_small")
    w = workloads.make_weights(cfg); inp = workloads.make_inputs(cfg, w)
    ctx, buf = _gpu_ctx(lib, cfg, w, inp)
    outs = []
    for seed in (5, 5, 6):
        lib.pg_sample_group(ctx, seed)
        lib.pg_check(ctx)
        st = lib.pg_state(ctx, 1)
        outs.append((buf.x[st["cur_x"]][:st["M"]].clone(), buf.logp_sum.clone(), buf.masks.clone()))
    assert torch.equal(outs[0][0], outs[1][0]) and torch.equal(outs[0][1], outs[1][1])
    assert not torch.equal(outs[0][0], outs[2][0])
    lib.pg_destroy(ctx)


def test_whole_loop_replays_from_a_hip_graph(lib):
    """The one-call loop copies nothing from the host and never waits for the device, so it can be recorded into a
    HIP graph (a caller that must not pay 2 400 launches per tiny group does that).  Every replay, with eager work
    of the library and synchronisations in between, must give the eager loop's result bit for bit."""
    name, seed = "cfg1", 4242
    say(f"graph capture {name}")
    cfg = workloads.get_config(name)
    w = workloads.make_weights(cfg); inp = workloads.make_inputs(cfg, w)
    ctx, buf = _gpu_ctx(lib, cfg, w, inp)
    P = cfg["P"]
    lib.pg_sample_group(ctx, seed)                       # eager: also warms every one-time set-up of the launches
    lib.pg_check(ctx)
    st = lib.pg_state(ctx, P)
    M = st["M"]
    want = dict(x=buf.x[st["cur_x"]][:M].clone(), adv=buf.adv[:M].clone(), hist=buf.logp_hist.clone(),
                ids=buf.orig_id[st["cur_id"]][:M].clone(), masks=buf.masks.clone())
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        graph.capture_begin()
        lib.pg_sample_group(ctx, seed)                   # launches go to the capturing stream
        graph.capture_end()
    torch.cuda.synchronize()
    for rep in range(3):
        # eager work of the library between the replays, with another seed, so that a replay cannot pass on leftovers
        lib.pg_sample_group(ctx, seed + 1 + rep)
        lib.pg_check(ctx)
        assert not torch.equal(buf.x[lib.pg_state(ctx, P)["cur_x"]][:M], want["x"])
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(buf.x[st["cur_x"]][:M], want["x"]), rep
        assert torch.equal(buf.adv[:M], want["adv"]) and torch.equal(buf.masks, want["masks"])
        assert torch.equal(buf.orig_id[st["cur_id"]][:M], want["ids"])
        assert torch.equal(buf.logp_hist.view(torch.int32), want["hist"].view(torch.int32))
        assert int(buf.status[0]) == 0
    lib.pg_destroy(ctx)
