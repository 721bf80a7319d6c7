"""Pins for oracle/loop.py (CPU only): the survivor funnel follows the schedule
(Sec. 5.1, Sec. 5.2), pruned trajectories take no further steps, noise is tied to
the original trajectory, and analytic point-mass networks give known outcomes."""
import math
import numpy as np

from oracle import loop, sampler, philox, ovf
from paper_2512_15347_amd import workloads


def _setup(name):
    cfg = workloads.get_config(name)
    w = workloads.make_weights(cfg)
    inp = workloads.make_inputs(cfg, w)
    s = cfg["sampler"]
    tables = (sampler.flow_sde_tables(cfg["T"], s["a"]) if s["kind"] == "flow"
              else sampler.ddim_sde_tables(cfg["T"], s["eta"], s["beta0"], s["beta1"], s["T_train"]))
    return cfg, w, inp, tables


def test_trajectory_step_counts_of_the_benchmark_configs():
    # evaluations happen before the prune of a checkpoint step
    want = dict(cfg1=60, cfg2=312, cfg3=288, cfg4=2496)
    for name, n in want.items():
        assert workloads.network_evals(workloads.get_config(name)) == n


def test_cfg1_funnel_counts_and_records():
    cfg, w, inp, tables = _setup("cfg1")
    rec = loop.run(cfg, tables, inp, workloads.MASTER_SEED, wts=w, keep_u_steps=(0,))
    assert rec["evals"] == 60 and rec["updates"] == 56
    assert rec["active"] == [8] * 5 + [4] * 5
    assert rec["offsets"].tolist() == [0, 4] and len(rec["orig_id"]) == 4
    assert np.all(np.diff(rec["orig_id"]) > 0)
    surv = set(rec["orig_id"].tolist())
    for i in range(8):
        col = rec["logp_hist"][:, i]
        if i in surv:
            assert np.all(np.isfinite(col))
            assert abs(rec["logp_sum"][i] - np.sum(col)) < 1e-9
        else:                                      # early-terminated: steps 0..3 only
            assert np.all(np.isfinite(col[:4])) and np.all(np.isnan(col[4:]))
    m = int(rec["ovf_masks"][4][0])
    assert bin(m).count("1") == 4 and sorted(surv) == [i for i in range(8) if (m >> i) & 1]
    # the recorded OVF decision is the OVF of the recorded proxy rewards
    ids, r = rec["proxy"][4]
    assert ovf.ovf_select(r.astype(np.float32), 4)[0] == m
    assert abs(rec["adv"].mean()) < 1e-9


def test_multi_group_ragged_funnel():
    cfg, w, inp, tables = _setup("cfg4_small")
    rec = loop.run(cfg, tables, inp, 5, wts=w)
    assert rec["active"] == [36, 36, 27, 27, 21, 21]
    assert rec["offsets"].tolist() == [0, 4, 9, 21]
    assert rec["evals"] == sum(rec["active"]) == workloads.network_evals(cfg)
    assert rec["orig_id"][9:].tolist() == list(range(24, 36))      # pinned group untouched
    for g in range(3):
        seg = rec["orig_id"][rec["offsets"][g]:rec["offsets"][g + 1]]
        assert np.all((seg >= 12 * g) & (seg < 12 * (g + 1))) and np.all(np.diff(seg) > 0)
        a = rec["adv"][rec["offsets"][g]:rec["offsets"][g + 1]]
        assert abs(a.mean()) < 1e-9 and abs(a.std() - 1) < 1e-4


def test_forced_masks_are_obeyed_and_noise_follows_original_id():
    cfg, w, inp, tables = _setup("cfg1")
    forced = {4: np.array([0b10100101], dtype=np.uint64)}
    rec = loop.run(cfg, tables, inp, 77, wts=w, forced_masks=forced)
    assert rec["orig_id"].tolist() == [0, 2, 5, 7]
    free = loop.run(cfg, tables, inp, 77, wts=w)
    # before the checkpoint both runs are identical; a trajectory that survives in both
    # runs sees the same noise afterwards, so its whole path is identical
    both = sorted(set(rec["orig_id"].tolist()) & set(free["orig_id"].tolist()))
    for i in both:
        a = rec["x"][rec["orig_id"].tolist().index(i)]
        b = free["x"][free["orig_id"].tolist().index(i)]
        np.testing.assert_array_equal(a, b)
        np.testing.assert_array_equal(rec["logp_hist"][:, i], free["logp_hist"][:, i])


def test_logprob_history_is_closed_form_of_the_noise():
    cfg, w, inp, tables = _setup("cfg1")
    rec = loop.run(cfg, tables, inp, 3, wts=w)
    d = cfg["d"]
    for s in (0, 6):
        for i in rec["orig_id"][:2]:
            xi = philox.normals(3, philox.STREAM_STEP, int(i), s, d)
            want = -0.5 * np.sum(xi * xi) - d * math.log(tables["C"][s]) - 0.5 * d * math.log(2 * math.pi)
            assert abs(rec["logp_hist"][s, i] - want) < 1e-7 * abs(want)


def test_ddim_point_mass_network_reaches_the_data_point():
    # eps_hat exact for data concentrated at x*: every preview equals x*, the proxy reward
    # is the same for all trajectories, and the final latent is N(sqrt(abar_0) x*, (1-abar_0) I)
    cfg, w, inp, tables = _setup("cfg2_small")
    rng = np.random.default_rng(0)
    xstar = rng.standard_normal(cfg["d"])
    ab, ts = tables["abar"], tables["timesteps"]

    def net(x, s, g):
        at = ab[ts[s]]
        return (x - math.sqrt(at) * xstar) / math.sqrt(1 - at)

    rec = loop.run(cfg, tables, inp, 11, net=net)
    ids, r = rec["proxy"][2]
    want_r = inp["probe_b"] + float(inp["probe_w"].astype(np.float64) @ xstar)
    np.testing.assert_allclose(r, want_r, rtol=0, atol=1e-9)
    resid = (rec["x"] - math.sqrt(ab[0]) * xstar) / math.sqrt(1 - ab[0])
    assert abs(resid.mean()) < 5 / math.sqrt(resid.size) and abs(resid.var() - 1) < 0.1
    assert np.max(np.abs(rec["x"] - xstar)) < 0.1
    # initial latents at t = 999 are pure noise from the init stream
    np.testing.assert_array_equal(rec["x_after"][0][0], np.arange(6))


def test_flow_point_mass_network_contracts_to_the_data_point():
    cfg, w, inp, tables = _setup("cfg3_small")
    cfg["T"] = 40; cfg["schedule"] = [[(10, 8), (20, 4)]]
    tables = sampler.flow_sde_tables(40, 0.7)
    rng = np.random.default_rng(1)
    xstar = rng.standard_normal(cfg["d"])

    def net(x, s, g):
        tau = tables["tau"][s]
        return (x - xstar) / tau                    # v = e - x* with e = (x - (1-tau) x*)/tau

    rec = loop.run(cfg, tables, inp, 12, net=net)
    for s in (10, 20):
        np.testing.assert_allclose(rec["proxy"][s][1], inp["probe_b"] + inp["probe_w"].astype(np.float64) @ xstar, atol=1e-9)
    assert np.sqrt(np.mean((rec["x"] - xstar) ** 2)) < 0.12
    assert rec["active"][0] == 12 and rec["active"][11] == 8 and rec["active"][-1] == 4
