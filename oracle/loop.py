"""The expanded-group sampling loop with in-loop pruning, fp64 (test infrastructure only).

Control flow follows Sec. 5.1 / Sec. 5.2 and the pipeline figure of the paper:
draw G_max initial latents per prompt; for each of the T steps evaluate the
network on every ACTIVE trajectory; at a checkpoint step score the one-step ODE
preview of every active trajectory (Eq. 14-16), keep the variance-maximising
subset per group (the arg-max after Eq. 16) and drop the rest before the update;
apply the Euler-Maruyama update (Eq. 13) and record the Gaussian log-prob of
the step; after the last step compute final rewards and the group-normalised
advantages of the survivors (Eq. 18).

Reading taken where the paper is silent: "prune at step s" means after the
network evaluation of step s and before its update, so the evaluation is
shared by the preview and the update of the survivors.
"""
import numpy as np

from . import philox, sampler, ovf, dit


def run(cfg, tables, inputs, seed, wts=None, net=None, forced_masks=None, eps=1e-6,
        keep_u_steps=()):
    """Sample P groups of N trajectories with pruning.

    cfg:     dict with P, N, C, H, W, T, schedule (per group: list of (step, k)),
             and the network fields used by dit.forward.
    tables:  output of sampler.flow_sde_tables / ddim_sde_tables.
    inputs:  dict with probe_w [d], probe_b, y [P, D], optional ctx [P, L_c, D_c].
    net:     optional callable (x[M,d], step, group) -> u[M,d] replacing the DiT
             (analytic networks in the pins).
    forced_masks: optional {step: uint64[P]} survivor masks over each group's
             CURRENT slots, imposed instead of the OVF result (the OVF result
             is still computed and recorded).
    """
    P, N, T = cfg["P"], cfg["N"], cfg["T"]
    d = cfg["C"] * cfg["H"] * cfg["W"]
    M0 = P * N
    orig_id = np.arange(M0, dtype=np.int64)
    offsets = np.arange(P + 1, dtype=np.int64) * N
    x = np.stack([philox.normals(seed, philox.STREAM_INIT, i, 0, d) for i in range(M0)])
    logp_hist = np.full((T, M0), np.nan)
    logp_sum = np.zeros(M0)
    rec = dict(proxy={}, ovf_masks={}, used_masks={}, ovf_j={}, u={}, x_after={},
               evals=0, updates=0, active=[], x_init=x.copy())
    sched = [dict(cfg["schedule"][g]) for g in range(P)]

    for s in range(T):
        rec["active"].append(len(orig_id))
        # network evaluation on every active trajectory, group by group
        u = np.empty_like(x)
        for g in range(P):
            b, e = offsets[g], offsets[g + 1]
            if net is not None:
                u[b:e] = net(x[b:e], s, g)
            else:
                ctx = inputs["ctx"][g] if inputs.get("ctx") is not None else None
                u[b:e] = dit.forward(wts, cfg, x[b:e], tables["t_in"][s], inputs["y"][g], ctx)
        rec["evals"] += len(orig_id)
        if s in keep_u_steps:
            rec["u"][s] = (orig_id.copy(), u.copy())

        if any(s in sc for sc in sched):
            k_g = np.array([sched[g].get(s, offsets[g + 1] - offsets[g]) for g in range(P)])
            xh = sampler.preview(x, u, tables["P"][s], tables["Q"][s])
            r = sampler.linear_reward(xh, inputs["probe_w"], inputs["probe_b"])
            r32 = r.astype(np.float32)
            masks, sel, new_off = ovf.ovf_groups(r32, offsets, k_g)
            rec["proxy"][s] = (orig_id.copy(), r.copy())
            rec["ovf_masks"][s] = masks.copy()
            if forced_masks is not None and s in forced_masks:
                masks = np.asarray(forced_masks[s], dtype=np.uint64)
                sel = []
                new_off = np.zeros(P + 1, dtype=np.int64)
                for g in range(P):
                    n_g = int(offsets[g + 1] - offsets[g])
                    idx = [i for i in range(n_g) if (int(masks[g]) >> i) & 1]
                    sel.extend(int(offsets[g]) + i for i in idx)
                    new_off[g + 1] = new_off[g] + len(idx)
                sel = np.asarray(sel, dtype=np.int64)
            rec["used_masks"][s] = masks.copy()
            x, u, orig_id = ovf.compact(x, sel), ovf.compact(u, sel), ovf.compact(orig_id, sel)
            offsets = np.asarray(new_off, dtype=np.int64)

        A, B, C = tables["A"][s], tables["B"][s], tables["C"][s]
        xi = np.stack([philox.normals(seed, philox.STREAM_STEP, int(i), s, d) for i in orig_id])
        x_next, mean = sampler.sde_step(x, u, A, B, C, xi)
        lp = sampler.gaussian_logprob(x_next, mean, C)
        logp_hist[s, orig_id] = lp
        logp_sum[orig_id] += lp
        x = x_next
        rec["updates"] += len(orig_id)
        rec["x_after"][s] = (orig_id.copy(), x.copy())

    rewards = sampler.linear_reward(x, inputs["probe_w"], inputs["probe_b"])
    adv = ovf.group_advantages(rewards, offsets, eps)
    rec.update(x=x, orig_id=orig_id, offsets=offsets, logp_hist=logp_hist, logp_sum=logp_sum,
               rewards=rewards, adv=adv)
    return rec
