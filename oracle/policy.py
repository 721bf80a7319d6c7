"""Per-step importance ratio and clipped surrogate of the pruned group, forward only, fp64
(test infrastructure only).

Sec. 5.1 after Eq. 18: with a_t = x_{t+dt} - x_t and s_t = (x_t, t), the per-step ratio is
r_t = pi_theta(a_t | s_t) / pi_old(a_t | s_t) (Eq. 19), pi being the Gaussian policy induced by the
Euler-Maruyama step (Eq. 13): N(A_t x_t + B_t u_theta(x_t, t), C_t^2 I).  The objective restricted to
the K survivors is the mean over survivors and steps of min(r A, clip(r, 1-e, 1+e) A) (Eq. 20, first
term).  The KL term of Eq. 20 needs a reference policy and is not computed here.

Pins: identical weights give ratio 1 and the objective equal to the mean advantage; a constant shift of
the network output gives a closed-form log-ratio; the clipping cases are checked branch by branch.
"""
import numpy as np

from . import sampler, dit


def transition_logprob(x, u, x_next, A, B, C):
    """log N(x_next; A x + B u, C^2 I) summed over the latent dimensions."""
    return sampler.gaussian_logprob(x_next, A * x + B * u, C)


def clipped_surrogate(ratio, adv, clip_eps):
    """Eq. 20, first term, for arrays ratio[T, K] and adv[K]: mean over K and T of
    min(r A, clip(r, 1 - eps, 1 + eps) A)."""
    r = np.asarray(ratio, dtype=np.float64)
    a = np.asarray(adv, dtype=np.float64)[None, :]
    return float(np.mean(np.minimum(r * a, np.clip(r, 1.0 - clip_eps, 1.0 + clip_eps) * a)))


def policy_ratio(cfg, tables, inputs, rec, wts_new, clip_eps=0.2, net=None):
    """Re-evaluate the stored transitions of the survivors of `rec` (a loop.run record) under new
    network weights.  Returns dict with logp_new [T, M0] (NaN off the survivors), ratio [T, M0] and
    J [P] = the clipped surrogate of each group."""
    P, N, T = cfg["P"], cfg["N"], cfg["T"]
    M0 = P * N
    ids = np.asarray(rec["orig_id"])
    off = np.asarray(rec["offsets"])
    logp_new = np.full((T, M0), np.nan)

    def state(s):                      # x_s of the survivors, from the stored trajectory
        if s == 0:
            return rec["x_init"][ids]
        sid, xs = rec["x_after"][s - 1]
        pos = {int(i): k for k, i in enumerate(sid)}
        return xs[[pos[int(i)] for i in ids]]

    for s in range(T):
        x, x_next = state(s), state(s + 1)
        u = np.empty_like(x)
        for g in range(P):
            b, e = off[g], off[g + 1]
            if net is not None:
                u[b:e] = net(x[b:e], s, g)
            else:
                ctx = inputs["ctx"][g] if inputs.get("ctx") is not None else None
                u[b:e] = dit.forward(wts_new, cfg, x[b:e], tables["t_in"][s], inputs["y"][g], ctx)
        logp_new[s, ids] = transition_logprob(x, u, x_next, tables["A"][s], tables["B"][s], tables["C"][s])
    ratio = np.exp(logp_new - rec["logp_hist"])
    J = np.array([clipped_surrogate(ratio[:, ids[off[g]:off[g + 1]]], rec["adv"][off[g]:off[g + 1]], clip_eps)
                  for g in range(P)])
    return dict(logp_new=logp_new, ratio=ratio, J=J)
