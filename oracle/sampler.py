"""Reverse-SDE sampler of the pruned-sampling loop, fp64 (test infrastructure only).

What the paper fixes (Sec. 5.1): one reverse step is the Euler-Maruyama update
    x' = x + b(x, t) dt + sigma_t sqrt(dt) xi,           xi ~ N(0, I)      (Eq. 13)
with the backbone-specific drift of Eq. 12, the policy of a step is the
isotropic Gaussian that update induces (the sentence after Eq. 19), and the
pruning preview is ONE deterministic Euler step of the probability-flow ODE
(Eq. 14) from the current latent to the terminal time (Eq. 15).

What the paper leaves open and the reading taken here:
* Rectified flow (Eq. 3, Eq. 4).  Time is the noise fraction tau running
  1 -> 0:  x_tau = (1 - tau) x_data + tau eps,  the network predicts
  v = dx/dtau = eps - x_data.  Then eps_hat = x + (1 - tau) v and the score is
  -eps_hat / tau, so the drift of Eq. 12 (RF case) is
      b = v + sigma^2 / (2 tau) * (x + (1 - tau) v)        (dt = dtau < 0).
  sigma_tau = a sqrt(tau / (1 - tau)) with noise level a; at tau = 1 the
  denominator is clamped to (1 - tau_1) = 1/T.
* Diffusion (Eq. 1, Eq. 2).  The paper gives only the continuous SDE; the
  discretisation is the DDIM(eta) posterior step on a T_train-entry linear
  beta table with an (S+1)-point integer timestep grid from T_train-1 to 0.
Both are written as the affine map  x' = A x + B u + C xi  with per-step
scalars, u being the network output (v for flow, eps_hat for diffusion).

Pins: marginal preservation with an analytic point-mass network (exact for the
DDIM step, exact in the mean and O(dt^2) in the variance for the flow step),
reduction to the plain Euler ODE when the noise level is 0, closed-form
Gaussian log-density via scipy, chi-square moments of the log-prob.
"""
import math
import numpy as np

LN_2PI = math.log(2.0 * math.pi)


def flow_sde_tables(T, a):
    """Per-step scalars for the rectified-flow SDE, steps s = 0..T-1.

    Returns dict of fp64 arrays A, B, C (update), P, Q (preview x_hat = P x + Q u),
    tau (noise fraction at the start of step s), t_in (network time input)."""
    A = np.zeros(T); B = np.zeros(T); C = np.zeros(T)
    P = np.zeros(T); Q = np.zeros(T); tau = np.zeros(T); t_in = np.zeros(T)
    for s in range(T):
        ts = 1.0 - s / T
        tn = 1.0 - (s + 1) / T
        dt = tn - ts                                   # negative
        denom = max(1.0 - ts, 1.0 / T)                 # clamp at tau = 1
        sig2 = a * a * ts / denom
        # x' = x + [v + sig2/(2 tau) (x + (1-tau) v)] dt + sqrt(sig2 |dt|) xi
        A[s] = 1.0 + sig2 * dt / (2.0 * ts)
        B[s] = dt * (1.0 + sig2 * (1.0 - ts) / (2.0 * ts))
        C[s] = math.sqrt(sig2 * abs(dt))
        # ODE preview (Eq. 15, RF case of Eq. 14): remaining time is tau, drift v
        P[s] = 1.0
        Q[s] = -ts
        tau[s] = ts
        t_in[s] = 1000.0 * ts
    return dict(A=A, B=B, C=C, P=P, Q=Q, tau=tau, t_in=t_in)


def ddim_timesteps(S, T_train):
    """S+1 integer timesteps from T_train-1 down to 0, evenly spread, rounded."""
    return [((S - i) * (T_train - 1) + S // 2) // S for i in range(S + 1)]


def ddim_sde_tables(S, eta, beta0, beta1, T_train=1000):
    """Per-step scalars for the DDIM(eta) posterior step on a linear beta table."""
    betas = np.linspace(beta0, beta1, T_train, dtype=np.float64)
    abar = np.cumprod(1.0 - betas)
    ts = ddim_timesteps(S, T_train)
    A = np.zeros(S); B = np.zeros(S); C = np.zeros(S)
    P = np.zeros(S); Q = np.zeros(S); t_in = np.zeros(S)
    for i in range(S):
        at = abar[ts[i]]
        ap = abar[ts[i + 1]]
        # x0_hat = (x - sqrt(1-at) eps) / sqrt(at)
        s2 = eta * eta * (1.0 - ap) / (1.0 - at) * (1.0 - at / ap)
        # mean = sqrt(ap) x0_hat + sqrt(1 - ap - s2) eps
        A[i] = math.sqrt(ap / at)
        B[i] = math.sqrt(1.0 - ap - s2) - math.sqrt(ap * (1.0 - at) / at)
        C[i] = math.sqrt(s2)
        # preview: the deterministic single jump to the terminal time = x0_hat
        P[i] = 1.0 / math.sqrt(at)
        Q[i] = -math.sqrt((1.0 - at) / at)
        t_in[i] = float(ts[i])
    return dict(A=A, B=B, C=C, P=P, Q=Q, t_in=t_in, abar=abar, timesteps=ts)


def sde_step(x, u, A, B, C, xi):
    """Euler-Maruyama update in affine form (Eq. 13): returns (x', mean)."""
    mean = A * x + B * u
    return mean + C * xi, mean


def gaussian_logprob(x_next, mean, C):
    """log N(x_next; mean, C^2 I) summed over all latent dimensions of each
    trajectory (last axis) -- the log-density of the policy induced by Eq. 13."""
    d = x_next.shape[-1]
    r2 = np.sum((x_next - mean) ** 2, axis=-1)
    return -r2 / (2.0 * C * C) - d * math.log(C) - 0.5 * d * LN_2PI


def noise_logprob(xi, C):
    """Same quantity written through the noise itself: x' - mean = C xi."""
    d = xi.shape[-1]
    return -0.5 * np.sum(xi * xi, axis=-1) - d * math.log(C) - 0.5 * d * LN_2PI


def preview(x, u, P, Q):
    """One-step ODE projection to the terminal time (Eq. 15) in affine form."""
    return P * x + Q * u


def linear_reward(x_hat, w, b):
    """Synthetic stand-in for decoder + reward model of Eq. 16: R = b + <w, x_hat>."""
    return b + x_hat @ w
