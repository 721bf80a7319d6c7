"""Pins for oracle/sampler.py (CPU only): what the mathematics fixes about the
reverse step (Eq. 13), its Gaussian policy and the one-step preview (Eq. 15)."""
import math
import numpy as np
from scipy import stats

from oracle import sampler, philox


def test_flow_first_step_values():
    # noise level 0.7, T = 10: with the clamp at tau = 1, sigma^2 = a^2 T, so
    # A = 1 - a^2/2, B = -1/T (the (1-tau) factor vanishes), C = a.
    t = sampler.flow_sde_tables(10, 0.7)
    assert abs(t["A"][0] - (1 - 0.49 / 2)) < 1e-15
    assert abs(t["B"][0] + 0.1) < 1e-15
    assert abs(t["C"][0] - 0.7) < 1e-15
    assert np.all(t["C"] > 0)                       # every step is stochastic


def test_flow_zero_noise_is_plain_euler():
    t = sampler.flow_sde_tables(7, 0.0)
    np.testing.assert_allclose(t["A"], 1.0, atol=0)
    np.testing.assert_allclose(t["B"], -1.0 / 7, rtol=1e-15)
    np.testing.assert_allclose(t["C"], 0.0, atol=0)


def test_flow_marginals_point_mass():
    # Data = point mass at x*: x_tau = (1-tau) x* + tau e, and the exact velocity is
    # v = e - x*.  One step must map the mean coefficient (1-tau) -> (1-tau') exactly.
    # The noise variance goes tau^2 -> tau'^2 + a^2/(sT) + a^4/(4 s^2) (expand the
    # square by hand with 1 - tau = s/T): the Euler-Maruyama defect, second order in
    # the step and vanishing away from tau = 1.
    a = 0.7
    for T in (10, 50, 400):
        t = sampler.flow_sde_tables(T, a)
        for s in range(1, T):                       # s = 0 uses the clamp
            tau, taun = 1 - s / T, 1 - (s + 1) / T
            A, B, C = t["A"][s], t["B"][s], t["C"][s]
            assert abs(A * (1 - tau) - B - (1 - taun)) < 1e-13
            var = (A * tau + B) ** 2 + C ** 2
            assert abs(var - (taun ** 2 + a * a / (s * T) + a ** 4 / (4 * s * s))) < 1e-12


def test_flow_variance_recursion_converges():
    # scalar recursion of the noise variance under the exact point-mass-at-0 velocity
    # v = x / tau (clamped first step included) lands near tau_T^2 = 0 as T grows
    finals = []
    for T in (10, 100, 1000):
        t = sampler.flow_sde_tables(T, 0.7)
        V = 1.0
        for s in range(T):
            tau = 1 - s / T
            V = (t["A"][s] + t["B"][s] / tau) ** 2 * V + t["C"][s] ** 2
        finals.append(V)
    assert finals[2] < finals[1] < finals[0] < 0.1
    assert finals[2] < 2e-3


def test_flow_preview_recovers_point_mass():
    rng = np.random.default_rng(0)
    xs = rng.standard_normal(32)
    t = sampler.flow_sde_tables(10, 0.7)
    for s in range(10):
        tau = 1 - s / 10
        e = rng.standard_normal(32)
        x = (1 - tau) * xs + tau * e
        v = e - xs
        np.testing.assert_allclose(sampler.preview(x, v, t["P"][s], t["Q"][s]), xs, atol=1e-13)


def test_ddim_grid_and_positivity():
    t = sampler.ddim_sde_tables(20, 1.0, 1e-4, 0.02)
    ts = t["timesteps"]
    assert ts[0] == 999 and ts[-1] == 0 and len(ts) == 21
    assert all(a > b for a, b in zip(ts[:-1], ts[1:]))
    assert np.all(t["C"] > 0)
    # linear beta table: abar_0 = 1 - 1e-4
    assert abs(t["abar"][0] - (1 - 1e-4)) < 1e-15
    assert abs(t["abar"][999] - np.prod(1 - np.linspace(1e-4, 0.02, 1000))) < 1e-15


def test_ddim_marginals_point_mass_exact():
    # x_t = sqrt(abar_t) x* + sqrt(1-abar_t) e with the exact noise prediction e:
    # the posterior step gives x_prev ~ N(sqrt(abar_p) x*, (1-abar_p) I) for ANY step size.
    for S, eta in ((20, 1.0), (7, 1.0), (20, 0.5), (20, 0.0)):
        t = sampler.ddim_sde_tables(S, eta, 1e-4, 0.02)
        ab, ts = t["abar"], t["timesteps"]
        for i in range(S):
            at, ap = ab[ts[i]], ab[ts[i + 1]]
            A, B, C = t["A"][i], t["B"][i], t["C"][i]
            assert abs(A * math.sqrt(at) - math.sqrt(ap)) < 1e-12
            assert abs((A * math.sqrt(1 - at) + B) ** 2 + C ** 2 - (1 - ap)) < 1e-12
            # preview returns x* exactly
            assert abs(t["P"][i] * math.sqrt(at) - 1) < 1e-12
            assert abs(t["P"][i] * math.sqrt(1 - at) + t["Q"][i]) < 1e-12
        if eta == 0.0:
            np.testing.assert_allclose(t["C"], 0.0, atol=0)


def test_ddim_eta1_is_ancestral_variance():
    # eta = 1 makes the step variance the DDPM posterior variance
    # beta~ = (1-abar_p)/(1-abar_t) * (1 - abar_t/abar_p)
    t = sampler.ddim_sde_tables(999, 1.0, 1e-4, 0.02)       # unit stride: abar_t/abar_p = 1-beta_t
    assert t["timesteps"] == list(range(999, -1, -1))
    betas = np.linspace(1e-4, 0.02, 1000)
    ab = t["abar"]
    for i in (0, 10, 500, 998):
        tt = 999 - i
        want = (1 - ab[tt - 1]) / (1 - ab[tt]) * betas[tt]
        assert abs(t["C"][i] ** 2 - want) < 1e-14


def test_logprob_is_gaussian_density():
    rng = np.random.default_rng(3)
    x = rng.standard_normal((3, 50)); u = rng.standard_normal((3, 50)); xi = rng.standard_normal((3, 50))
    A, B, C = 0.9, -0.13, 0.37
    xn, mean = sampler.sde_step(x, u, A, B, C, xi)
    np.testing.assert_allclose(xn, x * A + u * B + xi * C, rtol=1e-15)
    lp = sampler.gaussian_logprob(xn, mean, C)
    want = stats.norm.logpdf(xn, loc=mean, scale=C).sum(axis=-1)
    np.testing.assert_allclose(lp, want, rtol=1e-12)
    np.testing.assert_allclose(sampler.noise_logprob(xi, C), lp, rtol=1e-9)
    # multivariate form, one trajectory
    mv = stats.multivariate_normal(mean=mean[0], cov=C * C * np.eye(50)).logpdf(xn[0])
    assert abs(mv - lp[0]) < 1e-9 * abs(mv)


def test_logprob_chi_square_moments():
    d, n = 4096, 64
    C = 0.25
    xi = np.stack([philox.normals(5, philox.STREAM_STEP, i, 0, d) for i in range(n)])
    core = sampler.noise_logprob(xi, C) + d * math.log(C) + 0.5 * d * sampler.LN_2PI   # = -1/2 sum xi^2
    assert abs(core.mean() + d / 2) < 5 * math.sqrt(d / 2 / n)
    assert 0.6 < core.var() / (d / 2) < 1.5


def test_linear_reward():
    rng = np.random.default_rng(1)
    w = rng.standard_normal(40); xh = rng.standard_normal((5, 40))
    r = sampler.linear_reward(xh, w, 0.3)
    for i in range(5):
        assert abs(r[i] - (0.3 + sum(float(a) * float(b) for a, b in zip(w, xh[i])))) < 1e-12
