"""Pins for the oracle's metric (paper Eq. 1) and DDIM scheduler.

Each check compares the oracle with something fixed outside it: values worked by
hand, closed forms of the DDIM recursion, and the DDPM posterior-mean coefficient the
paper prints (Preliminaries, equation for mu_theta).
"""
import math

import numpy as np
import pytest

from oracle import parastep_oracle as O


# ---------------------------------------------------------------- rel_mae, Eq. (1)
def test_rel_mae_hand_worked():
    a = [1.0, -2.0, 3.0, 0.0, 4.0]
    b = [0.0, 1.0, 3.0, -1.0, 2.0]
    # |a-b| = 1,3,0,1,2 -> 7 ; |a| = 1,2,3,0,4 -> 10 ; |b| = 0,1,3,1,2 -> 7
    num, den, r = O.rel_mae(a, b)
    assert (num, den) == (7.0, 10.0) and r == pytest.approx(0.7, abs=1e-15)
    assert O.rel_mae(b, a)[2] == pytest.approx(1.0, abs=1e-15)   # denominator = first arg


def test_rel_mae_closed_forms():
    rng = np.random.default_rng(0)
    a = rng.standard_normal(1000)
    b = rng.standard_normal(1000)
    assert O.rel_mae(a, a)[2] == 0.0
    assert O.rel_mae(a, np.zeros_like(a))[2] == pytest.approx(1.0, abs=1e-14)
    assert O.rel_mae(a, -a)[2] == pytest.approx(2.0, abs=1e-14)
    assert O.rel_mae(a, 1.25 * a)[2] == pytest.approx(0.25, abs=1e-14)
    assert O.rel_mae(a, 0.9 * a)[2] == pytest.approx(0.1, abs=1e-14)
    assert O.rel_mae(3.7 * a, 3.7 * b)[2] == pytest.approx(O.rel_mae(a, b)[2], rel=1e-13)


def test_rel_mae_zero_denominator():
    assert math.isinf(O.rel_mae([0.0, 0.0], [1.0, 0.0])[2])
    assert math.isnan(O.rel_mae([0.0, 0.0], [0.0, 0.0])[2])


# ---------------------------------------------------------------------- DDIM grid
def test_timestep_grids():
    assert list(O.ddim_timesteps(1000, 8)) == [875, 750, 625, 500, 375, 250, 125, 0]
    t50 = O.ddim_timesteps(1000, 50)
    assert t50[0] == 980 and t50[-1] == 0 and np.all(np.diff(t50) == -20)
    assert list(O.ddim_timesteps(1000, 5)) == [800, 600, 400, 200, 0]


def test_alphas_cumprod_endpoints_and_monotone():
    ab = O.ddim_alphas_cumprod()
    assert ab[0] == pytest.approx(0.9999, abs=1e-15)
    assert np.all(np.diff(ab) < 0)
    # independent evaluation through logarithms, and the order of magnitude every
    # linear 1e-4..2e-2 / 1000-step schedule is known for (abar_T ~ 4e-5)
    betas = [1e-4 + k * (2e-2 - 1e-4) / 999 for k in range(1000)]
    assert ab[-1] == pytest.approx(math.exp(math.fsum(math.log1p(-bb) for bb in betas)), rel=1e-12)
    assert 3.9e-5 < ab[-1] < 4.2e-5


def test_last_step_coefficients():
    for S in (5, 8, 50):
        tau, a, b = O.ddim_coefficients(steps=S)
        assert tau[-1] == 0
        assert a[-1] == pytest.approx(1.0 / math.sqrt(0.9999), rel=1e-14)
        assert b[-1] == pytest.approx(-0.01 * a[-1], rel=1e-12)


def test_adjacent_step_matches_ddpm_mean_coefficient():
    """With one sampling step per training step, a_i must equal the 1/sqrt(alpha_t)
    factor of the posterior mean the paper prints, and b_i must agree with that mean's
    eps coefficient -(1-alpha_t)/(sqrt(alpha_t) sqrt(1-abar_t)) to first order in beta."""
    tau, a, b = O.ddim_coefficients(steps=1000)
    ab = O.ddim_alphas_cumprod()
    for i in (0, 1, 250, 640, 998):
        t = tau[i]
        alpha_t = ab[t] / ab[t - 1]
        assert a[i] == pytest.approx(1.0 / math.sqrt(alpha_t), rel=1e-13)
        b_ddpm = -(1.0 - alpha_t) / (math.sqrt(alpha_t) * math.sqrt(1.0 - ab[t]))
        # to first order in beta the deterministic update's eps coefficient is half the
        # posterior mean's (b ~ -beta / (2 sqrt(1-abar)) against -beta / sqrt(1-abar))
        assert 0.5 < b[i] / b_ddpm < (0.51 if t > 100 else 0.6)
        # exact relation: b = sqrt(1-abar_prev) - sqrt(1-abar_t)/sqrt(alpha_t)
        assert b[i] == pytest.approx(math.sqrt(1 - ab[t - 1]) - math.sqrt(1 - ab[t]) / math.sqrt(alpha_t),
                                     rel=1e-10)


def test_two_forms_of_the_update_agree():
    rng = np.random.default_rng(1)
    x, e = rng.standard_normal(64), rng.standard_normal(64)
    ab = O.ddim_alphas_cumprod()
    tau, a, b = O.ddim_coefficients(steps=8)
    for i in range(8):
        ab_t = ab[tau[i]]
        ab_p = ab[tau[i + 1]] if i < 7 else 1.0
        x0_hat = (x - math.sqrt(1 - ab_t) * e) / math.sqrt(ab_t)
        ref = math.sqrt(ab_p) * x0_hat + math.sqrt(1 - ab_p) * e
        np.testing.assert_allclose(O.sampler_step(x, e, a[i], b[i]), ref, rtol=0, atol=1e-12)


@pytest.mark.parametrize("S", [5, 8, 50])
def test_constant_predictor_closed_form(S):
    """If eps never changes, x0_hat never changes, so the run ends at
    (x_T - sqrt(1-abar_tau0) eps) / sqrt(abar_tau0)."""
    rng = np.random.default_rng(2)
    x, e = rng.standard_normal(32), rng.standard_normal(32)
    ab = O.ddim_alphas_cumprod()
    tau, a, b = O.ddim_coefficients(steps=S)
    xx = x.copy()
    for i in range(S):
        xx = O.sampler_step(xx, e, a[i], b[i])
    ref = (x - math.sqrt(1 - ab[tau[0]]) * e) / math.sqrt(ab[tau[0]])
    np.testing.assert_allclose(xx, ref, rtol=0, atol=1e-10)


def test_jump_consistency():
    """r steps with one eps equal a single step across the r-times coarser grid."""
    rng = np.random.default_rng(3)
    x, e = rng.standard_normal(16), rng.standard_normal(16)
    tau50, a50, b50 = O.ddim_coefficients(steps=50)
    tau25, a25, b25 = O.ddim_coefficients(steps=25)     # stride 40 = 2 * 20
    # the 25-step grid is 960, 920, ...; the 50-step grid passes through the same points
    i = list(tau50).index(960)
    two = O.sampler_step(O.sampler_step(x, e, a50[i], b50[i]), e, a50[i + 1], b50[i + 1])
    one = O.sampler_step(x, e, a25[0], b25[0])
    assert tau25[0] == 960 and tau50[i + 2] == tau25[1]
    np.testing.assert_allclose(two, one, rtol=0, atol=1e-12)


def test_point_mass_data_trajectory():
    """For data concentrated at 0 the exact predictor is x / sqrt(1-abar_tau); the
    sample then shrinks as sqrt(1-abar) along the grid and ends at 0."""
    rng = np.random.default_rng(4)
    x = rng.standard_normal(8)
    ab = O.ddim_alphas_cumprod()
    tau, a, b = O.ddim_coefficients(steps=8)
    xx = x.copy()
    for i in range(8):
        e = xx / math.sqrt(1 - ab[tau[i]])
        xx = O.sampler_step(xx, e, a[i], b[i])
        if i < 7:
            ref = x * math.sqrt(1 - ab[tau[i + 1]]) / math.sqrt(1 - ab[tau[0]])
            np.testing.assert_allclose(xx, ref, rtol=0, atol=1e-12)
    np.testing.assert_allclose(xx, 0.0, atol=1e-12)


# ------------------------------------------------------------- other deterministic schedulers
@pytest.mark.parametrize("S", [5, 8, 50])
def test_euler_discrete_is_ddim_in_sigma_space(S):
    """Dividing a DDIM sample by sqrt(abar) gives x0 + sigma*eps, and the DDIM update becomes an Euler step in
    sigma: b_ddim = sqrt(abar_next) * b_euler, a_ddim = sqrt(abar_next / abar_t) (Section 4.2's scheduler
    against the DDIM of the preliminaries).  A plausible slip (sigma of the wrong grid point, sign) breaks it."""
    ab = O.ddim_alphas_cumprod()
    tau, a, b = O.ddim_coefficients(steps=S)
    tau_e, a_e, b_e = O.euler_discrete_coefficients(steps=S)
    np.testing.assert_array_equal(tau, tau_e)
    np.testing.assert_array_equal(a_e, np.ones(S))
    ab_next = np.array([ab[tau[i + 1]] if i + 1 < S else 1.0 for i in range(S)])
    np.testing.assert_allclose(b, np.sqrt(ab_next) * b_e, rtol=1e-12, atol=1e-15)
    assert np.all(b_e < 0)                                    # sigma decreases to 0
    np.testing.assert_allclose(b_e.sum(), -math.sqrt((1 - ab[tau[0]]) / ab[tau[0]]), rtol=1e-12)   # telescopes


def test_euler_discrete_trajectory_equals_scaled_ddim_trajectory():
    """Same predictor, the two parameterisations: x_euler,i = x_ddim,i / sqrt(abar_i) at every step, and
    both end at the same x0."""
    S = 8
    rng = np.random.default_rng(5)
    ab = O.ddim_alphas_cumprod()
    tau, a, b = O.ddim_coefficients(steps=S)
    _, a_e, b_e = O.euler_discrete_coefficients(steps=S)
    f = lambda u, t: np.tanh(u) * (1.0 + 0.001 * t)           # a predictor of the sigma-space sample
    x = rng.standard_normal(16)
    xe = x / math.sqrt(ab[tau[0]])
    for i in range(S):
        x = O.sampler_step(x, f(x / math.sqrt(ab[tau[i]]), tau[i]), a[i], b[i])
        xe = O.sampler_step(xe, f(xe, tau[i]), a_e[i], b_e[i])
        ab_next = ab[tau[i + 1]] if i + 1 < S else 1.0
        np.testing.assert_allclose(xe, x / math.sqrt(ab_next), rtol=0, atol=1e-12)


@pytest.mark.parametrize("S", [4, 10, 50])
def test_flow_euler_closed_forms(S):
    """Constant velocity moves the sample by exactly that velocity over t in [0, 1]; the straight path of
    rectified flow (v = z1 - z0) is integrated exactly; v = z gives (1 + 1/S)^S, Euler's approximation of e."""
    tau, a, b = O.flow_euler_coefficients(steps=S)
    assert tau[0] == 0 and np.all(np.diff(tau) > 0) and tau[-1] == ((S - 1) * 1000) // S
    np.testing.assert_array_equal(a, np.ones(S))
    np.testing.assert_allclose(b.sum(), 1.0, rtol=1e-14)
    rng = np.random.default_rng(6)
    z0, z1 = rng.standard_normal(8), rng.standard_normal(8)
    z = z0.copy()
    g = z0.copy()
    for i in range(S):
        z = O.sampler_step(z, z1 - z0, a[i], b[i])
        g = O.sampler_step(g, g, a[i], b[i])
    np.testing.assert_allclose(z, z1, rtol=0, atol=1e-13)
    np.testing.assert_allclose(g, z0 * (1.0 + 1.0 / S) ** S, rtol=1e-13)
