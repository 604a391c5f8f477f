"""Pins for the oracle's reverse-SDE step (Eq. 1, App. B.1) and transition density."""
import numpy as np
from scipy import stats

from oracle import sde


def test_hand_worked_scalar_step():
    # t_i = 0.5, t_{i+1} = 0.4, sigma = 0.3, z = 1, v = 2:
    # mu = 1 - 0.1*2 - 0.1*0.09/(2*0.5) * (1 + 0.5*2) = 0.8 - 0.009*2 = 0.782
    assert np.isclose(sde.drift_mean(1.0, 2.0, 0.5, 0.4, 0.3), 0.782, rtol=0, atol=1e-15)
    h, std = sde.step_coefficients(0.5, 0.4, 0.3)
    assert np.isclose(h, 0.1) and np.isclose(std, 0.3 * np.sqrt(0.1))
    assert np.isclose(std, 0.0948683298, atol=1e-9)


def test_sigma_zero_is_the_euler_step_of_the_flow_ode():
    rng = np.random.default_rng(0)
    z, v = rng.standard_normal(16), rng.standard_normal(16)
    assert np.allclose(sde.drift_mean(z, v, 0.7, 0.55, 0.0), z - 0.15 * v, rtol=0, atol=1e-15)


def _gaussian_flow(a2, t):
    """For data x ~ N(0, a2), z_t = (1-t) x + t e has variance m_t and the exact
    velocity field E[e - x | z_t] = k_t z_t (joint Gaussian regression)."""
    m = (1 - t) ** 2 * a2 + t ** 2
    k = (t - (1 - t) * a2) / m
    return m, k


def test_step_preserves_the_exact_marginals_to_second_order():
    """Eq. 1 has the marginals p_t of the forward process for every noise level.
    With a Gaussian data law everything is closed-form: one Euler-Maruyama step
    from z_i ~ N(0, m(t_i)) has variance c^2 m(t_i) + sigma^2 h, which must equal
    m(t_i - h) up to O(h^2) -- a wrong sign or a dropped term leaves an O(h) error."""
    a2 = 0.36
    for sigma in (0.0, 0.3, 0.9):
        for t in (0.9, 0.5, 0.2):
            errs = []
            for h in (0.02, 0.01, 0.005):
                m, k = _gaussian_flow(a2, t)
                c = sde.drift_mean(1.0, k, t, t - h, sigma)      # mu is linear in z: mu = c z
                var_next = c * c * m + sigma ** 2 * h
                errs.append(abs(var_next - _gaussian_flow(a2, t - h)[0]))
            assert errs[0] < 5e-3
            assert 3.0 < errs[0] / errs[1] < 5.0 and 3.0 < errs[1] / errs[2] < 5.0   # second order


def test_many_small_steps_converge_to_the_data_variance():
    a2, sigma, N = 0.36, 0.5, 4000
    ts = np.linspace(1.0, 0.02, N + 1)
    var = 1.0                                                     # z_{t=1} = e ~ N(0, 1)
    for i in range(N):
        _, k = _gaussian_flow(a2, ts[i])
        c = sde.drift_mean(1.0, k, ts[i], ts[i + 1], sigma)
        var = c * c * var + sigma ** 2 * (ts[i] - ts[i + 1])
    assert abs(var - _gaussian_flow(a2, 0.02)[0]) < 2e-3


def test_logp_hand_value_and_library_density():
    # D = 2, mu = 0, std = 0.5, z = (0.5, -0.5): -1 + 2 ln 2 - ln 2pi
    lp = sde.transition_logp(np.array([0.5, -0.5]), np.zeros(2), 0.5)
    assert np.isclose(lp, -1.0 + 2 * np.log(2.0) - np.log(2 * np.pi), atol=1e-14)
    assert np.isclose(lp, -1.4515827, atol=1e-7)
    assert np.isclose(sde.transition_logp(np.array([0.5, -0.5]), np.zeros(2), 0.5, True), lp / 2)
    rng = np.random.default_rng(1)
    z, mu = rng.standard_normal(7), rng.standard_normal(7)
    ref = stats.multivariate_normal(mean=mu, cov=0.3 ** 2 * np.eye(7)).logpdf(z)
    assert np.isclose(sde.transition_logp(z, mu, 0.3), ref, rtol=1e-12)


def test_expected_logp_under_the_behaviour_policy():
    D, std = 1 << 16, 0.07
    xi = np.random.default_rng(2).standard_normal(D)
    lp = sde.transition_logp(std * xi, np.zeros(D), std)
    expect = -D / 2 - D * np.log(std) - D / 2 * np.log(2 * np.pi)
    assert abs(lp - expect) < 5 * np.sqrt(D / 2)
