"""Reverse-SDE step and transition log-density for the oracle (test infrastructure).

Eq. 1: dz = (f_t z - (1+eps_t^2)/2 g_t^2 grad log p_t(z)) dt + eps_t g_t dw.
App. B.1: Euler-Maruyama on a reverse grid t_0 > t_1 > ... > t_N with
h_i = t_i - t_{i+1}:  z_{i+1} = mu_theta(z_i, t_i) + g_i * noise.

The paper never writes mu_theta out.  Reading used: the rectified-flow path
z_t = (1-t) x + t e, whose velocity field is v = e - x.  Then
f_t = -1/(1-t), g_t^2 = 2t/(1-t), E[e | z_t] = z_t + (1-t) v and the score is
-(z_t + (1-t) v)/t, which turns the drift of Eq. 1 into
v + sigma^2/(2t) (z + (1-t) v) with sigma = eps_t g_t the diffusion coefficient.
One backward Euler-Maruyama step of size h_i therefore has

    mu_i(z, v) = z - h_i v - h_i sigma_i^2 / (2 t_i) (z + (1 - t_i) v)
    std_i      = sigma_i sqrt(h_i)

Pins (tests/test_oracle_sde.py): sigma = 0 reduces to the textbook Euler step
of dz/dt = v; a hand-worked scalar value; for a Gaussian data law the exact
reverse-SDE marginals are known in closed form and the step reproduces them to
first order in h; the log-density equals scipy's multivariate normal.
PARITY UNPINNED against the authors' own mu_theta (not printed in the paper).
"""
import numpy as np


def step_coefficients(t_i, t_next, sigma_i):
    """(h_i, std_i) of step i."""
    h = float(t_i) - float(t_next)
    return h, float(sigma_i) * np.sqrt(h)


def drift_mean(z, v, t_i, t_next, sigma_i):
    """mu_i(z, v): mean of the Gaussian transition of step i (see header)."""
    h = float(t_i) - float(t_next)
    ti = float(t_i)
    sig2 = float(sigma_i) ** 2
    return z - h * v - h * sig2 / (2.0 * ti) * (z + (1.0 - ti) * v)


def branch_noise(xi0, eta, s):
    """Eq. 2: xi_b = (xi_0 + s eta_b) / sqrt(1 + s^2)."""
    return (xi0 + float(s) * eta) / np.sqrt(1.0 + float(s) ** 2)


def transition_logp(z_child, mu, std, reduce_mean=False):
    """log N(z_child; mu, std^2 I): the density whose ratio is rho_e in Eq. 5.
    reduce_mean divides by the number of latent elements."""
    d = (np.asarray(z_child, np.float64) - np.asarray(mu, np.float64)).ravel()
    D = d.size
    lp = -np.sum(d * d) / (2.0 * std * std) - D * np.log(std) - 0.5 * D * np.log(2.0 * np.pi)
    return lp / D if reduce_mean else lp
