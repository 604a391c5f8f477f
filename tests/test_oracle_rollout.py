"""Pins for the oracle's tree rollout (Alg. 1 tree-building loop, Eq. 2, App. B.1)
and the synthetic rewards."""
import numpy as np

from oracle import dit, philox, rewards, rollout, sde, tree
from paper_2509_06040_amd import synth


def _tiny_velocity(cfg, W, cond):
    return lambda z, t, cidx: dit.forward(cfg, W, z, t, cond, cidx)


def test_branching_factor_one_is_the_flat_rollout():
    wl = synth.WORKLOADS["tiny"]
    cfg = wl["model"]
    D = synth.model_sizes(cfg)["D"]
    W = synth.make_weights(cfg, 0)
    N, T = 3, 4
    cond = synth.cond_tokens(cfg, N).astype(np.float64)
    sched = synth.schedule(T, 1.0, logp_mean=False)
    vel = _tiny_velocity(cfg, W, cond)
    t = tree.tree_build(T, (1, 2), 1)                      # K = 1 ignores the splits
    groups = [0, 0, 5]
    zt, lpt, _ = rollout.tree_rollout(t, vel, sched, 77, groups, D, N)
    zf, lpf = rollout.flat_rollout(N, T, vel, sched, 77, groups, D)
    assert np.array_equal(zt, zf) and np.array_equal(lpt, lpf)
    # "init same noise": equal groups share z_0, other groups do not
    assert np.array_equal(zt[0], zt[T + 1]) and not np.array_equal(zt[0], zt[2 * (T + 1)])
    assert not np.array_equal(zt[1], zt[T + 2])            # but their paths differ afterwards


def test_siblings_share_the_parent_and_differ_only_by_eta():
    wl = synth.WORKLOADS["tiny"]
    cfg = wl["model"]
    D = synth.model_sizes(cfg)["D"]
    W = synth.make_weights(cfg, 0)
    cond = synth.cond_tokens(cfg, 1).astype(np.float64)
    sched = synth.schedule(wl["T"], wl["kappa"], logp_mean=False)
    t = tree.tree_build(wl["T"], wl["splits"], wl["K"])
    z, lp, v = rollout.tree_rollout(t, _tiny_velocity(cfg, W, cond), sched, 5, [0], D, 1)
    s = sched["s"]
    for n in range(1, t["n_nodes"]):
        p, i = t["parent"][n], t["depth"][n] - 1
        mu = sde.drift_mean(z[p], v[p], sched["t"][i], sched["t"][i + 1], sched["sigma"][i])
        _, std = sde.step_coefficients(sched["t"][i], sched["t"][i + 1], sched["sigma"][i])
        xi = (z[n] - mu) / std
        eta = philox.normals(5, n, i, philox.TAG_ETA, D)
        if i in t["splits"]:
            xi0 = philox.normals(5, p, i, philox.TAG_XI0, D)
            assert np.allclose(xi, (xi0 + s * eta) / np.sqrt(1 + s * s), atol=1e-9)
        else:
            assert np.allclose(xi, eta, atol=1e-9)
        # stored log-prob is the closed-form Gaussian density of the stored latent
        ref = -0.5 * np.sum(xi ** 2) - D * np.log(std) - 0.5 * D * np.log(2 * np.pi)
        assert np.isclose(lp[n], ref, rtol=1e-9)
    # siblings: same mean, noise correlation 1/(1+s^2)
    a, b = t["off"][3], t["off"][3] + 1                     # children of the split at step 2
    assert t["parent"][a] == t["parent"][b]
    assert lp[0] == 0.0
    # re-evaluating the behaviour policy on its own tree returns the stored log-probs
    ids = np.arange(1, t["n_nodes"])
    again = rollout.edge_logprob(t, _tiny_velocity(cfg, W, cond), sched, z, ids, 1)
    assert np.allclose(again, lp[1:], rtol=1e-9)


def test_leaf_law_of_a_linear_gaussian_toy_matches_closed_form():
    """App. B.1 theorem: branching leaves every leaf with the law of a plain SDE
    rollout.  With v = a z every element is Gaussian: var_{i+1} = c_i^2 var_i +
    std_i^2, and two leaves that separated at split step i0 have covariance
    c^2 var + std^2/(1+s^2) right after it, multiplied by c_j^2 afterwards."""
    D, T, a, s = 1 << 16, 6, -0.8, 2.0
    splits = (1, 3)
    t = tree.tree_build(T, splits, 2)
    sched = dict(t=synth.time_grid(T, 1.0) * 0.9 + 0.05, sigma=np.full(T, 0.7, np.float32), s=s, logp_mean=False)
    z, _, _ = rollout.tree_rollout(t, lambda zz, tt, ci: a * zz, sched, 9, [0], D, 1)
    c = [sde.drift_mean(1.0, a, sched["t"][i], sched["t"][i + 1], sched["sigma"][i]) for i in range(T)]
    sd2 = [sde.step_coefficients(sched["t"][i], sched["t"][i + 1], sched["sigma"][i])[1] ** 2 for i in range(T)]
    var = [1.0]
    for i in range(T):
        var.append(c[i] ** 2 * var[i] + sd2[i])
    leaves = z[t["off"][T]:]
    tol = 6 / np.sqrt(D)
    for l in range(4):
        assert abs(leaves[l].var() / var[T] - 1) < tol * np.sqrt(2)

    def cov_after(i0):
        cv = c[i0] ** 2 * var[i0] + sd2[i0] / (1 + s * s)
        for j in range(i0 + 1, T):
            cv *= c[j] ** 2
        return cv
    assert abs(np.mean(leaves[0] * leaves[1]) - cov_after(3)) < tol * var[T]    # split at step 3
    assert abs(np.mean(leaves[0] * leaves[2]) - cov_after(1)) < tol * var[T]    # split at step 1


def test_ode_steps_are_deterministic_and_carry_no_logprob():
    D, T = 64, 3
    t = tree.tree_build(T, (1,), 2)
    sched = dict(t=synth.time_grid(T, 1.0), sigma=np.array([0.0, 0.3, 0.0], np.float32), s=4.0, logp_mean=False)
    z, lp, _ = rollout.tree_rollout(t, lambda zz, tt, ci: 0.5 * zz, sched, 1, [0], D, 1)
    h = sched["t"][0] - sched["t"][1]
    assert np.allclose(z[1], z[0] - h * 0.5 * z[0]) and lp[1] == 0.0 and lp[2] != 0.0


def test_rewards_by_hand():
    z = np.array([[1.0, 2.0, 3.0, 4.0], [0.0, 0.0, 0.0, 0.0]])
    w = np.array([1.0, -1.0, 0.5, 0.25])
    assert np.allclose(rewards.reward_linear(z, w), [(1 - 2 + 1.5 + 1) / 2, 0.0])
    assert np.allclose(rewards.reward_linear(z, w, True), np.tanh([0.75, 0.0]))
    # video: C = 1, F = 2, 1x2 pixels: frame means m = (1.5, 3.5); w = (2, 1):
    # lin = (2*1.5 + 1*3.5)/sqrt(2); penalty = (3.5-1.5)^2 / 1 = 4
    zv = np.array([[1.0, 2.0, 3.0, 4.0]])
    r = rewards.reward_video(zv, np.array([[2.0], [1.0]]), 1, 2, 1, 2, lam=0.5)
    assert np.isclose(r[0], 6.5 / np.sqrt(2) - 0.5 * 4.0)
    # C = 2, F = 1: no temporal term
    r = rewards.reward_video(zv, np.array([[1.0, 1.0]]), 2, 1, 1, 2)
    assert np.isclose(r[0], (1.5 + 3.5) / np.sqrt(2))
