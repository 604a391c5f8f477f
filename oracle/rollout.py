"""Tree rollout and flat sequential rollout for the oracle (test infrastructure).

Alg. 1 (tree-building loop) with Eq. 2 / App. B.1: from one root latent per
prompt, every depth-i node is advanced by one Euler-Maruyama step of the
reverse SDE; at a split step the parent's drift is shared by K children whose
noises are xi_b = (xi_0 + s eta_b)/sqrt(1+s^2) with xi_0 drawn per parent and
eta_b per child, freshly at every split.  Each edge stores the Gaussian
log-density of the child given the parent (behaviour log-prob, Eq. 3's p_beh
and the denominator of rho_e in Eq. 5).

Global node id = condition * n_nodes + local id; it keys the noise streams.

Pins (tests/test_oracle_rollout.py): K = 1 reproduces the separately written
flat rollout exactly; siblings share one parent latent and differ only through
eta_b; leaf marginals of a linear-Gaussian toy network match the closed form
(App. B.1 theorem); stored log-probs equal the closed-form density of the
stored latents.
"""
import numpy as np

from . import philox, sde


def root_latent(seed, group, D):
    """z_0 ~ N(0, I) for one prompt (Alg. 1 "sample root noise"); prompts in the
    same noise group share it."""
    return philox.normals(seed, group, 0, philox.TAG_ROOT, D)


def tree_rollout(tree, velocity, sched, seed, noise_group, D, n_cond):
    """velocity(z [B, D], t, cond_index [B]) -> v [B, D].
    sched: dict t [T+1] (strictly decreasing), sigma [T], s, logp_mean (bool).
    Returns z [n_cond*n_nodes, D], logp [n_cond*n_nodes] (0 at roots and on
    deterministic sigma = 0 edges), v [n_cond*n_nodes, D] (velocity evaluated at
    every non-leaf node, zeros at leaves)."""
    T, K, nn = tree["T"], tree["K"], tree["n_nodes"]
    off, width, splits = tree["off"], tree["width"], tree["splits"]
    t, sigma, s = sched["t"], sched["sigma"], sched["s"]
    z = np.zeros((n_cond * nn, D))
    vv = np.zeros((n_cond * nn, D))
    logp = np.zeros(n_cond * nn)
    for c in range(n_cond):
        z[c * nn] = root_latent(seed, noise_group[c], D)
    for i in range(T):
        # frontier of depth i over all prompts, one batched network call
        ids = np.array([c * nn + off[i] + j for c in range(n_cond) for j in range(width[i])])
        cidx = np.array([c for c in range(n_cond) for _ in range(width[i])])
        v = velocity(z[ids], float(t[i]), cidx)
        vv[ids] = v
        h, std = sde.step_coefficients(t[i], t[i + 1], sigma[i])
        is_split = i in splits
        for row, p in enumerate(ids):
            c, j = cidx[row], p - cidx[row] * nn - off[i]
            mu = sde.drift_mean(z[p], v[row], t[i], t[i + 1], sigma[i])
            kids = [j * K + b for b in range(K)] if is_split else [j]
            xi0 = philox.normals(seed, p, i, philox.TAG_XI0, D) if is_split else None
            for jc in kids:
                ch = c * nn + off[i + 1] + jc
                if std == 0.0:
                    z[ch] = mu
                    continue
                eta = philox.normals(seed, ch, i, philox.TAG_ETA, D)
                xi = sde.branch_noise(xi0, eta, s) if is_split else eta
                z[ch] = mu + std * xi
                logp[ch] = sde.transition_logp(z[ch], mu, std, sched["logp_mean"])
    return z, logp, vv


def flat_rollout(n_traj, T, velocity, sched, seed, noise_group, D):
    """Sequential GRPO rollout: n_traj independent trajectories of T steps.
    Trajectory c is numbered like a K = 1 tree of its own: node (c, d) has id
    c*(T+1) + d.  Returns z [n_traj*(T+1), D], logp [n_traj*(T+1)]."""
    t, sigma = sched["t"], sched["sigma"]
    z = np.zeros((n_traj * (T + 1), D))
    logp = np.zeros(n_traj * (T + 1))
    for c in range(n_traj):
        cur = root_latent(seed, noise_group[c], D)
        z[c * (T + 1)] = cur
        for i in range(T):
            v = velocity(cur[None], float(t[i]), np.array([c]))[0]
            mu = sde.drift_mean(cur, v, t[i], t[i + 1], sigma[i])
            _, std = sde.step_coefficients(t[i], t[i + 1], sigma[i])
            node = c * (T + 1) + i + 1
            if std == 0.0:
                cur = mu
            else:
                cur = mu + std * philox.normals(seed, node, i, philox.TAG_ETA, D)
                logp[node] = sde.transition_logp(cur, mu, std, sched["logp_mean"])
            z[node] = cur
    return z, logp


def edge_logprob(tree, velocity, sched, z, edge_ids, n_cond):
    """Log-density of stored child latents under another policy (numerator of
    rho_e, Eq. 5): for edge e = (parent -> child = edge_ids[e]) at step
    i = depth(child) - 1, evaluate the policy's velocity at the stored parent and
    return log N(z_child; mu_i(z_parent, v'), std_i^2 I)."""
    nn = tree["n_nodes"]
    t, sigma = sched["t"], sched["sigma"]
    out = np.zeros(len(edge_ids))
    for e, g in enumerate(edge_ids):
        c, n = divmod(int(g), nn)
        p = c * nn + int(tree["parent"][n])
        i = int(tree["depth"][n]) - 1
        v = velocity(z[p][None], float(t[i]), np.array([c]))[0]
        mu = sde.drift_mean(z[p], v, t[i], t[i + 1], sigma[i])
        _, std = sde.step_coefficients(t[i], t[i + 1], sigma[i])
        out[e] = sde.transition_logp(z[g], mu, std, sched["logp_mean"]) if std > 0 else 0.0
    return out
