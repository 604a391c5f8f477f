"""Reward fusion (Eq. 3) and depth-wise normalisation (Eq. 4) for the oracle
(test infrastructure).

Eq. 3, written out as the plain definition: for every node n with descendant
leaves L(n),  rbar(n) = sum_l w_l r_l,  w = softmax_l(beta * s_l),
s_l = log p_beh(l | n) = the sum of the behaviour log-probs of the edges on the
path n -> l (0 when n is the leaf itself).  beta = 0 is the uniform mean,
beta = 1 weights by the behaviour path probability.

Eq. 4: per tree and per depth d, A_d(n) = (rbar(n) - mu_d) / (sigma_d + eps)
over all nodes of that depth; an edge takes the advantage of its child; the
result is optionally clipped to [-A_max, A_max] (Table 2: 5.0).
Readings where the paper is silent: population standard deviation (ddof = 0)
unless asked otherwise, eps = 1e-8, one tree per prompt.

Pins (tests/test_oracle_fusion.py): hand-worked 2- and 3-level trees, beta = 0
equals the arithmetic mean of descendant leaves, invariance to a per-depth
shift of the log-probs, chains carry rbar unchanged, zero mean / unit std per
depth, sibling advantages sum to zero (App. B.3).
"""
import numpy as np


def path_logp(tree, logp_tree, n, leaf_node):
    """Sum of edge log-probs on the path from node n down to leaf_node."""
    s, m = 0.0, int(leaf_node)
    while m != n:
        s += float(logp_tree[m])
        m = int(tree["parent"][m])
        assert m >= 0
    return s


def fuse_rewards(tree, leaf_rewards, logp_edges, beta, n_cond):
    """rbar [n_cond*n_nodes].  leaf_rewards [n_cond*w]; logp_edges [n_cond*n_nodes]
    indexed by child node."""
    nn, w, T = tree["n_nodes"], tree["n_leaves"], tree["T"]
    leaf0 = int(tree["off"][T])
    r = np.asarray(leaf_rewards, np.float64).reshape(n_cond, w)
    lp = np.asarray(logp_edges, np.float64).reshape(n_cond, nn)
    rbar = np.zeros((n_cond, nn))
    for c in range(n_cond):
        for n in range(nn):
            leaves = range(int(tree["leaf_lo"][n]), int(tree["leaf_hi"][n]))
            s = np.array([beta * path_logp(tree, lp[c], n, leaf0 + l) for l in leaves])
            e = np.exp(s - s.max())
            wgt = e / e.sum()
            rbar[c, n] = float(np.sum(wgt * r[c, list(leaves)]))
    return rbar.reshape(-1)


def depth_advantages(tree, rbar, n_cond, eps=1e-8, ddof=0, a_max=5.0):
    """A [n_cond*n_nodes] (Eq. 4); a_max <= 0 disables the clip.  A depth with
    fewer than ddof+1 nodes gets zero advantage."""
    nn, T = tree["n_nodes"], tree["T"]
    rb = np.asarray(rbar, np.float64).reshape(n_cond, nn)
    adv = np.zeros((n_cond, nn))
    for c in range(n_cond):
        for d in range(T + 1):
            lo, hi = int(tree["off"][d]), int(tree["off"][d + 1])
            x = rb[c, lo:hi]
            if x.size - ddof <= 0:
                continue
            mu = x.mean()
            sd = np.sqrt(np.sum((x - mu) ** 2) / (x.size - ddof))
            a = (x - mu) / (sd + eps) if sd + eps > 0 else np.zeros_like(x)   # no spread: A = 0
            if a_max > 0:
                a = np.clip(a, -a_max, a_max)
            adv[c, lo:hi] = a
    return adv.reshape(-1)


def ess(tree, logp_edges, beta, n_tree):
    """Effective sample size of the fusion weights of every node (appendix, self-normalised
    importance sampling view of Eq. 3): with w_l the Eq. 3 weights of the leaves under node n,
    ESS(n) = (sum_l w_l)^2 / sum_l w_l^2.  -> float64 [n_tree*n_nodes]."""
    n_nodes, T = tree["n_nodes"], tree["T"]
    parent, leaf_lo, leaf_hi = tree["parent"], tree["leaf_lo"], tree["leaf_hi"]
    leaf0 = tree["off"][T]
    lp = np.asarray(logp_edges, np.float64).reshape(n_tree, n_nodes)
    out = np.zeros((n_tree, n_nodes))
    for c in range(n_tree):
        for n in range(n_nodes):
            s = []
            for l in range(leaf_lo[n], leaf_hi[n]):
                acc, m = 0.0, leaf0 + l
                while m != n:                 # log-probs of the edges on the path n -> leaf
                    acc += lp[c, m]
                    m = parent[m]
                s.append(beta * acc)
            s = np.array(s)
            w = np.exp(s - s.max())
            out[c, n] = w.sum() ** 2 / (w * w).sum()
    return out.reshape(-1)
