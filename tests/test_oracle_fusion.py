"""Pins for reward fusion (Eq. 3), depth-wise advantages (Eq. 4) and the clipped
objective (Eq. 5) of the oracle."""
import json
import os

import numpy as np
import pytest

from oracle import fusion, objective, tree

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "fusion_hand_trees.json")))


@pytest.mark.parametrize("name", ["tree_A", "tree_B"])
def test_hand_worked_trees(name):
    g = GOLD[name]
    t = tree.tree_build(g["T"], g["splits"], g["K"])
    for beta, key in ((1.0, "rbar_beta1"), (0.0, "rbar_beta0")):
        rb = fusion.fuse_rewards(t, g["leaf_rewards"], g["logp_edges"], beta, 1)
        assert np.allclose(rb, g[key], atol=1e-12)
    rb = fusion.fuse_rewards(t, g["leaf_rewards"], g["logp_edges"], 1.0, 1)
    if name == "tree_A":
        assert np.allclose(fusion.depth_advantages(t, rb, 1, eps=0.0), g["adv_beta1_ddof0"], atol=1e-12)
    else:
        a0 = fusion.depth_advantages(t, rb, 1, eps=0.0, ddof=0)
        a1 = fusion.depth_advantages(t, rb, 1, eps=0.0, ddof=1)
        assert np.allclose(a0[3:], g["adv_leaf_ddof0"], atol=1e-12)
        assert np.allclose(a1[3:], g["adv_leaf_ddof1"], atol=1e-12)
        assert np.allclose(a0[1:3], g["adv_depth1_beta1_ddof0"], atol=1e-12)
        assert a0[0] == 0.0 and a1[0] == 0.0


def test_tree_c_chain_between_splits_carries_rbar():
    # T = 3, splits {0, 2}: the middle step does not branch, so rbar at depth 2
    # equals rbar at depth 1 node for node whatever the middle log-probs are
    t = tree.tree_build(3, (0, 2), 2)
    rng = np.random.default_rng(0)
    lp = rng.standard_normal(t["n_nodes"]) * 3
    r = rng.standard_normal(4)
    rb = fusion.fuse_rewards(t, r, lp, 1.0, 1)
    assert np.allclose(rb[1:3], rb[3:5], atol=1e-14)


def _random_case(seed, T=6, splits=(0, 2, 3), K=3, n_cond=2):
    t = tree.tree_build(T, splits, K)
    rng = np.random.default_rng(seed)
    return t, rng.standard_normal(n_cond * t["n_leaves"]), rng.standard_normal(n_cond * t["n_nodes"]) * 2, n_cond


def test_beta_zero_is_the_mean_of_descendant_leaves():
    t, r, lp, C = _random_case(1)
    rb = fusion.fuse_rewards(t, r, lp, 0.0, C).reshape(C, -1)
    for c in range(C):
        rc = r.reshape(C, -1)[c]
        for n in range(t["n_nodes"]):
            assert np.isclose(rb[c, n], rc[t["leaf_lo"][n]:t["leaf_hi"][n]].mean(), atol=1e-14)


def test_beta_one_weights_are_path_probabilities():
    # weights proportional to prod of edge probabilities: check against explicit products
    t, r, lp, C = _random_case(2, n_cond=1)
    rb = fusion.fuse_rewards(t, r, lp, 1.0, 1)
    T = t["T"]
    for n in range(t["n_nodes"]):
        num = den = 0.0
        for l in range(t["leaf_lo"][n], t["leaf_hi"][n]):
            p, m = 1.0, t["off"][T] + l
            while m != n:
                p *= np.exp(lp[m])
                m = t["parent"][m]
            num, den = num + p * r[l], den + p
        assert np.isclose(rb[n], num / den, rtol=1e-10)


def test_shift_of_one_depths_logprobs_changes_nothing():
    t, r, lp, C = _random_case(3)
    rb = fusion.fuse_rewards(t, r, lp, 0.7, C)
    lp2 = lp.reshape(C, -1).copy()
    lo, hi = t["off"][3], t["off"][4]
    lp2[:, lo:hi] += 123.0
    assert np.allclose(fusion.fuse_rewards(t, r, lp2.ravel(), 0.7, C), rb, atol=1e-10)


def test_fusion_matches_bottom_up_recursion():
    # equivalent formulation: logZ(leaf) = 0, logZ(n) = LSE_c(beta lp(c) + logZ(c)),
    # rbar(n) = sum_c softmax_c(...) rbar(c)
    t, r, lp, C = _random_case(4, n_cond=1)
    beta = 1.0
    nn, T = t["n_nodes"], t["T"]
    logZ, rb = np.zeros(nn), np.zeros(nn)
    rb[t["off"][T]:] = r
    for n in range(t["off"][T] - 1, -1, -1):
        kids = tree.children(t, n)
        a = np.array([beta * lp[k] + logZ[k] for k in kids])
        logZ[n] = np.log(np.sum(np.exp(a - a.max()))) + a.max()
        rb[n] = np.sum(np.exp(a - logZ[n]) * rb[kids])
    assert np.allclose(fusion.fuse_rewards(t, r, lp, beta, 1), rb, rtol=1e-11)


def test_depth_normalisation_invariants():
    t, r, lp, C = _random_case(5)
    rb = fusion.fuse_rewards(t, r, lp, 1.0, C)
    adv = fusion.depth_advantages(t, rb, C, eps=0.0, a_max=0.0).reshape(C, -1)
    for c in range(C):
        for d in range(t["T"] + 1):
            a = adv[c, t["off"][d]:t["off"][d + 1]]
            if a.size == 1:
                assert a[0] == 0.0
            else:
                assert abs(a.mean()) < 1e-12 and abs(a.std() - 1.0) < 1e-12
    # App. B.3: for a depth made of one sibling group the advantages sum to zero
    t2 = tree.tree_build(2, (0,), 2)
    rb2 = fusion.fuse_rewards(t2, [0.3, 1.9], np.zeros(t2["n_nodes"]), 0.0, 1)
    a2 = fusion.depth_advantages(t2, rb2, 1)
    assert abs(a2[1] + a2[2]) < 1e-12 and a2[1] < 0 < a2[2]


def test_equal_rewards_give_zero_not_nan_and_clip_applies():
    t = tree.tree_build(2, (0, 1), 2)
    rb = fusion.fuse_rewards(t, [2.0] * 4, np.zeros(7), 1.0, 1)
    assert np.array_equal(fusion.depth_advantages(t, rb, 1), np.zeros(7))
    # 32 leaves, one outlier: z-score of the outlier is sqrt(31) = 5.57 -> clipped to 5
    t = tree.tree_build(5, (0, 1, 2, 3, 4), 2)
    r = np.zeros(32)
    r[7] = 1.0
    rb = fusion.fuse_rewards(t, r, np.zeros(t["n_nodes"]), 0.0, 1)
    adv = fusion.depth_advantages(t, rb, 1, eps=0.0, a_max=5.0)
    assert adv[t["off"][5] + 7] == 5.0
    raw = fusion.depth_advantages(t, rb, 1, eps=0.0, a_max=0.0)
    assert np.isclose(raw[t["off"][5] + 7], np.sqrt(31.0))


def test_grpo_objective_hand_values():
    # rho = 1: J is the mean advantage
    J, _ = objective.grpo_objective([0.1, -2.0], [0.1, -2.0], [1.0, -3.0], 0.2)
    assert np.isclose(J, -1.0)
    # rho = e^{0.5} = 1.6487 with A > 0 is clipped to 1.2 A; with A < 0 the min keeps rho A
    J, clipped = objective.grpo_objective([0.5, 0.5], [0.0, 0.0], [2.0, -2.0], 0.2)
    assert np.isclose(J, (1.2 * 2.0 + np.exp(0.5) * -2.0) / 2)
    assert list(clipped) == [True, False]
    # rho = e^{-0.5} = 0.6065: A > 0 keeps rho A, A < 0 clips to 0.8 A
    J, clipped = objective.grpo_objective([-0.5, -0.5], [0.0, 0.0], [2.0, -2.0], 0.2)
    assert np.isclose(J, (np.exp(-0.5) * 2.0 + 0.8 * -2.0) / 2)
    assert list(clipped) == [False, True]


def test_ess_of_fusion_weights():
    # appendix (self-normalised importance sampling): ESS = (sum w)^2 / sum w^2
    t = tree.tree_build(4, (0, 2), 2)                      # 4 leaves, widths 1,2,2,4,4
    n, off = t["n_nodes"], t["off"]
    # uniform weights: ESS = number of leaves under the node
    e = fusion.ess(t, np.zeros(n), 1.0, 1)
    assert np.allclose(e, np.array(t["leaf_hi"]) - np.array(t["leaf_lo"]))
    # two leaves under a depth-2 node with weights 3:1 -> 1 / (0.75^2 + 0.25^2) = 1.6
    lp = np.zeros(n)
    lp[off[3] + 0] = np.log(3.0)                           # edge into the first depth-3 node (split at step 2)
    e = fusion.ess(t, lp, 1.0, 1)
    assert np.isclose(e[off[2] + 0], 1.6) and np.isclose(e[off[2] + 1], 2.0)
    assert np.isclose(e[off[3] + 0], 1.0) and np.isclose(e[off[4] + 2], 1.0)
    # root: weights 3,1,1,1 -> 36 / 12 = 3; with beta = 0 the weights are uniform again
    assert np.isclose(e[0], 3.0)
    assert np.isclose(fusion.ess(t, lp, 0.0, 1)[0], 4.0)
    # one dominating leaf -> ESS -> 1; shifting all log-probs of a depth changes nothing
    lp2 = np.zeros(n)
    lp2[off[4] + 1] = 50.0
    assert np.isclose(fusion.ess(t, lp2, 1.0, 1)[0], 1.0)
    lp3 = lp.copy()
    lp3[off[1]:off[2]] += 7.5
    assert np.allclose(fusion.ess(t, lp3, 1.0, 1), e)
    # consistency with the fused reward: with rewards = leaf weights' indicator the weights are recovered
    rng = np.random.default_rng(5)
    lp4 = rng.standard_normal(n)
    w = np.array([fusion.fuse_rewards(t, np.eye(4)[l], lp4, 1.3, 1)[0] for l in range(4)])   # root weights of each leaf
    assert np.isclose(fusion.ess(t, lp4, 1.3, 1)[0], w.sum() ** 2 / (w * w).sum())
