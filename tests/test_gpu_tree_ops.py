"""GPU parity: leaf rewards, reward fusion (Eq. 3), depth-wise advantages (Eq. 4),
pruning (Sec. 3.4, bit-exact) and the clipped objective (Eq. 5) against the oracle."""
import json
import os

import numpy as np
import pytest
import torch

from oracle import fusion, objective, prune, rewards, tree
from paper_2509_06040_amd import binding as br
from gpu_util import DEV, bytes_buffer, dev, host

pytestmark = pytest.mark.gpu
GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "fusion_hand_trees.json")))


def _fuse(t, r, lp, beta, eps=1e-8, ddof=0, a_max=5.0):
    n = t.n_tree * t.n_nodes
    rbar, adv = torch.empty(n, device=DEV), torch.empty(n, device=DEV)
    br.fuse_advantage(t, dev(np.asarray(r, np.float32)), dev(np.asarray(lp, np.float32)), beta, eps, ddof, a_max, rbar, adv)
    return host(rbar), host(adv)


@pytest.mark.parametrize("name", ["tree_A", "tree_B"])
def test_fusion_hand_worked_trees(lib, name):
    g = GOLD[name]
    t = br.Tree(g["T"], g["splits"], g["K"])
    rb1, adv = _fuse(t, g["leaf_rewards"], g["logp_edges"], 1.0, eps=0.0)
    rb0, _ = _fuse(t, g["leaf_rewards"], g["logp_edges"], 0.0)
    assert np.abs(rb1 - g["rbar_beta1"]).max() < 1e-6 and np.abs(rb0 - g["rbar_beta0"]).max() < 1e-6
    if name == "tree_A":
        assert np.abs(adv - g["adv_beta1_ddof0"]).max() < 1e-5
    else:
        assert np.abs(adv[3:] - g["adv_leaf_ddof0"]).max() < 1e-5
        assert np.abs(adv[1:3] - g["adv_depth1_beta1_ddof0"]).max() < 1e-5
        _, adv1 = _fuse(t, g["leaf_rewards"], g["logp_edges"], 1.0, eps=0.0, ddof=1)
        assert np.abs(adv1[3:] - g["adv_leaf_ddof1"]).max() < 1e-5 and adv1[0] == 0.0


@pytest.mark.parametrize("T,splits,K,C,lp_scale", [(8, (2, 4, 6), 2, 1, 1.0), (20, (4, 8, 12, 16), 2, 4, 0.05),
                                                   (20, (0, 3, 6, 9), 3, 2, 2.0), (16, (3, 6, 9, 12), 4, 2, 300.0),
                                                   (10, (0, 1, 2, 3, 4, 5, 6), 2, 2, 1.0), (6, (), 2, 3, 1.0),
                                                   (5, (1, 3), 1, 5, 1.0),
                                                   (16, (3, 6, 9, 12), 2, 2, 0.05),            # the large-image workload's trees
                                                   (16, (4, 8, 12), 2, 1, 0.05),               # the video workload's tree
                                                   (100, (0, 1, 2, 3, 4, 5), 2, 1, 0.3)])      # 6143 nodes: not LDS-cached
def test_fusion_and_advantages_match_oracle(lib, T, splits, K, C, lp_scale):
    t = br.Tree(T, splits, K, n_tree=C)
    o = tree.tree_build(T, splits, K)
    rng = np.random.default_rng(T * 7 + K)
    r = np.tanh(rng.standard_normal(C * t.n_leaves)).astype(np.float32)
    lp = (rng.standard_normal(C * t.n_nodes) * lp_scale - 3 * lp_scale).astype(np.float32)
    for beta, ddof, a_max in ((1.0, 0, 5.0), (0.0, 0, 5.0), (0.5, 1, 0.0), (1.0, 0, 1.0)):
        rb, adv = _fuse(t, r, lp, beta, ddof=ddof, a_max=a_max)
        rb_ref = fusion.fuse_rewards(o, r, lp, beta, C)
        adv_ref = fusion.depth_advantages(o, rb_ref, C, eps=1e-8, ddof=ddof, a_max=a_max)
        assert np.abs(rb - rb_ref).max() < 1e-6, np.abs(rb - rb_ref).max()
        assert np.abs(adv - adv_ref).max() <= 1e-5, np.abs(adv - adv_ref).max()       # stated tolerance
    # equal rewards: zero advantages, not NaN
    rb, adv = _fuse(t, np.full(C * t.n_leaves, 0.25, np.float32), lp, 1.0)
    assert np.array_equal(adv, np.zeros_like(adv)) and np.allclose(rb, 0.25)


@pytest.mark.parametrize("kind", [br.REWARD_LINEAR, br.REWARD_TANH, br.REWARD_VIDEO])
def test_leaf_rewards_match_oracle(lib, kind):
    latent = (4, 5, 6, 10) if kind == br.REWARD_VIDEO else (4, 1, 37, 20)
    D = int(np.prod(latent))
    t = br.Tree(3, (0, 1), 2, n_tree=3)
    o = tree.tree_build(3, (0, 1), 2)
    rng = np.random.default_rng(kind)
    z = rng.standard_normal((3 * t.n_nodes, D)).astype(np.float32) * 2
    w = rng.standard_normal(latent[1] * latent[0] if kind == br.REWARD_VIDEO else D).astype(np.float32)
    out = torch.empty(3 * t.n_leaves, device=DEV)
    br.leaf_reward(t, dev(z), kind, dev(w), 0.7, latent, out, bytes_buffer(br.reward_scratch_bytes(t, kind, latent)))
    leaves = np.concatenate([z[c * t.n_nodes + t.off[3]: (c + 1) * t.n_nodes] for c in range(3)])
    if kind == br.REWARD_VIDEO:
        ref = rewards.reward_video(leaves, w.reshape(latent[1], latent[0]), *latent, lam=0.7)
    else:
        ref = rewards.reward_linear(leaves, w, kind == br.REWARD_TANH)
    assert np.abs(host(out) - ref).max() < 2e-5 * max(1.0, np.abs(ref).max())


@pytest.mark.parametrize("T,splits,K,C", [(8, (2, 4, 6), 2, 1), (20, (4, 8, 12, 16), 2, 4), (20, (0, 3, 6, 9), 3, 3),
                                          (16, (3, 6, 9, 12), 4, 5), (6, (), 2, 2), (4, (1, 2), 1, 3),
                                          (12, tuple(range(10)), 2, 2),
                                          (16, (3, 6, 9, 12), 2, 2), (16, (4, 8, 12), 2, 1)])   # large-image and video trees
def test_pruned_edge_sets_are_bit_exact(lib, T, splits, K, C):
    t = br.Tree(T, splits, K, n_tree=C)
    o = tree.tree_build(T, splits, K)
    rng = np.random.default_rng(T + K + C)
    r = rng.standard_normal(C * t.n_leaves).astype(np.float32)
    r[rng.integers(0, r.size, r.size // 3)] = 0.5            # many exact ties
    masks = [None, prune.depth_mask_seeded(T, min(4, T), 42), prune.depth_mask_window(T, max(o["splits"] or [0]), 4, 60, 30, T)]
    kept = torch.empty(C * t.n_edges, dtype=torch.int32, device=DEV)
    nk = torch.zeros(1, dtype=torch.int32, device=DEV)
    for mode, b in ((0, 0), (1, 0), (2, 1), (2, 4), (2, 0), (2, 10 ** 6)):
        for mask in masks:
            kept.fill_(-7)
            br.prune(t, dev(r), mode, b, mask, kept, nk)
            ref = prune.kept_edges(o, r, C, mode, b, mask if mask is not None else np.zeros(T, np.uint8))
            n = int(host(nk)[0])
            assert n == len(ref), (mode, b, n, len(ref))
            assert np.array_equal(host(kept)[:n], ref)


def test_grpo_objective_matches_oracle(lib):
    rng = np.random.default_rng(3)
    n_nodes, n = 500, 317
    ids = np.sort(rng.choice(n_nodes, n, replace=False)).astype(np.int32)
    lo = rng.standard_normal(n_nodes).astype(np.float32)
    adv = rng.standard_normal(n_nodes).astype(np.float32) * 2
    ln = (lo[ids] + rng.standard_normal(n).astype(np.float32) * 1e-2).astype(np.float32)
    J = torch.empty(1, device=DEV)
    clipped = torch.empty(n, dtype=torch.uint8, device=DEV)
    for eps in (1e-4, 0.2):
        br.grpo_objective(dev(ln), dev(lo), dev(adv), dev(ids), n, eps, J, clipped)
        ref, ref_clipped = objective.grpo_objective(ln, lo[ids], adv[ids], eps)
        assert abs(float(host(J)[0]) - ref) < 1e-6
        assert np.array_equal(host(clipped).astype(bool), ref_clipped)
        assert (0 < ref_clipped.sum() < n) == (eps == 1e-4)      # |log rho| ~ 1e-2: only the tight range clips
        br.grpo_objective(dev(ln), dev(lo), dev(adv), dev(ids), n, eps, J)          # the mask is optional
        assert abs(float(host(J)[0]) - ref) < 1e-6
    br.grpo_objective(dev(ln), dev(lo), dev(adv), dev(ids), 0, 0.2, J)
    assert float(host(J)[0]) == 0.0


@pytest.mark.parametrize("T,splits,K,C", [(8, (2, 4, 6), 2, 1), (20, (4, 8, 12, 16), 2, 4), (20, (0, 3, 6, 9), 3, 3),
                                          (16, (3, 6, 9, 12), 4, 2), (6, (), 2, 2),
                                          (16, (3, 6, 9, 12), 2, 2), (16, (4, 8, 12), 2, 1)])
def test_fusion_ess_matches_oracle(lib, T, splits, K, C):
    t, o = br.Tree(T, splits, K, n_tree=C), tree.tree_build(T, splits, K)
    rng = np.random.default_rng(T + K)
    n = C * t.n_nodes
    logp = (rng.standard_normal(n) * 0.7).astype(np.float32)
    ess = torch.full((n,), -1.0, device=DEV)
    for beta in (1.0, 0.0, 3.5):
        br.fusion_ess(t, dev(logp), beta, ess)
        ref = fusion.ess(o, logp, beta, C)
        assert np.all(np.abs(host(ess) - ref) <= 1e-5 * ref), beta


def test_tree_kernels_at_and_beyond_their_largest_trees(lib):
    """4096 leaves per tree is the most fusion and ESS take, 8191 the most pruning takes; beyond that the
    calls refuse with a shape error before anything is launched."""
    T = 12
    t, o = br.Tree(T, tuple(range(12)), 2, n_tree=1), tree.tree_build(T, tuple(range(12)), 2)
    assert t.n_leaves == 4096 and t.n_nodes == 8191
    rng = np.random.default_rng(12)
    r = rng.standard_normal(t.n_leaves).astype(np.float32)
    lp = (rng.standard_normal(t.n_nodes) * 0.5).astype(np.float32)
    rb, adv = _fuse(t, r, lp, 1.0)
    rb_ref = fusion.fuse_rewards(o, r, lp, 1.0, 1)
    assert np.abs(rb - rb_ref).max() < 1e-6
    assert np.abs(adv - fusion.depth_advantages(o, rb_ref, 1, eps=1e-8, ddof=0, a_max=5.0)).max() <= 1e-5
    ess = torch.empty(t.n_nodes, device=DEV)
    br.fusion_ess(t, dev(lp), 1.0, ess)
    ref = fusion.ess(o, lp, 1.0, 1)
    assert np.all(np.abs(host(ess) - ref) <= 1e-5 * ref)
    kept = torch.empty(t.n_edges, dtype=torch.int32, device=DEV)
    nk = torch.zeros(1, dtype=torch.int32, device=DEV)
    br.prune(t, dev(r), br.PRUNE_EXTREME, 100, None, kept, nk)
    assert np.array_equal(host(kept)[:int(host(nk)[0])], prune.kept_edges(o, r, 1, 2, 100, np.zeros(T, np.uint8)))
    big = br.Tree(13, tuple(range(13)), 2, n_tree=1)          # 8192 leaves
    r2, lp2 = dev(np.zeros(big.n_leaves, np.float32)), dev(np.zeros(big.n_nodes, np.float32))
    out = torch.empty(big.n_nodes, device=DEV)
    for call in (lambda: br.fuse_advantage(big, r2, lp2, 1.0, 1e-8, 0, 5.0, out, out.clone()),
                 lambda: br.fusion_ess(big, lp2, 1.0, out),
                 lambda: br.prune(big, r2, br.PRUNE_NONE, 0, None, torch.empty(big.n_edges, dtype=torch.int32, device=DEV), nk)):
        with pytest.raises(br.BranchRolloutError) as e:
            call()
        assert e.value.code == -3
