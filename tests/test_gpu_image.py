"""GPU parity at the image-shaped workload's full size, in the launch configuration
the benchmark times: the network on sampled nodes (teacher-forced, bf16 tolerance
2e-2), the SDE step / log-prob on every edge of sampled parents, and rewards,
fusion, advantages, pruned-edge sets and the re-evaluated log-probs in full."""
import numpy as np
import pytest
import torch

from oracle import dit, fusion, philox, prune, rewards, sde, tree
from paper_2509_06040_amd import binding as br
from paper_2509_06040_amd import synth
from gpu_util import DEV, assert_velocity, bytes_buffer, cond_dev, dev, host, make_model

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def image_run(lib):
    wl = synth.WORKLOADS["image"]
    cfg, T, C = wl["model"], wl["T"], wl["n_cond"]
    D = synth.model_sizes(cfg)["D"]
    W = synth.make_weights(cfg, 0)
    model = make_model(cfg, W)
    cond = synth.cond_tokens(cfg, C)
    sched = synth.schedule(T, wl["kappa"], logp_mean=True)
    t = br.Tree(T, wl["splits"], wl["K"], n_tree=C)
    n = C * t.n_nodes
    z, v = torch.empty((n, D), device=DEV), torch.zeros((n, D), device=DEV)
    logp = torch.empty(n, device=DEV)
    ws = bytes_buffer(br.workspace_bytes(t, model, C * t.n_leaves))
    br.rollout(t, model, sched, synth.SAMPLER_SEED, list(range(C)), cond_dev(cfg, cond), z, logp, v, ws)
    torch.cuda.synchronize()
    return dict(wl=wl, cfg=cfg, T=T, C=C, D=D, W=W, model=model, cond=cond, sched=sched, t=t, z=z, v=v, logp=logp, ws=ws,
                o=tree.tree_build(T, wl["splits"], wl["K"]))


# one node of every frontier size the rollout sends through the network (4 prompts x width 1, 2, 4, 8,
# 16 = batches of 4 to 64 samples; the GEMM tile kernel chosen differs with the batch size); different
# prompts, first / middle / last node of a frontier
@pytest.mark.parametrize("depth,cond,j", [(2, 1, 0), (5, 0, 1), (9, 2, 2), (14, 3, 7), (18, 3, 11)])
def test_velocity_on_a_node_of_every_frontier_size(image_run, depth, cond, j):
    r = image_run
    t, cfg = r["t"], r["cfg"]
    assert 4 * int(t.width[depth]) in (4, 8, 16, 32, 64)
    g = cond * t.n_nodes + int(t.off[depth]) + j
    z, v = host(r["z"][g:g + 1]), host(r["v"][g])
    ref = dit.forward(cfg, r["W"], z, float(r["sched"]["t"][depth]), r["cond"], [cond], act_round=dit.round_bf16)[0]
    assert np.linalg.norm(ref) > 1.0
    assert_velocity(cfg, v, ref, 2e-2, "image depth %d (batch %d)" % (depth, 4 * int(t.width[depth])))


def test_sde_step_and_logprob_on_sampled_parents(image_run):
    r = image_run
    t, o, sched, D = r["t"], r["o"], r["sched"], r["D"]
    seed = synth.SAMPLER_SEED
    lp = host(r["logp"])
    for g in (0, 2 * t.n_nodes + t.off[8] + 1, 3 * t.n_nodes + t.off[16] + 7, 1 * t.n_nodes + t.off[19] + 15):
        c, p = divmod(g, t.n_nodes)
        i = int(t.depth[p])
        zp, vp = host(r["z"][g]).astype(np.float64), host(r["v"][g]).astype(np.float64)
        mu = sde.drift_mean(zp, vp, sched["t"][i], sched["t"][i + 1], sched["sigma"][i])
        _, std = sde.step_coefficients(sched["t"][i], sched["t"][i + 1], sched["sigma"][i])
        kids = tree.children(o, p)
        xi0 = philox.normals(seed, g, i, philox.TAG_XI0, D) if len(kids) > 1 else None
        for ch in kids:
            gc = c * t.n_nodes + ch
            eta = philox.normals(seed, gc, i, philox.TAG_ETA, D)
            xi = sde.branch_noise(xi0, eta, sched["s"]) if xi0 is not None else eta
            ref = mu + std * xi
            got = host(r["z"][gc])
            assert np.abs(got - ref).max() < 2e-5
            ref_lp = sde.transition_logp(ref, mu, std, True)
            assert abs(lp[gc] - ref_lp) <= 1e-3 * abs(ref_lp)
    assert all(lp[c * t.n_nodes] == 0.0 for c in range(r["C"]))


def test_rewards_fusion_advantages_and_prune_in_full(image_run):
    r = image_run
    t, o, cfg, C, D, T = r["t"], r["o"], r["cfg"], r["C"], r["D"], r["T"]
    latent = (cfg["latent_c"], cfg["latent_t"], cfg["latent_h"], cfg["latent_w"])
    w = synth.reward_vector(D, 7)
    rew = torch.empty(C * t.n_leaves, device=DEV)
    br.leaf_reward(t, r["z"], br.REWARD_TANH, dev(w), 0.0, latent, rew, bytes_buffer(br.reward_scratch_bytes(t, 1, latent)))
    leaves = np.concatenate([host(r["z"][c * t.n_nodes + t.off[T]:(c + 1) * t.n_nodes]) for c in range(C)])
    ref = rewards.reward_linear(leaves, w, True)
    got = host(rew)
    assert np.abs(got - ref).max() < 1e-5
    lp = host(r["logp"])
    rbar, adv = torch.empty(C * t.n_nodes, device=DEV), torch.empty(C * t.n_nodes, device=DEV)
    br.fuse_advantage(t, rew, r["logp"], 1.0, 1e-8, 0, synth.ADV_CLIP, rbar, adv)
    rb_ref = fusion.fuse_rewards(o, got, lp, 1.0, C)                    # identical leaf rewards and log-probs
    adv_ref = fusion.depth_advantages(o, rb_ref, C, 1e-8, 0, synth.ADV_CLIP)
    assert np.abs(host(adv) - adv_ref).max() <= 1e-5
    a = host(adv).reshape(C, -1)
    for c in range(C):
        for d in range(5, T + 1):                                        # depths with more than one node
            x = a[c, t.off[d]:t.off[d + 1]]
            # std is sigma / (sigma + eps): slightly below 1 where the fused rewards of a depth are close
            assert abs(x.mean()) < 1e-5 and (abs(x.std() - 1) < 2e-3 or np.abs(x).max() == synth.ADV_CLIP)
    mask = prune.depth_mask_seeded(T, 4, synth.DATA_SEED)
    assert np.array_equal(mask, br.depth_mask_seeded(T, 4, synth.DATA_SEED))
    kept, nk = torch.empty(C * t.n_edges, dtype=torch.int32, device=DEV), torch.zeros(1, dtype=torch.int32, device=DEV)
    br.prune(t, rew, br.PRUNE_EXTREME, 4, mask, kept, nk)
    ids = host(kept)[:int(host(nk)[0])]
    assert np.array_equal(ids, prune.kept_edges(o, got, C, 2, 4, mask))
    image_run["ids"] = ids


def test_logprob_reevaluation_on_kept_edges(image_run):
    r = image_run
    t, o, cfg, C, D, sched = r["t"], r["o"], r["cfg"], r["C"], r["D"], r["sched"]
    ids = r.get("ids")
    if ids is None:
        pytest.skip("needs the kept-edge set of the previous test")
    # same policy: the re-evaluation reproduces the behaviour log-probs on every kept edge
    out = torch.empty(len(ids), device=DEV)
    br.logprob(t, r["model"], sched, cond_dev(cfg, r["cond"]), r["z"], ids, out, r["ws"])
    lp = host(r["logp"])
    assert np.all(np.abs(host(out) - lp[ids]) <= 1e-3 * np.abs(lp[ids]))
    # perturbed policy: kept for the oracle checks below
    W2 = synth.perturb_weights(cfg, r["W"], 11, 0.002)
    model2 = make_model(cfg, W2)
    br.logprob(t, model2, sched, cond_dev(cfg, r["cond"]), r["z"], ids, out, r["ws"])
    got = host(out)
    assert np.abs(got - lp[ids]).max() > 0
    image_run["lp_new"], image_run["W2"] = got, W2


# the oracle on one kept edge of every retained step (teacher-forced on the stored latents), four
# steps per case; the edge's prompt and position rotate with the step
@pytest.mark.parametrize("part", [0, 1, 2, 3])
def test_reevaluated_logprob_on_an_edge_of_every_retained_step(image_run, part):
    r = image_run
    t, cfg, sched = r["t"], r["cfg"], r["sched"]
    ids, got, W2 = r.get("ids"), r.get("lp_new"), r.get("W2")
    if got is None:
        pytest.skip("needs the re-evaluated log-probs of the previous test")
    step_of = np.array([int(t.depth[g % t.n_nodes]) - 1 for g in ids])
    steps = sorted(set(step_of.tolist()))
    assert len(steps) == r["T"] - 4                       # 4 of the 20 steps are dropped
    for i in steps[part::4]:
        where = np.nonzero(step_of == i)[0]
        e = int(where[(3 * i + 1) % len(where)])
        g = int(ids[e])
        c, nloc = divmod(g, t.n_nodes)
        p = c * t.n_nodes + int(t.parent[nloc])
        zp = host(r["z"][p]).astype(np.float64)
        v2 = dit.forward(cfg, W2, zp[None], float(sched["t"][i]), r["cond"], [c], act_round=dit.round_bf16)[0]
        mu = sde.drift_mean(zp, v2, sched["t"][i], sched["t"][i + 1], sched["sigma"][i])
        _, std = sde.step_coefficients(sched["t"][i], sched["t"][i + 1], sched["sigma"][i])
        ref = sde.transition_logp(host(r["z"][g]).astype(np.float64), mu, std, True)
        assert abs(got[e] - ref) <= 1e-3 * abs(ref), (i, g, got[e], ref)
