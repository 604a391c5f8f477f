"""GPU parity of the whole path on the tiny workload (end to end against the
oracle) and the structural properties the method fixes."""
import numpy as np
import pytest
import torch

from oracle import dit, fusion, prune, rewards, rollout, tree
from paper_2509_06040_amd import binding as br
from paper_2509_06040_amd import synth
from gpu_util import DEV, assert_velocity, bytes_buffer, cond_dev, dev, host, make_model, rel_l2

pytestmark = pytest.mark.gpu


def _run_rollout(wl, n_cond, seed, groups, K=None, splits=None, logp_mean=False, want_v=True, W=None, max_batch=None,
                 ode_steps=()):
    cfg = wl["model"]
    W = W if W is not None else synth.make_weights(cfg, 0)
    D = synth.model_sizes(cfg)["D"]
    K = wl["K"] if K is None else K
    splits = wl["splits"] if splits is None else splits
    t = br.Tree(wl["T"], splits, K, n_tree=n_cond)
    model = make_model(cfg, W)
    cond = synth.cond_tokens(cfg, n_cond)
    sched = synth.schedule(wl["T"], wl["kappa"], logp_mean=logp_mean, ode_steps=ode_steps)
    n = n_cond * t.n_nodes
    z = torch.full((n, D), 9.0, device=DEV)
    logp = torch.full((n,), 9.0, device=DEV)
    v = torch.zeros((n, D), device=DEV) if want_v else None
    mb = max_batch or n_cond * t.n_leaves
    ws = bytes_buffer(br.workspace_bytes(t, model, mb))
    br.rollout(t, model, sched, seed, groups, cond_dev(cfg, cond), z, logp, v, ws)
    return dict(t=t, model=model, W=W, cond=cond, sched=sched, z=z, logp=logp, v=v, D=D, ws=ws, cfg=cfg)


def test_tiny_workload_end_to_end_matches_oracle(lib):
    wl = synth.WORKLOADS["tiny"]
    C = 2
    r = _run_rollout(wl, C, synth.SAMPLER_SEED, [0, 1])
    t, cfg, W, cond, sched, D = r["t"], r["cfg"], r["W"], r["cond"], r["sched"], r["D"]
    o = tree.tree_build(wl["T"], wl["splits"], wl["K"])
    vel = lambda zz, tt, ci: dit.forward(cfg, W, zz, tt, cond, ci)
    zr, lpr, vr = rollout.tree_rollout(o, vel, sched, synth.SAMPLER_SEED, [0, 1], D, C)
    z, lp, v = host(r["z"]), host(r["logp"]), host(r["v"])
    assert np.abs(z - zr).max() < 2e-4, np.abs(z - zr).max()
    for nrow in range(C * t.n_nodes):
        if t.depth[nrow % t.n_nodes] < t.T:
            assert_velocity(cfg, v[nrow], vr[nrow], 1e-4, "tiny rollout node %d" % nrow)
        if nrow % t.n_nodes:
            assert abs(lp[nrow] - lpr[nrow]) <= 1e-3 * abs(lpr[nrow])
        else:
            assert lp[nrow] == 0.0
    # rewards -> fusion -> advantages -> pruning -> re-evaluation under perturbed weights
    w = synth.reward_vector(D, 7)
    latent = (cfg["latent_c"], cfg["latent_t"], cfg["latent_h"], cfg["latent_w"])
    rew = torch.empty(C * t.n_leaves, device=DEV)
    br.leaf_reward(t, r["z"], br.REWARD_LINEAR, dev(w), 0.0, latent, rew, bytes_buffer(br.reward_scratch_bytes(t, 0, latent)))
    leaves = np.concatenate([zr[c * t.n_nodes + t.off[t.T]:(c + 1) * t.n_nodes] for c in range(C)])
    rew_ref = rewards.reward_linear(leaves, w)
    assert np.abs(host(rew) - rew_ref).max() < 1e-4
    # advantages from identical leaf rewards and log-probs (stated tolerance 1e-5)
    rew_same, lp_same = host(rew).copy(), lp.copy()
    rbar, adv = torch.empty(C * t.n_nodes, device=DEV), torch.empty(C * t.n_nodes, device=DEV)
    br.fuse_advantage(t, rew, r["logp"], 1.0, 1e-8, 0, synth.ADV_CLIP, rbar, adv)
    rb_ref = fusion.fuse_rewards(o, rew_same, lp_same / D, 1.0, C)      # MEAN log-probs keep the softmax soft
    br.fuse_advantage(t, rew, dev((lp_same / D).astype(np.float32)), 1.0, 1e-8, 0, synth.ADV_CLIP, rbar, adv)
    rb_ref = fusion.fuse_rewards(o, rew_same, (lp_same / D).astype(np.float32), 1.0, C)
    adv_ref = fusion.depth_advantages(o, rb_ref, C, 1e-8, 0, synth.ADV_CLIP)
    assert np.abs(host(adv) - adv_ref).max() <= 1e-5 and np.abs(host(rbar) - rb_ref).max() < 1e-6
    mask = prune.depth_mask_seeded(wl["T"], 2, synth.DATA_SEED)
    kept, nk = torch.empty(C * t.n_edges, dtype=torch.int32, device=DEV), torch.zeros(1, dtype=torch.int32, device=DEV)
    br.prune(t, rew, br.PRUNE_EXTREME, 2, mask, kept, nk)
    ids = host(kept)[:int(host(nk)[0])]
    assert np.array_equal(ids, prune.kept_edges(o, rew_same, C, 2, 2, mask))
    W2 = synth.perturb_weights(cfg, W, 11, 0.002)
    model2 = make_model(cfg, W2)
    lp_new = torch.empty(len(ids), device=DEV)
    br.logprob(t, model2, sched, cond_dev(cfg, cond), r["z"], ids, lp_new, r["ws"])
    vel2 = lambda zz, tt, ci: dit.forward(cfg, W2, zz, tt, cond, ci)
    ref_new = rollout.edge_logprob(o, vel2, sched, z.astype(np.float64), ids, C)   # teacher-forced on the stored latents
    got_new = host(lp_new)
    assert np.all(np.abs(got_new - ref_new) <= 1e-3 * np.abs(ref_new))
    assert np.abs(got_new - lp[ids]).max() > 0                                       # the policy did change
    # same weights: the re-evaluation reproduces the behaviour log-probs
    br.logprob(t, r["model"], sched, cond_dev(cfg, cond), r["z"], ids, lp_new, r["ws"])
    assert np.all(np.abs(host(lp_new) - lp[ids]) <= 1e-3 * np.abs(lp[ids]))


def test_branching_factor_one_is_the_flat_rollout(lib):
    wl = synth.WORKLOADS["tiny"]
    N = 4
    r = _run_rollout(wl, N, 5, [0, 0, 1, 2], K=1)
    cfg, W, cond, sched, D = r["cfg"], r["W"], r["cond"], r["sched"], r["D"]
    vel = lambda zz, tt, ci: dit.forward(cfg, W, zz, tt, cond, ci)
    zf, lpf = rollout.flat_rollout(N, wl["T"], vel, sched, 5, [0, 0, 1, 2], D)
    assert np.abs(host(r["z"]) - zf).max() < 2e-4
    lp = host(r["logp"])
    nz = lpf != 0
    assert np.all(np.abs(lp[nz] - lpf[nz]) <= 1e-3 * np.abs(lpf[nz])) and np.all(lp[~nz] == 0)
    z = host(r["z"])
    assert np.array_equal(z[0], z[wl["T"] + 1])                 # same noise group: same z_0


@pytest.mark.parametrize("K,splits", [(3, (1, 4)), (4, (0, 5)), (5, (2,))])
def test_larger_branching_factors_end_to_end(lib, K, splits):
    """Larger trees of the scaling study: K = 3, 4 (fused kernel) and 5 (generic kernel)."""
    wl = synth.WORKLOADS["tiny"]
    C = 2
    r = _run_rollout(wl, C, 31, [0, 0], K=K, splits=splits, logp_mean=True)
    t, cfg, W, cond, sched, D = r["t"], r["cfg"], r["W"], r["cond"], r["sched"], r["D"]
    o = tree.tree_build(wl["T"], splits, K)
    assert t.n_leaves == K ** len(splits)
    vel = lambda zz, tt, ci: dit.forward(cfg, W, zz, tt, cond, ci)
    zr, lpr, _ = rollout.tree_rollout(o, vel, sched, 31, [0, 0], D, C)
    z, lp = host(r["z"]), host(r["logp"])
    assert np.abs(z - zr).max() < 2e-4
    nz = lpr != 0
    assert np.all(np.abs(lp[nz] - lpr[nz]) <= 1e-3 * np.abs(lpr[nz])) and np.all(lp[~nz] == 0)
    # fusion, advantages and Parent-Top1 pruning on the same tree
    rew = np.tanh(zr[[c * t.n_nodes + t.off[t.T] + l for c in range(C) for l in range(t.n_leaves)]].mean(axis=1) * 30)
    rew = rew.astype(np.float32)
    rbar, adv = torch.empty(C * t.n_nodes, device=DEV), torch.empty(C * t.n_nodes, device=DEV)
    br.fuse_advantage(t, dev(rew), r["logp"], 1.0, 1e-8, 0, synth.ADV_CLIP, rbar, adv)
    rb_ref = fusion.fuse_rewards(o, rew, lp, 1.0, C)
    adv_ref = fusion.depth_advantages(o, rb_ref, C, 1e-8, 0, synth.ADV_CLIP)
    assert np.abs(host(adv) - adv_ref).max() <= 1e-5
    kept = torch.empty(C * t.n_edges, dtype=torch.int32, device=DEV)
    nk = torch.zeros(1, dtype=torch.int32, device=DEV)
    br.prune(t, dev(rew), br.PRUNE_PARENT_TOP1, 0, None, kept, nk)
    assert np.array_equal(host(kept)[:int(host(nk)[0])], prune.kept_edges(o, rew, C, 1, 0, np.zeros(t.T, np.uint8)))


def test_siblings_share_their_prefix_and_chunking_changes_nothing(lib):
    wl = synth.WORKLOADS["tiny"]
    a = _run_rollout(wl, 2, 9, [0, 1])
    b = _run_rollout(wl, 2, 9, [0, 1], max_batch=3, want_v=False)       # frontier processed in chunks of <= 3
    assert np.array_equal(host(a["z"]), host(b["z"])) and np.array_equal(host(a["logp"]), host(b["logp"]))
    t, z = a["t"], host(a["z"])
    o = tree.tree_build(wl["T"], wl["splits"], wl["K"])
    # every node has exactly one stored latent per (tree, level slot); children of one
    # parent differ, and the velocity was evaluated once per parent (non-leaf rows only)
    v = host(a["v"])
    for n in range(t.n_nodes):
        assert (np.abs(v[n]).sum() > 0) == (t.depth[n] < t.T)
    for n in range(t.n_nodes):
        kids = tree.children(o, n)
        if len(kids) == 2:
            assert not np.array_equal(z[kids[0]], z[kids[1]])
    # a rerun with the same seed is bit-identical; another seed is not
    c = _run_rollout(wl, 2, 9, [0, 1])
    assert np.array_equal(host(c["z"]), z)
    d = _run_rollout(wl, 2, 10, [0, 1])
    assert not np.array_equal(host(d["z"]), z)


def test_ode_steps_in_the_rollout(lib):
    wl = synth.WORKLOADS["tiny"]
    r = _run_rollout(wl, 1, 3, [0], ode_steps=(0, 3, 7))
    t, lp = r["t"], host(r["logp"])
    for n in range(1, t.n_nodes):
        assert (lp[n] == 0.0) == (t.depth[n] - 1 in (0, 3, 7))


def test_hybrid_ode_sde_schedule_end_to_end(lib):
    """Hybrid ODE-SDE ablation: split steps and a sliding window stay stochastic, the other steps are
    deterministic, carry no log-prob and are left out of the update."""
    wl = synth.WORKLOADS["tiny"]
    T, splits, C = wl["T"], wl["splits"], 2
    win = br.depth_mask_window(T, splits[-1], 2, 0, 30, T)
    sigma, ode = br.mix_schedule(T, splits, win, synth.ETA)
    assert 0 < ode.sum() < T
    r = _run_rollout(wl, C, 77, [0, 1], ode_steps=tuple(np.nonzero(ode)[0]))
    assert np.array_equal(r["sched"]["sigma"], sigma)
    t, cfg, W, cond, sched, D = r["t"], r["cfg"], r["W"], r["cond"], r["sched"], r["D"]
    o = tree.tree_build(T, splits, wl["K"])
    vel = lambda zz, tt, ci: dit.forward(cfg, W, zz, tt, cond, ci)
    zr, lpr, _ = rollout.tree_rollout(o, vel, sched, 77, [0, 1], D, C)
    z, lp = host(r["z"]), host(r["logp"])
    assert np.abs(z - zr).max() < 2e-4
    for n in range(C * t.n_nodes):
        step = t.depth[n % t.n_nodes] - 1
        if step < 0 or ode[step]:
            assert lp[n] == 0.0 and lpr[n] == 0.0
        else:
            assert abs(lp[n] - lpr[n]) <= 1e-3 * abs(lpr[n])
    # the ODE mask as depth mask keeps exactly the edges of stochastic steps
    rew = dev(np.arange(C * t.n_leaves, dtype=np.float32))
    kept = torch.empty(C * t.n_edges, dtype=torch.int32, device=DEV)
    nk = torch.zeros(1, dtype=torch.int32, device=DEV)
    br.prune(t, rew, br.PRUNE_NONE, 0, ode, kept, nk)
    ids = host(kept)[:int(host(nk)[0])]
    assert np.array_equal(ids, prune.kept_edges(o, host(rew), C, 0, 0, ode))
    assert all(not ode[t.depth[g % t.n_nodes] - 1] for g in ids) and len(ids) == sum(
        C * t.width[i + 1] for i in range(T) if not ode[i])
    out = torch.empty(len(ids), device=DEV)
    br.logprob(t, r["model"], sched, cond_dev(cfg, cond), r["z"], ids, out, r["ws"])
    ref = rollout.edge_logprob(o, vel, sched, z.astype(np.float64), ids, C)
    assert np.all(np.abs(host(out) - ref) <= 1e-3 * np.abs(ref))


def test_logprob_batches_spanning_and_cutting_steps(lib):
    """The re-evaluation batches parents across steps (one time per modulation group); with a
    workspace for 3 samples at a time the batches both span several steps and cut steps in two."""
    wl = synth.WORKLOADS["tiny"]
    C = 2
    r = _run_rollout(wl, C, 21, [0, 1], ode_steps=(3,))
    t, cfg, W, cond, sched, D = r["t"], r["cfg"], r["W"], r["cond"], r["sched"], r["D"]
    o = tree.tree_build(wl["T"], wl["splits"], wl["K"])
    W2 = synth.perturb_weights(cfg, W, 5, 0.01)
    model2 = make_model(cfg, W2)
    rng = np.random.default_rng(0)
    all_edges = np.array([c * t.n_nodes + n for c in range(C) for n in range(1, t.n_nodes)], np.int32)
    ids = np.sort(rng.choice(all_edges, size=len(all_edges) * 2 // 3, replace=False)).astype(np.int32)
    vel2 = lambda zz, tt, ci: dit.forward(cfg, W2, zz, tt, cond, ci)
    z = host(r["z"])
    ref = rollout.edge_logprob(o, vel2, sched, z.astype(np.float64), ids, C)
    for max_batch in (3, C * t.n_leaves):
        ws = bytes_buffer(br.workspace_bytes(t, model2, max_batch))
        out = torch.full((len(ids),), 7.0, device=DEV)
        br.logprob(t, model2, sched, cond_dev(cfg, cond), r["z"], ids, out, ws)
        got = host(out)
        ode = np.array([t.depth[g % t.n_nodes] - 1 == 3 for g in ids])
        assert np.all(got[ode] == 0.0) and np.all(ref[ode] == 0.0)
        assert np.all(np.abs(got[~ode] - ref[~ode]) <= 1e-3 * np.abs(ref[~ode])), max_batch


def test_rollout_rejects_bad_arguments(lib):
    wl = synth.WORKLOADS["tiny"]
    r = _run_rollout(wl, 1, 3, [0])
    t, model, cfg = r["t"], r["model"], r["cfg"]
    cond = cond_dev(cfg, r["cond"])
    with pytest.raises(br.BranchRolloutError) as e:
        br.rollout(t, model, r["sched"], 1, [0], cond, r["z"], r["logp"], None, bytes_buffer(1024))
    assert e.value.code == -4
    bad = dict(r["sched"], t=r["sched"]["t"][:-1], sigma=r["sched"]["sigma"][:-1])
    with pytest.raises(br.BranchRolloutError) as e:
        br.rollout(t, model, bad, 1, [0], cond, r["z"], r["logp"], None, r["ws"])
    assert e.value.code == -1
    out = torch.empty(2, device=DEV)
    for ids in ([0, 3], [5, 4], [3, 3], [10 ** 6]):
        with pytest.raises(br.BranchRolloutError):
            br.logprob(t, model, r["sched"], cond, r["z"], ids, out, r["ws"])
