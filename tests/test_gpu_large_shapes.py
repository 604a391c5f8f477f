"""GPU parity at the large-image and video shapes (hidden 3072 / 1536, head dim 128,
4608 / 33272 tokens, 2M-element latents), at the batch sizes of the workloads' widest
frontiers: batched networks of two blocks / one block teacher-forced against the oracle
(bf16 tolerance 2e-2, per sample, per token and per element), the full frontier against the
oracle-checked samples, the attention launch of each workload's shape on sampled queries, the SDE
step and the video reward at full latent size, and fusion, advantages and pruning on the two
workloads' trees."""
import numpy as np
import pytest
import torch

from oracle import dit, philox, rewards, sde, tree
from paper_2509_06040_amd import binding as br
from paper_2509_06040_amd import synth
from gpu_util import DEV, assert_tokens, assert_velocity, bytes_buffer, cond_dev, dev, host, make_model

pytestmark = pytest.mark.gpu


def _blocks(name, n):
    cfg = dict(synth.WORKLOADS[name]["model"])
    cfg["n_blocks"] = n
    return cfg


@pytest.fixture(scope="module")
def large_case(lib):
    """Two blocks of the large-image network (hidden 3072, 24 heads of 128, L = 4096 + 512, fp32
    residual stream carried from one block into the next), two prompts, 32 latents: the frontier
    size of the workload's last depths (GEMM rows M = 147 456)."""
    cfg = _blocks("image_large", 2)
    D = synth.model_sizes(cfg)["D"]
    W = synth.make_weights(cfg, 1, 0.02)
    z = synth.random_latents(32, D, 2)
    cond = synth.cond_tokens(cfg, 2, 3)
    cidx = np.array([0, 1, 0] + [(b * 7 + 1) % 2 for b in range(3, 32)])
    model = make_model(cfg, W)
    return dict(cfg=cfg, D=D, W=W, z=z, cond=cond, cidx=cidx, model=model)


# the oracle takes about a minute per sample here (two blocks of 1.3 TFLOP in fp64, single-threaded
# exp / tanh), hence one case per sample of the batch
@pytest.mark.parametrize("b", [0, 1, 2])
def test_large_image_shape_two_blocks_batch_of_three_matches_oracle(large_case, b):
    r = large_case
    cfg, D = r["cfg"], r["D"]
    if "v3" not in r:
        v = torch.empty((3, D), device=DEV)
        br.velocity(r["model"], dev(r["z"][:3]), 0.6, cond_dev(cfg, r["cond"]), r["cidx"][:3], v,
                    bytes_buffer(br.workspace_bytes(None, r["model"], 3)))
        r["v3"] = host(v)
    ref = dit.forward(cfg, r["W"], r["z"][b:b + 1], 0.6, r["cond"], r["cidx"][b:b + 1], act_round=dit.round_bf16)[0]
    assert_velocity(cfg, r["v3"][b], ref, 2e-2, "large image, 2 blocks, sample %d of 3" % b)


def test_large_image_shape_full_frontier_agrees_with_the_checked_batch(large_case):
    r = large_case
    cfg, D = r["cfg"], r["D"]
    if "v3" not in r:
        pytest.skip("needs the oracle-checked batch of the previous test")
    v = torch.empty((32, D), device=DEV)
    br.velocity(r["model"], dev(r["z"]), 0.6, cond_dev(cfg, r["cond"]), r["cidx"], v,
                bytes_buffer(br.workspace_bytes(None, r["model"], 32)))
    got = host(v)
    # the same three latents inside the batch of 32 (other tiles, other workgroups, the attention's
    # grouped launch order): far inside the bf16 tolerance of the oracle check above
    for b in range(3):
        assert_velocity(cfg, got[b], r["v3"][b], 2e-3, "large image, sample %d in the batch of 32" % b)
    # and no sample of the batch is a copy of another or left unwritten
    n = np.linalg.norm(got, axis=1)
    assert np.all(n > 0.5 * n[0]) and np.all(n < 2 * n[0])
    assert len({got[b].tobytes() for b in range(32)}) == 32


@pytest.fixture(scope="module")
def video_case(lib):
    """One block of the video network (hidden 1536, 12 heads of 128, L = 32760 + 512: not a multiple
    of the 128-row wave tiles, so tiles span two samples), two prompts, 8 latents: the workload's
    widest frontier (GEMM rows M = 266 176)."""
    cfg = _blocks("video", 1)
    sz = synth.model_sizes(cfg)
    W = synth.make_weights(cfg, 4, 0.02)
    z = synth.random_latents(8, sz["D"], 5)
    cond = synth.cond_tokens(cfg, 2, 6)
    cidx = np.array([0, 1, 1, 0, 1, 0, 0, 1])
    model = make_model(cfg, W)
    v = torch.empty((8, sz["D"]), device=DEV)
    br.velocity(model, dev(z), 0.3, cond_dev(cfg, cond), cidx, v, bytes_buffer(br.workspace_bytes(None, model, 8)))
    return dict(cfg=cfg, sz=sz, W=W, z=z, cond=cond, cidx=cidx, model=model, v=host(v))


@pytest.mark.parametrize("b", [0, 5])
def test_video_shape_batch_of_eight_matches_oracle_on_sampled_tokens(video_case, b):
    r = video_case
    cfg, sz = r["cfg"], r["sz"]
    rows = np.sort(np.random.default_rng(7 + b).choice(sz["n_img"], 96, replace=False))
    rows[0], rows[-1] = 0, sz["n_img"] - 1
    ref = dit.forward_rows(cfg, r["W"], r["z"][b:b + 1], 0.3, r["cond"], r["cidx"][b:b + 1], rows, act_round=dit.round_bf16)[0]
    got = dit.patchify(cfg, r["v"][b:b + 1].astype(np.float64))[0][rows]
    assert np.linalg.norm(ref) > 0.1
    assert_tokens(got, ref, 2e-2, "video, sample %d of 8" % b)


def test_video_shape_batch_of_eight_agrees_with_single_samples(video_case):
    r = video_case
    cfg, sz = r["cfg"], r["sz"]
    ws = bytes_buffer(br.workspace_bytes(None, r["model"], 2))     # sized for the two prompts' conditioning
    for b in (3, 7):                                     # one sample of each prompt, alone
        v1 = torch.empty((1, sz["D"]), device=DEV)
        br.velocity(r["model"], dev(r["z"][b:b + 1]), 0.3, cond_dev(cfg, r["cond"]), r["cidx"][b:b + 1], v1, ws)
        assert_velocity(cfg, r["v"][b], host(v1)[0], 2e-3, "video, sample %d alone against the batch of 8" % b)
    assert len({r["v"][b].tobytes() for b in range(8)}) == 8


def _tree_rollout(name, n_blocks, seed):
    """The workload's own tree (all prompts, every frontier size) through br_rollout with a network
    of n_blocks blocks; returns what the sampled-node checks below need."""
    wl = synth.WORKLOADS[name]
    cfg = _blocks(name, n_blocks)
    D = synth.model_sizes(cfg)["D"]
    C, T = wl["n_cond"], wl["T"]
    W = synth.make_weights(cfg, seed, 0.02)
    cond = synth.cond_tokens(cfg, C, seed + 1)
    model = make_model(cfg, W)
    t = br.Tree(T, wl["splits"], wl["K"], n_tree=C)
    sched = synth.schedule(T, wl["kappa"], logp_mean=True)
    n = C * t.n_nodes
    z, v = torch.empty((n, D), device=DEV), torch.zeros((n, D), device=DEV)
    logp = torch.empty(n, device=DEV)
    ws = bytes_buffer(br.workspace_bytes(t, model, C * t.n_leaves))
    br.rollout(t, model, sched, synth.SAMPLER_SEED, list(range(C)), cond_dev(cfg, cond), z, logp, v, ws)
    torch.cuda.synchronize()
    return dict(wl=wl, cfg=cfg, D=D, C=C, T=T, W=W, cond=cond, t=t, sched=sched, z=z, v=v, logp=logp,
                o=tree.tree_build(T, wl["splits"], wl["K"]))


def _check_transition(r, g):
    """SDE step and log-prob of every child of global node g against the oracle, from the stored
    latent and velocity of g (Eq. 2, App. B.1)."""
    t, o, sched, D = r["t"], r["o"], r["sched"], r["D"]
    seed = synth.SAMPLER_SEED
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
        assert np.abs(host(r["z"][gc]) - ref).max() < 2e-5
        ref_lp = sde.transition_logp(ref, mu, std, True)
        assert abs(float(host(r["logp"][gc])) - ref_lp) <= 1e-3 * abs(ref_lp)


@pytest.fixture(scope="module")
def large_tree(lib):
    return _tree_rollout("image_large", 2, 21)


# the large-image workload's tree (2 prompts, T = 16, splits {3,6,9,12}: frontiers of 2 to 32 samples) rolled
# out by br_rollout with two blocks of its network; nodes of the smallest, a middle and the widest frontier,
# one of them a split parent, against the oracle: velocity (teacher-forced on the stored latent) and the
# transition to every child
@pytest.mark.parametrize("depth,cond,j", [(1, 1, 0), (6, 0, 1), (14, 1, 13)])
def test_large_image_tree_rollout_on_sampled_nodes(large_tree, depth, cond, j):
    r = large_tree
    t, cfg = r["t"], r["cfg"]
    assert j < int(t.width[depth])
    g = cond * t.n_nodes + int(t.off[depth]) + j
    ref = dit.forward(cfg, r["W"], host(r["z"][g:g + 1]), float(r["sched"]["t"][depth]), r["cond"], [cond],
                      act_round=dit.round_bf16)[0]
    assert_velocity(cfg, host(r["v"][g]), ref, 2e-2, "large-image tree, depth %d (batch %d)" % (depth, 2 * int(t.width[depth])))
    _check_transition(r, g)


def test_large_image_tree_rollout_structure(large_tree):
    r = large_tree
    t, C = r["t"], r["C"]
    lp = host(r["logp"]).reshape(C, -1)
    assert np.all(lp[:, 0] == 0.0) and np.all(lp[:, 1:] != 0.0) and np.all(np.isfinite(lp))
    z = r["z"].reshape(C, t.n_nodes, -1)
    # siblings differ after a split, and differ from their parent; different prompts differ
    for d in (4, 7, 10, 13):
        a, b = int(t.off[d]), int(t.off[d]) + 1
        assert int(t.parent[a]) == int(t.parent[b])
        assert float((z[0, a] - z[0, b]).abs().max()) > 1e-3
    assert float((z[0, 5] - z[1, 5]).abs().max()) > 1e-3


@pytest.fixture(scope="module")
def video_tree(lib):
    return _tree_rollout("video", 1, 31)


# the video workload's tree (1 prompt, T = 16, splits {4,8,12}: frontiers of 1 to 8 samples) with one block of
# its network: sampled tokens of a node of the first and of the widest frontier, and their transitions
@pytest.mark.parametrize("depth,j", [(2, 0), (13, 5)])
def test_video_tree_rollout_on_sampled_nodes(video_tree, depth, j):
    r = video_tree
    t, cfg = r["t"], r["cfg"]
    sz = synth.model_sizes(cfg)
    g = int(t.off[depth]) + j
    rows = np.sort(np.random.default_rng(depth).choice(sz["n_img"], 64, replace=False))
    rows[0], rows[-1] = 0, sz["n_img"] - 1
    ref = dit.forward_rows(cfg, r["W"], host(r["z"][g:g + 1]), float(r["sched"]["t"][depth]), r["cond"], [0], rows,
                           act_round=dit.round_bf16)[0]
    got = dit.patchify(cfg, host(r["v"][g:g + 1]).astype(np.float64))[0][rows]
    assert_tokens(got, ref, 2e-2, "video tree, depth %d (batch %d)" % (depth, int(t.width[depth])))
    _check_transition(r, g)


@pytest.mark.parametrize("name,B", [("video", 2), ("image_large", 3), ("image", 64)])
def test_attention_at_full_size_on_sampled_queries(lib, name, B):
    """The attention launch of the workload's shape (token count, heads, head dim; with 72 and
    1024 (sample, head) pairs the order that keeps a pair on one XCD), queries in the layout the
    QKV projection writes, against the oracle's attention on sampled query rows of the first and
    the last sample: first and last rows, the rows around query- and key-tile boundaries, the
    ragged tail."""
    cfg = synth.WORKLOADS[name]["model"]
    sz = synth.model_sizes(cfg)
    L, H, nh = sz["n_img"], cfg["hidden"], cfg["n_heads"]
    dh = H // nh
    c = np.log2(np.e) / np.sqrt(dh)
    gen = torch.Generator(device=DEV)
    gen.manual_seed(L + B)
    x = torch.randn((B, L, 3 * H), device=DEV, generator=gen) * 1.5
    x[..., :H] *= c
    qkv = x.to(torch.bfloat16)
    del x
    out = torch.full((B, L, H), 3.0, dtype=torch.bfloat16, device=DEV)
    br.op_attention(br.BF16, qkv, out, nh, q_prescaled=1)
    rows = np.unique(np.concatenate([[0, 1, 31, 32, 63, 64, 127, 128, 129, 255, 256, L // 2, L - 130, L - 129, L - 128,
                                      L - (L % 64) - 1, L - (L % 64), L - 2, L - 1],
                                     np.random.default_rng(L).choice(L, 24, replace=False)]) % L)
    for b in (0, B - 1):
        sample = qkv[b].float().cpu().numpy().astype(np.float64)
        q = sample[rows, :H] / c
        ref = dit.attention(q, sample[:, H:2 * H], sample[:, 2 * H:], nh)
        got = out[b].float().cpu().numpy()[rows]
        assert np.isfinite(got).all()
        # all sampled rows together as in the small attention tests; every row; every element against its
        # own size plus the rows' RMS (a head that looks at a dozen keys has elements ten times the RMS,
        # and the output is rounded to bf16)
        err = np.linalg.norm(got - ref) / np.linalg.norm(ref)
        assert err < 3e-3, (name, b, err)
        tok = np.linalg.norm(got - ref, axis=1) / np.linalg.norm(ref, axis=1)
        assert tok.max() < 1e-2, (name, b, int(rows[tok.argmax()]), tok.max())
        el = np.abs(got - ref) / (np.abs(ref) + np.sqrt((ref ** 2).mean()))
        assert el.max() < 1e-2, (name, b, el.max())


def test_sde_step_and_video_reward_at_video_latent_size(lib):
    cfg = synth.WORKLOADS["video"]["model"]
    latent = (cfg["latent_c"], cfg["latent_t"], cfg["latent_h"], cfg["latent_w"])
    D = int(np.prod(latent))
    t = br.Tree(2, (0,), 2, n_tree=1)
    sched = synth.schedule(2, 3.0, logp_mean=False)
    seed = 99
    z = torch.zeros((t.n_nodes, D), device=DEV)
    br.root_noise(t, seed, [0], D, z)
    logp = torch.zeros(t.n_nodes, device=DEV)
    scratch = bytes_buffer(br.sde_scratch_bytes(t, D))
    rng = np.random.default_rng(1)
    for i in range(2):
        B = int(t.width[i])
        vv = rng.standard_normal((B, D)).astype(np.float32)
        zin = host(z).copy()
        br.sde_step(t, sched, seed, i, D, dev(vv), z, logp, scratch)
        zout, lp = host(z), host(logp)
        _, std = sde.step_coefficients(sched["t"][i], sched["t"][i + 1], sched["sigma"][i])
        for j in range(B):
            p = t.off[i] + j
            mu = sde.drift_mean(zin[p].astype(np.float64), vv[j].astype(np.float64), sched["t"][i], sched["t"][i + 1], sched["sigma"][i])
            kids = [2 * j, 2 * j + 1] if i == 0 else [j]
            xi0 = philox.normals(seed, p, i, philox.TAG_XI0, D) if i == 0 else None
            for jc in kids:
                ch = t.off[i + 1] + jc
                eta = philox.normals(seed, ch, i, philox.TAG_ETA, D)
                xi = sde.branch_noise(xi0, eta, sched["s"]) if xi0 is not None else eta
                ref = mu + std * xi
                assert np.abs(zout[ch] - ref).max() < 1e-5
                ref_lp = sde.transition_logp(ref, mu, std, False)
                assert abs(lp[ch] - ref_lp) <= 1e-3 * abs(ref_lp)
    w = synth.reward_vector(latent[1] * latent[0], 3)
    out = torch.empty(t.n_leaves, device=DEV)
    br.leaf_reward(t, z, br.REWARD_VIDEO, dev(w), 1.0, latent, out, bytes_buffer(br.reward_scratch_bytes(t, 2, latent)))
    ref = rewards.reward_video(host(z)[t.off[2]:], w.reshape(latent[1], latent[0]), *latent, lam=1.0)
    assert np.abs(host(out) - ref).max() < 2e-5 * max(1.0, np.abs(ref).max())
