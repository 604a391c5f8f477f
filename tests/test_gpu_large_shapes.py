"""GPU parity at the large-image and video shapes (hidden 3072 / 1536, head dim 128,
4608 / 33272 tokens, 2M-element latents), at the batch sizes of the workloads' widest
frontiers: batched networks of two blocks / one block teacher-forced against the oracle
(bf16 tolerance 2e-2, per sample, per token and per element), the full frontier against the
oracle-checked samples, the SDE step and the video reward at full latent size, and fusion,
advantages and pruning on the two workloads' trees."""
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
