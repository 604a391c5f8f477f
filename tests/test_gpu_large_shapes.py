"""GPU parity at the large-image and video shapes (hidden 3072 / 1536, head dim 128,
4608 / 33272 tokens, 2M-element latents): one-block networks teacher-forced against
the oracle (bf16 tolerance 2e-2), the SDE step and the video reward at full latent size."""
import numpy as np
import pytest
import torch

from oracle import dit, philox, rewards, sde, tree
from paper_2509_06040_amd import binding as br
from paper_2509_06040_amd import synth
from gpu_util import DEV, bytes_buffer, cond_dev, dev, host, make_model, rel_l2

pytestmark = pytest.mark.gpu


def _one_block(name):
    cfg = dict(synth.WORKLOADS[name]["model"])
    cfg["n_blocks"] = 1
    return cfg


def test_large_image_shape_one_block_velocity(lib):
    cfg = _one_block("image_large")                       # hidden 3072, 24 heads of 128, L = 4096 + 512
    D = synth.model_sizes(cfg)["D"]
    W = synth.make_weights(cfg, 1, 0.02)
    z = synth.random_latents(1, D, 2)
    cond = synth.cond_tokens(cfg, 1, 3)
    model = make_model(cfg, W)
    v = torch.empty((1, D), device=DEV)
    br.velocity(model, dev(z), 0.6, cond_dev(cfg, cond), [0], v, bytes_buffer(br.workspace_bytes(None, model, 1)))
    ref = dit.forward(cfg, W, z, 0.6, cond, [0], act_round=dit.round_bf16)
    err = rel_l2(host(v)[0], ref[0])
    assert err <= 2e-2, err


def test_video_shape_one_block_velocity_on_sampled_tokens(lib):
    cfg = _one_block("video")                             # hidden 1536, 12 heads of 128, L = 32760 + 512
    sz = synth.model_sizes(cfg)
    D = sz["D"]
    W = synth.make_weights(cfg, 4, 0.02)
    z = synth.random_latents(1, D, 5)
    cond = synth.cond_tokens(cfg, 1, 6)
    model = make_model(cfg, W)
    v = torch.empty((1, D), device=DEV)
    br.velocity(model, dev(z), 0.3, cond_dev(cfg, cond), [0], v, bytes_buffer(br.workspace_bytes(None, model, 1)))
    rows = np.sort(np.random.default_rng(7).choice(sz["n_img"], 96, replace=False))
    rows[0], rows[-1] = 0, sz["n_img"] - 1
    ref = dit.forward_rows(cfg, W, z, 0.3, cond, [0], rows, act_round=dit.round_bf16)[0]
    got = dit.patchify(cfg, host(v).astype(np.float64))[0][rows]
    err = rel_l2(got, ref)
    assert err <= 2e-2, err
    assert np.linalg.norm(ref) > 0.1


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
