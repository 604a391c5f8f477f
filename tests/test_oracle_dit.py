"""Pins for the oracle's velocity network: textbook identities and an independent
float64 PyTorch-CPU composition of library primitives."""
import numpy as np
import torch
import torch.nn.functional as F

from oracle import dit
from paper_2509_06040_amd import synth

CFG = synth.model_cfg(2, 32, 4, (3, 2, 4, 6), (1, 2, 2), 5, synth.F32)
CFG_T = synth.model_cfg(2, 32, 2, (2, 4, 4, 4), (2, 2, 2), 3, synth.F32)   # temporal patch > 1


def test_layer_norm_and_softmax_identities():
    x = np.random.default_rng(0).standard_normal((5, 64)) * 3 + 1
    y = dit.layer_norm(x, eps=0.0)
    assert np.allclose(y.mean(-1), 0, atol=1e-13) and np.allclose(y.var(-1), 1, atol=1e-12)
    assert np.allclose(dit.layer_norm(x), F.layer_norm(torch.from_numpy(x), (64,), eps=1e-6).numpy(), atol=1e-13)
    p = dit.softmax_rows(x)
    assert np.allclose(p.sum(-1), 1) and (p > 0).all()
    assert np.allclose(dit.gelu_tanh(x), F.gelu(torch.from_numpy(x), approximate="tanh").numpy(), atol=1e-13)
    assert np.allclose(dit.silu(x), F.silu(torch.from_numpy(x)).numpy(), atol=1e-13)


def test_attention_special_cases():
    rng = np.random.default_rng(1)
    q, k, v = rng.standard_normal((3, 1, 8))
    assert np.allclose(dit.attention(q, k, v, 2), v)                    # one token: returns V
    q, k, v = rng.standard_normal((3, 6, 8))
    assert np.allclose(dit.attention(q * 0, k, v, 2), np.tile(v.mean(0), (6, 1)))   # zero scores: mean of V
    tq, tk, tv = (torch.from_numpy(a).reshape(6, 2, 4).transpose(0, 1) for a in (q, k, v))
    ref = F.scaled_dot_product_attention(tq, tk, tv).transpose(0, 1).reshape(6, 8).numpy()
    assert np.allclose(dit.attention(q, k, v, 2), ref, atol=1e-13)


def test_patchify_roundtrip_and_layout():
    for cfg in (CFG, CFG_T):
        D = dit.dims(cfg)["D"]
        z = np.arange(2 * D, dtype=np.float64).reshape(2, D)
        p = dit.patchify(cfg, z)
        assert p.shape == (2, dit.dims(cfg)["n_img"], dit.dims(cfg)["patch_dim"])
        assert np.array_equal(dit.unpatchify(cfg, p), z)
    # explicit index check: token (gt, gh, gw), element (c, dt, dh, dw)
    cfg = CFG_T
    C, Tt, Hh, Ww = 2, 4, 4, 4
    z = np.random.default_rng(2).standard_normal((1, C * Tt * Hh * Ww))
    lat = z.reshape(C, Tt, Hh, Ww)
    p = dit.patchify(cfg, z)[0]
    tok = (1 * 2 + 1) * 2 + 0            # gt=1, gh=1, gw=0 on a 2x2x2 grid
    el = ((1 * 2 + 1) * 2 + 0) * 2 + 1   # c=1, dt=1, dh=0, dw=1
    assert p[tok, el] == lat[1, 1 * 2 + 1, 1 * 2 + 0, 0 * 2 + 1]


def test_bf16_rounding_is_nearest_even():
    x = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 2 ** -7, 1.0 + 3 * 2 ** -8, -0.1, 3.14159], dtype=np.float64)
    ref = torch.from_numpy(x).float().bfloat16().double().numpy()
    assert np.array_equal(dit.round_bf16(x), ref)
    assert dit.round_bf16(np.array([1.0 + 2 ** -8]))[0] == 1.0           # tie -> even
    assert dit.round_bf16(np.array([1.0 + 3 * 2 ** -8]))[0] == 1.0 + 2 ** -6


def _torch_forward(cfg, W, z, t, cond, cond_index):
    """Independent composition from torch.nn.functional primitives (float64)."""
    Wt = {k: torch.from_numpy(np.asarray(v, np.float64)) for k, v in W.items()}
    H, nb, nh = cfg["hidden"], cfg["n_blocks"], cfg["n_heads"]
    C, Tt, Hh, Ww = cfg["latent_c"], cfg["latent_t"], cfg["latent_h"], cfg["latent_w"]
    pt, ph, pw = cfg["patch_t"], cfg["patch_h"], cfg["patch_w"]
    zt = torch.from_numpy(z).double().reshape(-1, C, Tt, Hh, Ww)
    B = zt.shape[0]
    # patch embedding as a strided 3-D convolution
    x = F.conv3d(zt, Wt["patch_w"].reshape(H, C, pt, ph, pw), Wt["patch_b"], stride=(pt, ph, pw))
    x = x.flatten(2).transpose(1, 2) + Wt["pos"]
    ct = torch.from_numpy(cond).double()
    ce = F.linear(ct, Wt["cond_w"], Wt["cond_b"])[torch.as_tensor(cond_index)]
    x = torch.cat([x, ce], dim=1)
    k = torch.arange(128, dtype=torch.float64)
    ang = 1000.0 * t * torch.exp(-np.log(10000.0) * k / 128)
    te = torch.cat([torch.cos(ang), torch.sin(ang)])
    cvec = F.linear(F.silu(F.linear(te, Wt["t1_w"], Wt["t1_b"])), Wt["t2_w"], Wt["t2_b"])
    cvec = cvec + F.linear(ct.mean(1), Wt["pool_w"], Wt["pool_b"])
    mods = F.linear(F.silu(cvec), Wt["ada_w"], Wt["ada_b"])[torch.as_tensor(cond_index)][:, None, :]
    L = x.shape[1]
    for b in range(nb):
        m = mods[..., b * 6 * H:(b + 1) * 6 * H].chunk(6, dim=-1)
        xn = F.layer_norm(x, (H,), eps=1e-6) * (1 + m[1]) + m[0]
        q, kk, v = F.linear(xn, Wt["qkv_w"][b], Wt["qkv_b"][b]).chunk(3, dim=-1)
        sp = lambda a: a.reshape(B, L, nh, H // nh).transpose(1, 2)
        a = F.scaled_dot_product_attention(sp(q), sp(kk), sp(v)).transpose(1, 2).reshape(B, L, H)
        x = x + m[2] * F.linear(a, Wt["proj_w"][b], Wt["proj_b"][b])
        xn = F.layer_norm(x, (H,), eps=1e-6) * (1 + m[4]) + m[3]
        x = x + m[5] * F.linear(F.gelu(F.linear(xn, Wt["fc1_w"][b], Wt["fc1_b"][b]), approximate="tanh"),
                                Wt["fc2_w"][b], Wt["fc2_b"][b])
    mf = mods[..., nb * 6 * H:].chunk(2, dim=-1)
    n_img = L - cfg["n_cond_tokens"]
    o = F.linear(F.layer_norm(x[:, :n_img], (H,), eps=1e-6) * (1 + mf[1]) + mf[0], Wt["final_w"], Wt["final_b"])
    # fold the patch vectors back with the transposed strided convolution of an identity kernel
    pd = C * pt * ph * pw
    eye = torch.eye(pd, dtype=torch.float64).reshape(pd, C, pt, ph, pw)
    o = o.transpose(1, 2).reshape(B, pd, Tt // pt, Hh // ph, Ww // pw)
    return F.conv_transpose3d(o, eye, stride=(pt, ph, pw)).reshape(B, -1).numpy()


def test_timestep_embedding_closed_form_values():
    # sinusoid_256(1000 t) = [cos(1000 t f_k), sin(1000 t f_k)], f_k = 10000^(-k/128), k = 0..127
    e0 = dit.timestep_embedding(0.0)
    assert e0.shape == (256,) and np.array_equal(e0[:128], np.ones(128)) and np.array_equal(e0[128:], np.zeros(128))
    e = dit.timestep_embedding(np.pi / 1000.0)                 # 1000 t = pi
    assert abs(e[0] + 1.0) < 1e-12 and abs(e[128]) < 1e-12     # k = 0: f = 1 -> cos(pi), sin(pi)
    assert abs(e[64] - np.cos(0.01 * np.pi)) < 1e-12           # k = 64: f = 10000^(-1/2) = 0.01
    assert abs(e[128 + 64] - 0.031410759078128) < 1e-12        # sin(0.01 pi), written out
    # the slowest frequency: f_127 = 10000^(-127/128); cos and sin are a unit vector per k
    assert abs(e[127] - np.cos(np.pi * 10000.0 ** (-127.0 / 128.0))) < 1e-12
    assert np.allclose(e[:128] ** 2 + e[128:] ** 2, 1.0, atol=1e-12)


def test_forward_matches_independent_torch_composition():
    for cfg in (CFG, CFG_T):
        W = synth.make_weights(cfg, seed=3, std=0.2)        # large weights: every term matters
        D = dit.dims(cfg)["D"]
        z = synth.random_latents(3, D, 4).astype(np.float64)
        cond = synth.cond_tokens(cfg, 2, seed=5).astype(np.float64)
        cidx = np.array([1, 0, 1])
        ours = dit.forward(cfg, W, z, 0.37, cond, cidx)
        ref = _torch_forward(cfg, W, z, 0.37, cond, cidx)
        assert np.allclose(ours, ref, rtol=1e-10, atol=1e-12)
        assert np.linalg.norm(ours) > 1e-3


def test_zero_gates_make_the_blocks_the_identity():
    cfg = CFG
    W = synth.make_weights(cfg, seed=6, std=0.2)
    H, nb = cfg["hidden"], cfg["n_blocks"]
    for k in range(nb):
        for j in (2, 5):
            W["ada_w"][k * 6 * H + j * H:k * 6 * H + (j + 1) * H] = 0
            W["ada_b"][k * 6 * H + j * H:k * 6 * H + (j + 1) * H] = 0
    z = synth.random_latents(1, dit.dims(cfg)["D"], 7).astype(np.float64)
    cond = synth.cond_tokens(cfg, 1).astype(np.float64)
    W2 = dict(W)
    W2["qkv_w"] = W["qkv_w"] * 3 + 1                       # block weights no longer matter
    W2["fc1_w"] = W["fc1_w"] * -2
    a = dit.forward(cfg, W, z, 0.5, cond, [0])
    b = dit.forward(cfg, W2, z, 0.5, cond, [0])
    assert np.allclose(a, b, atol=1e-13)


def test_row_subset_forward_equals_the_full_forward():
    cfg = synth.model_cfg(1, 32, 4, (3, 2, 4, 6), (1, 2, 2), 5, synth.F32)
    W = synth.make_weights(cfg, seed=8, std=0.2)
    D = dit.dims(cfg)["D"]
    z = synth.random_latents(2, D, 9).astype(np.float64)
    cond = synth.cond_tokens(cfg, 2, seed=10).astype(np.float64)
    rows = np.array([0, 3, 5, 11])
    for rnd in (dit.identity, dit.round_bf16):
        full = dit.patchify(cfg, dit.forward(cfg, W, z, 0.4, cond, [1, 0], act_round=rnd))
        sub = dit.forward_rows(cfg, W, z, 0.4, cond, [1, 0], rows, act_round=rnd)
        assert np.allclose(sub, full[:, rows], rtol=1e-11, atol=1e-13)
