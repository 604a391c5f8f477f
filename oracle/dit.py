"""The synthetic DiT velocity network v_theta(z, t, c) for the oracle (test
infrastructure).

The paper evaluates a denoiser mu_theta(z_i, t_i) at every tree node (Eq. 2;
NFE columns of Table 1) but uses pretrained backbones whose weights are not
available; the workloads replace it by a randomly initialised DiT.  Its
definition (not from the paper):

  tokens  = [patch_embed(z) + pos ; cond_embed(c)]               L = N_img + N_cond
  cvec    = t_mlp(sinusoid_256(1000 t)) + pool_lin(mean_tokens(c))
  mods    = ada_lin(silu(cvec))   -> per block (shift1, scale1, gate1, shift2, scale2, gate2),
                                     then (shift, scale) of the final layer
  block:  x += gate1 * proj(attn(LN(x) (1+scale1) + shift1))
          x += gate2 * fc2(gelu_tanh(fc1(LN(x) (1+scale2) + shift2)))
  out     = unpatchify(final_lin(LN(x_img) (1+scale) + shift))

LayerNorm has no affine part, eps 1e-6, biased variance.  Attention is full,
bidirectional, softmax(Q K^T / sqrt(d_h)) V over all L tokens.  Every matrix is
[out, in] row-major.  `act_round` (identity, or round-to-bf16) is applied to
every activation that enters a matrix product or the attention: patch vectors,
condition tokens, LN-modulate outputs, q/k/v, the attention output and the GELU
output.  The residual stream, the conditioning path and all sums are fp64.

Pins (tests/test_oracle_dit.py): textbook identities only -- LN output has mean
0 / variance 1, softmax rows sum to 1, attention over one token returns V,
zero gates make a block the identity, patchify/unpatchify are inverse
permutations, and the whole forward agrees with an independent PyTorch-CPU
float64 module built from torch.nn.functional primitives.
PARITY UNPINNED beyond that: the architecture is the workload's, not the paper's.
"""
import numpy as np

WEIGHT_NAMES = (
    "patch_w", "patch_b", "pos", "cond_w", "cond_b", "t1_w", "t1_b", "t2_w", "t2_b",
    "pool_w", "pool_b", "ada_w", "ada_b", "qkv_w", "qkv_b", "proj_w", "proj_b",
    "fc1_w", "fc1_b", "fc2_w", "fc2_b", "final_w", "final_b",
)
T_FREQ_DIM = 256


def identity(a):
    return a


def round_bf16(a):
    """Round-to-nearest-even to bfloat16 (via float32), returned as fp64."""
    f = np.ascontiguousarray(np.asarray(a, dtype=np.float32))
    u = f.view(np.uint32)
    r = ((u.astype(np.uint64) + np.uint64(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)).astype(np.uint64))
         & np.uint64(0xFFFF0000)).astype(np.uint32)
    return r.view(np.float32).astype(np.float64)


def dims(cfg):
    """Derived sizes of a model configuration (dict with the keys of br_model_cfg)."""
    gt, gh, gw = (cfg["latent_t"] // cfg["patch_t"], cfg["latent_h"] // cfg["patch_h"],
                  cfg["latent_w"] // cfg["patch_w"])
    n_img = gt * gh * gw
    pd = cfg["latent_c"] * cfg["patch_t"] * cfg["patch_h"] * cfg["patch_w"]
    D = cfg["latent_c"] * cfg["latent_t"] * cfg["latent_h"] * cfg["latent_w"]
    return dict(grid=(gt, gh, gw), n_img=n_img, patch_dim=pd, D=D,
                L=n_img + cfg["n_cond_tokens"], d_head=cfg["hidden"] // cfg["n_heads"])


def patchify(cfg, z):
    """z [B, D] (latent stored [C, T, H, W]) -> [B, N_img, patch_dim]; tokens in
    (t, h, w) raster order, patch vector in (c, dt, dh, dw) order."""
    C, Tt, Hh, Ww = cfg["latent_c"], cfg["latent_t"], cfg["latent_h"], cfg["latent_w"]
    pt, ph, pw = cfg["patch_t"], cfg["patch_h"], cfg["patch_w"]
    B = z.shape[0]
    a = z.reshape(B, C, Tt // pt, pt, Hh // ph, ph, Ww // pw, pw)
    a = a.transpose(0, 2, 4, 6, 1, 3, 5, 7)  # B, gt, gh, gw, C, pt, ph, pw
    return a.reshape(B, (Tt // pt) * (Hh // ph) * (Ww // pw), C * pt * ph * pw)


def unpatchify(cfg, p):
    """Inverse of patchify: [B, N_img, patch_dim] -> [B, D]."""
    C, Tt, Hh, Ww = cfg["latent_c"], cfg["latent_t"], cfg["latent_h"], cfg["latent_w"]
    pt, ph, pw = cfg["patch_t"], cfg["patch_h"], cfg["patch_w"]
    B = p.shape[0]
    a = p.reshape(B, Tt // pt, Hh // ph, Ww // pw, C, pt, ph, pw)
    a = a.transpose(0, 4, 1, 5, 2, 6, 3, 7)  # B, C, gt, pt, gh, ph, gw, pw
    return a.reshape(B, C * Tt * Hh * Ww)


def layer_norm(x, eps=1e-6):
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    return (x - mu) / np.sqrt(var + eps)


def silu(x):
    return x / (1.0 + np.exp(-x))


def gelu_tanh(x):
    return 0.5 * x * (1.0 + np.tanh(np.sqrt(2.0 / np.pi) * (x + 0.044715 * x ** 3)))


def softmax_rows(s):
    e = np.exp(s - s.max(axis=-1, keepdims=True))
    return e / e.sum(axis=-1, keepdims=True)


def attention(q, k, v, n_heads):
    """q, k, v [L, H] of one sample -> [L, H]; full softmax attention per head."""
    L, H = q.shape
    dh = H // n_heads
    out = np.empty((L, H), dtype=np.float64)
    for h in range(n_heads):
        sl = slice(h * dh, (h + 1) * dh)
        p = softmax_rows(q[:, sl] @ k[:, sl].T / np.sqrt(dh))
        out[:, sl] = p @ v[:, sl]
    return out


def timestep_embedding(t):
    """sinusoid_256(1000 t): [cos(1000 t f_k), sin(1000 t f_k)], f_k = 10000^(-k/128)."""
    half = T_FREQ_DIM // 2
    f = np.exp(-np.log(10000.0) * np.arange(half, dtype=np.float64) / half)
    a = 1000.0 * float(t) * f
    return np.concatenate([np.cos(a), np.sin(a)])


def conditioning(cfg, W, t, cond):
    """cvec [C, H] and mods [C, n_blocks*6H + 2H] for every condition at time t."""
    te = timestep_embedding(t)
    h1 = silu(W["t1_w"] @ te + W["t1_b"])
    ct = W["t2_w"] @ h1 + W["t2_b"]
    pooled = cond.mean(axis=1)                                # [C, cond_dim]
    cvec = ct[None, :] + pooled @ W["pool_w"].T + W["pool_b"]
    mods = silu(cvec) @ W["ada_w"].T + W["ada_b"]
    return cvec, mods


def forward(cfg, W, z, t, cond, cond_index, act_round=identity, trace=None):
    """Velocity for a batch.  z [B, D]; t scalar; cond [C, N_cond, cond_dim];
    cond_index [B] -> condition of each sample.  W: dict of fp64 arrays named as
    WEIGHT_NAMES (block weights stacked on a leading axis).  If `trace` is a dict
    it receives the intermediate tensors of sample 0 for op-by-op comparison."""
    W = {k: np.asarray(v, dtype=np.float64) for k, v in W.items()}
    z = np.asarray(z, dtype=np.float64)
    cond = np.asarray(cond, dtype=np.float64)
    dm = dims(cfg)
    H, nb, n_img = cfg["hidden"], cfg["n_blocks"], dm["n_img"]
    _, mods = conditioning(cfg, W, t, cond)
    cond_emb = act_round(cond) @ W["cond_w"].T + W["cond_b"]       # [C, N_cond, H]
    patches = act_round(patchify(cfg, z))
    out = np.empty_like(z)
    for b in range(z.shape[0]):
        c = int(cond_index[b])
        m = mods[c]
        x = np.concatenate([patches[b] @ W["patch_w"].T + W["patch_b"] + W["pos"], cond_emb[c]], axis=0)
        for k in range(nb):
            sh1, sc1, g1, sh2, sc2, g2 = (m[k * 6 * H + j * H: k * 6 * H + (j + 1) * H] for j in range(6))
            xn = act_round(layer_norm(x) * (1.0 + sc1) + sh1)
            qkv = act_round(xn @ W["qkv_w"][k].T + W["qkv_b"][k])
            a = act_round(attention(qkv[:, :H], qkv[:, H:2 * H], qkv[:, 2 * H:], cfg["n_heads"]))
            x = x + g1 * (a @ W["proj_w"][k].T + W["proj_b"][k])
            xn2 = act_round(layer_norm(x) * (1.0 + sc2) + sh2)
            hid = act_round(gelu_tanh(xn2 @ W["fc1_w"][k].T + W["fc1_b"][k]))
            x = x + g2 * (hid @ W["fc2_w"][k].T + W["fc2_b"][k])
            if trace is not None and b == 0:
                trace.setdefault("x_after_block", []).append(x.copy())
                if k == 0:
                    trace.update(xn=xn, qkv=qkv, attn=a, hid=hid)
        shf, scf = m[nb * 6 * H: nb * 6 * H + H], m[nb * 6 * H + H: nb * 6 * H + 2 * H]
        xf = act_round(layer_norm(x[:n_img]) * (1.0 + scf) + shf)
        o = xf @ W["final_w"].T + W["final_b"]
        out[b] = unpatchify(cfg, o[None])[0]
    return out


def forward_rows(cfg, W, z, t, cond, cond_index, rows, act_round=identity):
    """Velocity patches of selected image tokens for a ONE-block model: returns
    [B, len(rows), patch_dim], the rows `rows` of final_lin's output (before
    unpatchify).  With one block an output token depends on all tokens only through
    the keys and values, so everything after the attention is evaluated on the
    selected rows alone; used where the full forward is too slow on a CPU.
    Pinned against forward() in tests/test_oracle_dit.py."""
    assert cfg["n_blocks"] == 1
    W = {k: np.asarray(v, dtype=np.float64) for k, v in W.items()}
    z = np.asarray(z, dtype=np.float64)
    cond = np.asarray(cond, dtype=np.float64)
    rows = np.asarray(rows)
    dm = dims(cfg)
    H, nh, dh = cfg["hidden"], cfg["n_heads"], dm["d_head"]
    _, mods = conditioning(cfg, W, t, cond)
    cond_emb = act_round(cond) @ W["cond_w"].T + W["cond_b"]
    patches = act_round(patchify(cfg, z))
    out = np.empty((z.shape[0], len(rows), dm["patch_dim"]))
    for b in range(z.shape[0]):
        c = int(cond_index[b])
        m = mods[c]
        x = np.concatenate([patches[b] @ W["patch_w"].T + W["patch_b"] + W["pos"], cond_emb[c]], axis=0)
        sh1, sc1, g1, sh2, sc2, g2 = (m[j * H:(j + 1) * H] for j in range(6))
        xn = act_round(layer_norm(x) * (1.0 + sc1) + sh1)
        kv = act_round(xn @ W["qkv_w"][0][H:].T + W["qkv_b"][0][H:])           # keys and values of all tokens
        q = act_round(xn[rows] @ W["qkv_w"][0][:H].T + W["qkv_b"][0][:H])      # queries of the selected tokens
        a = np.empty((len(rows), H))
        for h in range(nh):
            sl = slice(h * dh, (h + 1) * dh)
            p = softmax_rows(q[:, sl] @ kv[:, :H][:, sl].T / np.sqrt(dh))
            a[:, sl] = p @ kv[:, H:][:, sl]
        a = act_round(a)
        xr = x[rows] + g1 * (a @ W["proj_w"][0].T + W["proj_b"][0])
        xn2 = act_round(layer_norm(xr) * (1.0 + sc2) + sh2)
        hid = act_round(gelu_tanh(xn2 @ W["fc1_w"][0].T + W["fc1_b"][0]))
        xr = xr + g2 * (hid @ W["fc2_w"][0].T + W["fc2_b"][0])
        shf, scf = m[6 * H:7 * H], m[7 * H:8 * H]
        xf = act_round(layer_norm(xr) * (1.0 + scf) + shf)
        out[b] = xf @ W["final_w"].T + W["final_b"]
    return out
