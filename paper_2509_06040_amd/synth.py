"""Seeded synthetic inputs shaped like the paper's image and video workloads.

Only input generation lives here: model configurations, random weights,
condition tokens, time grids, noise scales, reward vectors and perturbed
weights.  None of the method's arithmetic (network, SDE step, noise, fusion,
pruning) is in this module; both the GPU tests and the CPU checker are fed the
arrays produced here.

The paper trains FLUX.1-Dev at 720x720 with T = 20, K = 2, 16 leaves (Sec. 4.2)
and Wan2.1-1.3B video (Sec. 4.6); neither the weights nor the prompt sets are
available, so the shapes are kept and the contents replaced by seeded noise.
"""
import numpy as np

F32, BF16 = 0, 1

_MODEL_KEYS = ("n_blocks", "hidden", "n_heads", "mlp_ratio", "latent_c", "latent_t", "latent_h",
               "latent_w", "patch_t", "patch_h", "patch_w", "n_cond_tokens", "cond_dim", "dtype")


def model_cfg(n_blocks, hidden, n_heads, latent, patch, n_cond_tokens, dtype, mlp_ratio=4):
    c, t, h, w = latent
    pt, ph, pw = patch
    return dict(n_blocks=n_blocks, hidden=hidden, n_heads=n_heads, mlp_ratio=mlp_ratio,
                latent_c=c, latent_t=t, latent_h=h, latent_w=w, patch_t=pt, patch_h=ph, patch_w=pw,
                n_cond_tokens=n_cond_tokens, cond_dim=hidden, dtype=dtype)


# name -> (model, T, split steps, K, n_cond, time-shift kappa, reward kind)
WORKLOADS = {
    "tiny": dict(model=model_cfg(2, 64, 4, (4, 1, 8, 8), (1, 2, 2), 8, F32),
                 T=8, splits=(2, 4, 6), K=2, n_cond=1, kappa=1.0, reward="linear"),
    "image": dict(model=model_cfg(12, 1024, 16, (16, 1, 64, 64), (1, 2, 2), 77, BF16),
                  T=20, splits=(4, 8, 12, 16), K=2, n_cond=4, kappa=3.0, reward="tanh"),
    "image_large": dict(model=model_cfg(24, 3072, 24, (16, 1, 128, 128), (1, 2, 2), 512, BF16),
                        T=16, splits=(3, 6, 9, 12), K=2, n_cond=2, kappa=3.0, reward="tanh"),
    "video": dict(model=model_cfg(30, 1536, 12, (16, 21, 60, 104), (1, 2, 2), 512, BF16),
                  T=16, splits=(4, 8, 12), K=2, n_cond=1, kappa=3.0, reward="video"),
}
SAMPLER_SEED = 1223627   # Table 2 "Sampler seed"
DATA_SEED = 42           # Table 2 "Random seed"
ETA = 0.3                # Table 2 "Eta"
BRANCH_S = 4.0           # Sec. 4.4: best branch correlation
ADV_CLIP = 5.0           # Table 2 "Adv. clip max"
CLIP_RANGE = 1e-4        # Table 2 "Clip range"


def model_sizes(cfg):
    gt, gh, gw = cfg["latent_t"] // cfg["patch_t"], cfg["latent_h"] // cfg["patch_h"], cfg["latent_w"] // cfg["patch_w"]
    n_img = gt * gh * gw
    pd = cfg["latent_c"] * cfg["patch_t"] * cfg["patch_h"] * cfg["patch_w"]
    D = cfg["latent_c"] * cfg["latent_t"] * cfg["latent_h"] * cfg["latent_w"]
    return dict(n_img=n_img, patch_dim=pd, D=D, L=n_img + cfg["n_cond_tokens"])


def weight_shapes(cfg):
    """Ordered (name, shape, is_matrix).  Matrices are [out, in] row-major and are
    stored in the model dtype; biases and the positional table are always fp32."""
    H, N, R = cfg["hidden"], cfg["n_blocks"], cfg["mlp_ratio"]
    sz = model_sizes(cfg)
    pd, cd = sz["patch_dim"], cfg["cond_dim"]
    return [
        ("patch_w", (H, pd), True), ("patch_b", (H,), False), ("pos", (sz["n_img"], H), False),
        ("cond_w", (H, cd), True), ("cond_b", (H,), False),
        ("t1_w", (H, 256), True), ("t1_b", (H,), False), ("t2_w", (H, H), True), ("t2_b", (H,), False),
        ("pool_w", (H, cd), True), ("pool_b", (H,), False),
        ("ada_w", (N * 6 * H + 2 * H, H), True), ("ada_b", (N * 6 * H + 2 * H,), False),
        ("qkv_w", (N, 3 * H, H), True), ("qkv_b", (N, 3 * H), False),
        ("proj_w", (N, H, H), True), ("proj_b", (N, H), False),
        ("fc1_w", (N, R * H, H), True), ("fc1_b", (N, R * H), False),
        ("fc2_w", (N, H, R * H), True), ("fc2_b", (N, H), False),
        ("final_w", (pd, H), True), ("final_b", (pd,), False),
    ]


def to_bf16_bits(a):
    """float32 array -> uint16 bfloat16 bit patterns (round to nearest even; finite inputs)."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = (u >> np.uint32(16)) & np.uint32(1)
    r += np.uint32(0x7FFF)
    r += u
    r >>= np.uint32(16)
    return r.astype(np.uint16)


def from_bf16_bits(b):
    return (np.asarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def positional_table(n_img, H):
    """Fixed 1-D sin-cos table over the token index (an input like the weights)."""
    pos = np.arange(n_img, dtype=np.float64)[:, None]
    k = np.arange(H // 2, dtype=np.float64)[None, :]
    ang = pos / (10000.0 ** (2.0 * k / H))
    out = np.zeros((n_img, H), dtype=np.float32)
    out[:, 0:2 * (H // 2):2] = np.sin(ang)
    out[:, 1:2 * (H // 2):2] = np.cos(ang)
    return out


def make_weights(cfg, seed=0, std=0.02):
    """dict name -> float32 array.  For a bf16 model the matrices hold values that
    are exactly representable in bfloat16, so both sides start from the same bits."""
    rng = np.random.default_rng(seed)
    W = {}
    for name, shape, is_mat in weight_shapes(cfg):
        if name == "pos":
            W[name] = positional_table(*shape)
            continue
        a = (rng.standard_normal(shape, dtype=np.float32) * np.float32(std))
        if is_mat and cfg["dtype"] == BF16:
            a = from_bf16_bits(to_bf16_bits(a))
        W[name] = a
    return W


def perturb_weights(cfg, W, seed, std):
    """theta' = theta + N(0, std^2) on every matrix and bias (rounded to bf16 for
    bf16 matrices): the updated policy whose log-probs are re-evaluated."""
    rng = np.random.default_rng(seed)
    out = {}
    for name, shape, is_mat in weight_shapes(cfg):
        if name == "pos":
            out[name] = W[name]
            continue
        a = W[name] + rng.standard_normal(shape, dtype=np.float32) * np.float32(std)
        if is_mat and cfg["dtype"] == BF16:
            a = from_bf16_bits(to_bf16_bits(a))
        out[name] = a.astype(np.float32)
    return out


def cond_tokens(cfg, n_cond, seed=DATA_SEED):
    """[n_cond, n_cond_tokens, cond_dim] ~ N(0, 1), float32 (bf16-representable
    for a bf16 model)."""
    rng = np.random.default_rng(seed)
    a = rng.standard_normal((n_cond, cfg["n_cond_tokens"], cfg["cond_dim"]), dtype=np.float32)
    if cfg["dtype"] == BF16:
        a = from_bf16_bits(to_bf16_bits(a))
    return a


def time_grid(T, kappa):
    """t_0 = 1 > ... > t_T = 0 with the resolution shift t = kappa u / (1 + (kappa-1) u)."""
    u = 1.0 - np.arange(T + 1, dtype=np.float64) / T
    return (kappa * u / (1.0 + (kappa - 1.0) * u)).astype(np.float32)


def schedule(T, kappa, eta=ETA, s=BRANCH_S, logp_mean=True, ode_steps=()):
    sigma = np.full(T, eta, dtype=np.float32)
    for i in ode_steps:
        sigma[i] = 0.0
    return dict(T=T, t=time_grid(T, kappa), sigma=sigma, s=float(s), logp_mean=bool(logp_mean))


def reward_vector(n, seed):
    return np.random.default_rng(seed).standard_normal(n, dtype=np.float32)


def random_latents(n, D, seed):
    return np.random.default_rng(seed).standard_normal((n, D), dtype=np.float32)


def device_weights(cfg, seed, device="cuda", std=0.02):
    """The distribution of make_weights drawn on the device with a seeded torch generator, in the
    dtypes the library takes (matrices in the model dtype, biases and `pos` fp32): for networks
    whose billions of parameters take minutes to draw on the host.  Not the numbers of
    make_weights; used where nothing is compared with a host copy of the same weights."""
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    mat = torch.bfloat16 if cfg["dtype"] == BF16 else torch.float32
    W = {}
    for name, shape, is_mat in weight_shapes(cfg):
        if name == "pos":
            W[name] = torch.from_numpy(positional_table(*shape)).to(device)
            continue
        a = torch.randn(shape, generator=g, device=device, dtype=torch.float32) * std
        W[name] = a.to(mat).contiguous() if is_mat else a.contiguous()
    return W


def device_perturb_weights(cfg, W, seed, std, device="cuda"):
    """theta' = theta + N(0, std^2) on every matrix and bias of a device_weights dict."""
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    out = {}
    for name, shape, is_mat in weight_shapes(cfg):
        if name == "pos":
            out[name] = W[name]
            continue
        a = W[name].float() + torch.randn(shape, generator=g, device=device, dtype=torch.float32) * std
        out[name] = a.to(W[name].dtype).contiguous()
    return out
