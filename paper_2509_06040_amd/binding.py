"""Thin ctypes binding over libbranchrollout.so: argument marshalling only.

Every function has the name of the C entry point without the `br_` prefix and
takes torch tensors (device memory) or numpy arrays (host memory) where the C
header says `dev` / `host`.  Nothing is computed here; a missing library is an
error, there is no fallback path.
"""
import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libbranchrollout.so")
_lib = None

F32, BF16 = 0, 1
LOGP_SUM, LOGP_MEAN = 0, 1
PRUNE_NONE, PRUNE_PARENT_TOP1, PRUNE_EXTREME = 0, 1, 2
REWARD_LINEAR, REWARD_TANH, REWARD_VIDEO = 0, 1, 2
W_COUNT = 23
WEIGHT_ORDER = ("patch_w", "patch_b", "pos", "cond_w", "cond_b", "t1_w", "t1_b", "t2_w", "t2_b", "pool_w", "pool_b",
                "ada_w", "ada_b", "qkv_w", "qkv_b", "proj_w", "proj_b", "fc1_w", "fc1_b", "fc2_w", "fc2_b",
                "final_w", "final_b")
_MATRICES = {n for n in WEIGHT_ORDER if n.endswith("_w")}

EXPORTS = (
    "br_last_error", "br_tree_build", "br_tree_info", "br_tree_upload", "br_tree_free", "br_model_create", "br_model_free",
    "br_workspace_bytes", "br_rollout", "br_logprob", "br_fuse_advantage", "br_prune", "br_reward_scratch_bytes",
    "br_leaf_reward", "br_grpo_objective", "br_velocity", "br_sde_scratch_bytes", "br_sde_step", "br_sde_static_scratch_limit",
    "br_sde_step_static", "br_root_noise",
    "br_noise_stream", "br_depth_mask_window", "br_depth_mask_seeded", "br_mix_schedule", "br_fusion_ess", "br_op_gemm", "br_op_attention",
    "br_op_ln_modulate", "br_profile_enable", "br_profile_read",
)


class BranchRolloutError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("libbranchrollout error %d: %s" % (code, msg))
        self.code = code


class ModelCfg(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "n_blocks", "hidden", "n_heads", "mlp_ratio", "latent_c", "latent_t", "latent_h", "latent_w",
        "patch_t", "patch_h", "patch_w", "n_cond_tokens", "cond_dim", "dtype")]


class Sched(C.Structure):
    _fields_ = [("T", C.c_int32), ("t", C.POINTER(C.c_float)), ("sigma", C.POINTER(C.c_float)),
                ("s", C.c_float), ("logp_reduce", C.c_int32)]


def load():
    """Load the built library (build with `python -m paper_2509_06040_amd.build`)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError("%s is missing: build it with `python -m paper_2509_06040_amd.build`" % LIB_PATH)
    lib = C.CDLL(LIB_PATH)
    lib.br_last_error.restype = C.c_char_p
    for name in ("br_workspace_bytes", "br_reward_scratch_bytes", "br_sde_scratch_bytes", "br_sde_static_scratch_limit"):
        getattr(lib, name).restype = C.c_size_t
    lib.br_tree_free.restype = None
    lib.br_model_free.restype = None
    _lib = lib
    return lib


def _check(code):
    if code != 0:
        raise BranchRolloutError(code, load().br_last_error().decode())


def _p(x):
    """Device pointer of a torch tensor (None -> NULL)."""
    if x is None:
        return C.c_void_p(0)
    assert x.is_contiguous(), "tensor must be contiguous"
    return C.c_void_p(x.data_ptr())


def _h(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a, a.ctypes.data_as(C.c_void_p)


def _stream():
    import torch
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


class Tree:
    def __init__(self, T, split_steps, K, n_tree=1):
        lib = load()
        sp, spp = _h(list(split_steps), np.int32)
        self._h = C.c_void_p()
        _check(lib.br_tree_build(C.c_int32(T), spp, C.c_int32(len(sp)), C.c_int32(K), C.c_int32(n_tree),
                                 C.byref(self._h)))
        nn, ne, nl, nt = C.c_int32(), C.c_int32(), C.c_int32(), C.c_int32()
        ptrs = [C.POINTER(C.c_int32)() for _ in range(7)]
        _check(lib.br_tree_info(self._h, C.byref(nn), C.byref(ne), C.byref(nl), C.byref(nt),
                                *[C.byref(p) for p in ptrs]))
        self.T, self.K, self.n_tree = T, K, nt.value
        self.n_nodes, self.n_edges, self.n_leaves = nn.value, ne.value, nl.value
        cp = lambda p, n: np.ctypeslib.as_array(p, shape=(n,)).copy()
        self.width, self.off = cp(ptrs[0], T + 1), cp(ptrs[1], T + 2)
        self.parent, self.depth, self.branch, self.leaf_lo, self.leaf_hi = (cp(p, nn.value) for p in ptrs[2:])

    def upload(self):
        _check(load().br_tree_upload(self._h))
        return self

    def __del__(self):
        if _lib is not None and getattr(self, "_h", None):
            _lib.br_tree_free(self._h)
            self._h = None


class Model:
    """cfg: dict with the fields of br_model_cfg; weights: dict name -> device tensor
    (matrices in the model dtype, biases and `pos` fp32)."""

    def __init__(self, cfg, weights):
        import torch
        lib = load()
        self.cfg = dict(cfg)
        self.c = ModelCfg(**{k: int(cfg[k]) for k, _ in ModelCfg._fields_})
        want = torch.bfloat16 if cfg["dtype"] == BF16 else torch.float32
        self.weights = []
        for name in WEIGHT_ORDER:
            w = weights[name]
            assert w.is_cuda and w.is_contiguous(), name
            assert w.dtype == (want if name in _MATRICES else torch.float32), (name, w.dtype)
            self.weights.append(w)
        arr = (C.c_void_p * W_COUNT)(*[w.data_ptr() for w in self.weights])
        self._h = C.c_void_p()
        _check(lib.br_model_create(C.byref(self.c), arr, C.c_int32(W_COUNT), C.byref(self._h)))
        self.D = cfg["latent_c"] * cfg["latent_t"] * cfg["latent_h"] * cfg["latent_w"]

    def __del__(self):
        if _lib is not None and getattr(self, "_h", None):
            _lib.br_model_free(self._h)
            self._h = None


def upload_weights(cfg, W, device="cuda"):
    """numpy weight dict -> device tensors in the dtypes the library expects."""
    import torch
    out = {}
    for name in WEIGHT_ORDER:
        t = torch.from_numpy(np.ascontiguousarray(W[name], dtype=np.float32)).to(device)
        if cfg["dtype"] == BF16 and name in _MATRICES:
            t = t.to(torch.bfloat16)
        out[name] = t.contiguous()
    return out


def make_sched(sched):
    """dict(t, sigma, s, logp_mean) -> (Sched struct, keep-alive arrays)."""
    t, tp = _h(sched["t"], np.float32)
    sg, sp = _h(sched["sigma"], np.float32)
    s = Sched(len(sg), C.cast(tp, C.POINTER(C.c_float)), C.cast(sp, C.POINTER(C.c_float)), float(sched["s"]),
              LOGP_MEAN if sched["logp_mean"] else LOGP_SUM)
    s._keep = (t, sg)
    return s


def workspace_bytes(tree, model, max_batch):
    return load().br_workspace_bytes(tree._h if tree is not None else C.c_void_p(0), model._h, C.c_int32(max_batch))


def rollout(tree, model, sched, seed, noise_group, cond_tokens, z_nodes, logp_edges, v_nodes, workspace):
    s = make_sched(sched)
    _, gp = _h(noise_group, np.int32)
    _check(load().br_rollout(tree._h, model._h, C.byref(s), C.c_uint64(seed), gp, _p(cond_tokens), _p(z_nodes),
                             _p(logp_edges), _p(v_nodes), _p(workspace), C.c_size_t(workspace.numel() * workspace.element_size()),
                             _stream()))


def logprob(tree, model, sched, cond_tokens, z_nodes, edge_ids, logp_out, workspace):
    s = make_sched(sched)
    e, ep = _h(edge_ids, np.int32)
    _check(load().br_logprob(tree._h, model._h, C.byref(s), _p(cond_tokens), _p(z_nodes), ep, C.c_int32(len(e)),
                             _p(logp_out), _p(workspace), C.c_size_t(workspace.numel() * workspace.element_size()),
                             _stream()))


def fuse_advantage(tree, leaf_rewards, logp_edges, beta, eps, ddof, a_max, rbar_nodes, adv_nodes):
    _check(load().br_fuse_advantage(tree._h, _p(leaf_rewards), _p(logp_edges), C.c_float(beta), C.c_float(eps),
                                    C.c_int32(ddof), C.c_float(a_max), _p(rbar_nodes), _p(adv_nodes), _stream()))


def prune(tree, leaf_rewards, width_mode, b, depth_pruned, kept_edges, n_kept):
    if depth_pruned is None:
        dp = C.c_void_p(0)
    else:
        _keep, dp = _h(depth_pruned, np.uint8)
        assert len(_keep) == tree.T
    _check(load().br_prune(tree._h, _p(leaf_rewards), C.c_int32(width_mode), C.c_int32(b), dp, _p(kept_edges),
                           _p(n_kept), _stream()))


def reward_scratch_bytes(tree, kind, latent):
    return load().br_reward_scratch_bytes(tree._h, C.c_int32(kind), *[C.c_int32(x) for x in latent])


def leaf_reward(tree, z_nodes, kind, w, lam, latent, rewards, scratch):
    _check(load().br_leaf_reward(tree._h, _p(z_nodes), C.c_int32(kind), _p(w), C.c_float(lam),
                                 *[C.c_int32(x) for x in latent], _p(rewards), _p(scratch),
                                 C.c_size_t(scratch.numel() * scratch.element_size()), _stream()))


def grpo_objective(logp_new, logp_old_nodes, adv_nodes, edge_ids, n_edges, clip_eps, J, clipped=None):
    _check(load().br_grpo_objective(_p(logp_new), _p(logp_old_nodes), _p(adv_nodes), _p(edge_ids), C.c_int32(n_edges),
                                    C.c_float(clip_eps), _p(J), _p(clipped), _stream()))


def fusion_ess(tree, logp_edges, beta, ess_nodes):
    _check(load().br_fusion_ess(tree._h, _p(logp_edges), C.c_float(beta), _p(ess_nodes), _stream()))


def velocity(model, z, t, cond_tokens, cond_index, v_out, workspace):
    ci, cp = _h(cond_index, np.int32)
    _check(load().br_velocity(model._h, _p(z), C.c_float(t), _p(cond_tokens), C.c_int32(cond_tokens.shape[0]), cp,
                              C.c_int32(len(ci)), _p(v_out), _p(workspace),
                              C.c_size_t(workspace.numel() * workspace.element_size()), _stream()))


def sde_scratch_bytes(tree, D):
    return load().br_sde_scratch_bytes(tree._h, C.c_int64(D))


def sde_step(tree, sched, seed, step, D, v_parents, z_nodes, logp_edges, scratch):
    s = make_sched(sched)
    _check(load().br_sde_step(tree._h, C.byref(s), C.c_uint64(seed), C.c_int32(step), C.c_int64(D), _p(v_parents),
                              _p(z_nodes), _p(logp_edges), _p(scratch),
                              C.c_size_t(scratch.numel() * scratch.element_size()), _stream()))


def sde_static_scratch_limit():
    return load().br_sde_static_scratch_limit()


def sde_step_static(tree, sched, seed, step, D, v_parents, z_nodes, logp_edges):
    s = make_sched(sched)
    _check(load().br_sde_step_static(tree._h, C.byref(s), C.c_uint64(seed), C.c_int32(step), C.c_int64(D),
                                     _p(v_parents), _p(z_nodes), _p(logp_edges), _stream()))


def root_noise(tree, seed, noise_group, D, z_nodes):
    _, gp = _h(noise_group, np.int32)
    _check(load().br_root_noise(tree._h, C.c_uint64(seed), gp, C.c_int64(D), _p(z_nodes), _stream()))


def noise_stream(seed, node_id, step, tag, n_quads, words, normals):
    _check(load().br_noise_stream(C.c_uint64(seed), C.c_uint32(node_id), C.c_uint32(step), C.c_uint32(tag),
                                  C.c_int64(n_quads), _p(words), _p(normals), _stream()))


def depth_mask_window(T, last_split, window, iteration, every, stop):
    out = np.zeros(T, dtype=np.uint8)
    _check(load().br_depth_mask_window(C.c_int32(T), C.c_int32(last_split), C.c_int32(window), C.c_int32(iteration),
                                       C.c_int32(every), C.c_int32(stop), out.ctypes.data_as(C.c_void_p)))
    return out


def depth_mask_seeded(T, n_drop, seed):
    out = np.zeros(T, dtype=np.uint8)
    _check(load().br_depth_mask_seeded(C.c_int32(T), C.c_int32(n_drop), C.c_uint64(seed),
                                       out.ctypes.data_as(C.c_void_p)))
    return out


def mix_schedule(T, split_steps, window_mask, eta):
    """-> (sigma [T] float32, ode_mask [T] uint8) of the hybrid ODE-SDE schedule."""
    sp = np.ascontiguousarray(split_steps, dtype=np.int32)
    wm = np.ascontiguousarray(window_mask, dtype=np.uint8)
    if wm.shape != (T,):
        raise ValueError("window_mask must have T entries")
    sigma, ode = np.zeros(T, dtype=np.float32), np.zeros(T, dtype=np.uint8)
    _check(load().br_mix_schedule(C.c_int32(T), sp.ctypes.data_as(C.c_void_p) if sp.size else C.c_void_p(0),
                                  C.c_int32(sp.size), wm.ctypes.data_as(C.c_void_p), C.c_float(eta),
                                  sigma.ctypes.data_as(C.c_void_p), ode.ctypes.data_as(C.c_void_p)))
    return sigma, ode


def op_gemm(dtype, epilogue, A, W, bias, out, mods=None, gate_off=0, cond=None, L=1, variant=-1):
    M, K = A.shape
    N = W.shape[0]
    _check(load().br_op_gemm(C.c_int32(dtype), C.c_int32(epilogue), _p(A), C.c_int32(A.stride(0)), _p(W),
                             C.c_int32(W.stride(0)), C.c_int32(M), C.c_int32(N), C.c_int32(K), _p(bias), _p(out),
                             C.c_int32(out.stride(0)), _p(mods), C.c_int32(mods.shape[1] if mods is not None else 0),
                             C.c_int32(gate_off), _p(cond), C.c_int32(L), C.c_int32(variant), _stream()))


def op_attention(dtype, qkv, out, n_heads, q_prescaled=0):
    B, L, H3 = qkv.shape
    _check(load().br_op_attention(C.c_int32(dtype), _p(qkv), _p(out), C.c_int32(B), C.c_int32(L), C.c_int32(n_heads),
                                  C.c_int32(H3 // 3 // n_heads), C.c_int32(q_prescaled), _stream()))


def op_ln_modulate(dtype, x, out, rows_per_sample, L_in, mods, shift_off, scale_off, cond):
    n_rows, H = out.shape
    _check(load().br_op_ln_modulate(C.c_int32(dtype), _p(x), _p(out), C.c_int32(n_rows), C.c_int32(rows_per_sample),
                                    C.c_int32(L_in), C.c_int32(H), _p(mods), C.c_int32(mods.shape[1]),
                                    C.c_int32(shift_off), C.c_int32(scale_off), _p(cond), _stream()))


def profile_enable(on):
    _check(load().br_profile_enable(C.c_int32(1 if on else 0)))


def profile_read(max_ids=64):
    """-> {kernel id: (work, milliseconds, launches)} since the last read."""
    ids = (C.c_int32 * max_ids)()
    work, ms = (C.c_double * max_ids)(), (C.c_double * max_ids)()
    launches = (C.c_int64 * max_ids)()
    n = C.c_int32()
    _check(load().br_profile_read(C.c_int32(max_ids), ids, work, ms, launches, C.byref(n)))
    return {ids[i]: (work[i], ms[i], launches[i]) for i in range(n.value)}
