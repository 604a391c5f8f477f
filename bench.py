#!/usr/bin/env python3
"""Benchmark of the BranchGRPO tree-rollout hot path on one MI355X.

One step = one pass of the whole path over one batch of synthetic prompts:
  br_rollout (tree rollout under the behaviour policy) -> br_leaf_reward ->
  br_fuse_advantage -> br_prune -> br_logprob (re-evaluation of the kept edges
  under perturbed weights) -> br_grpo_objective.

Three workload shapes run in one invocation (all synthetic, seeded):
  image        DiT 12 blocks, hidden 1024, 16 heads, latent 16x64x64, 1024+77 tokens, T = 20,
               splits {4,8,12,16}, K = 2, 4 prompts -> 64 leaves
  video        30 blocks, hidden 1536, 12 heads, latent 16x21x60x104, 32760+512 tokens with full
               attention, T = 16, splits {4,8,12}, 1 prompt -> 8 leaves
  image_large  24 blocks, hidden 3072, 24 heads, latent 16x128x128, 4096+512 tokens, T = 16,
               splits {3,6,9,12}, 2 prompts -> 32 leaves                    (the headline)
each with Extreme-b width pruning (b = leaves/4) and 4 seeded dropped depths.  The headline
workload is timed for exactly --steps steps after --warmup warm-up steps; image takes the same
counts (it is cheap), video one warm-up and one timed step (a step is 15-20 s).

Prints ONE JSON line: leaf trajectories/s of the headline workload's whole step, with the roofline
of its dominant kernel (HIP events around every launch inside the timed region), the flat N*T
rollout and the CPU oracle (bounded sample) beside it, and under "workloads" the same figures
for every workload that ran.
"""
import argparse
import gc
import json
import math
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA, data-sheet figure
PEAK_HBM_GBS = 8000.0          # MI355X HBM3E
GEMM_NAMES = {0: "bias", 1: "bias_gelu", 2: "bias_gate_residual", 3: "patch_embed", 4: "bias_f32", 5: "unpatchify"}
TILE_NAMES = {4: "256x256 lds-direct", 5: "128x128 lds-direct",
              6: "256x128 lds-direct", 7: "256x256 persistent stream"}
HEADLINE = "image_large"
ORDER = ("image", "video", "image_large")


# HBM-side traffic per launch, from two rocprofv3 --pmc runs of this file on one workload (FETCH_SIZE,
# then WRITE_SIZE, KiB per dispatch averaged over the launches of one step), each scaled by what the
# same counter reads for a plain 1 GiB device copy; see profiles/hot_kernels_hbm_traffic.md.  Keyed
# by (workload, kernel label); valid only for the kernel sources hashed beside the figures.
TRAFFIC = {
    'image_large|gemm_bf16[bias_gate_residual,256x256 persistent stream]': dict(bytes_per_launch=6612766740, sources=('gemm_bf16_stream.hip', 'gemm_epilogue.h', 'dit.h', 'common.h'), sha1='d08d8047b1b8c4977796a3d75174dee298cd7cee'),
    'image_large|gemm_bf16[bias_gelu,256x256 persistent stream]': dict(bytes_per_launch=9183573064, sources=('gemm_bf16_stream.hip', 'gemm_epilogue.h', 'dit.h', 'common.h'), sha1='d08d8047b1b8c4977796a3d75174dee298cd7cee'),
    'image_large|gemm_bf16[bias,256x256 persistent stream]': dict(bytes_per_launch=7166651914, sources=('gemm_bf16_stream.hip', 'gemm_epilogue.h', 'dit.h', 'common.h'), sha1='d08d8047b1b8c4977796a3d75174dee298cd7cee'),
    'image_large|attn_bf16[d128]': dict(bytes_per_launch=2340423731, sources=('attn_bf16.hip',), sha1='deb7cb68be1bb871d37e9d8f4121d812368a0ff2'),
    'image_large|ln_modulate': dict(bytes_per_launch=1213816248, sources=('dit_kernels.hip', 'common.h'), sha1='123bdb315659e2bc89a1f7bd3071b9530aa623d9'),
    'image|gemm_bf16[bias_gate_residual,256x256 persistent stream]': dict(bytes_per_launch=636361196, sources=('gemm_bf16_stream.hip', 'gemm_epilogue.h', 'dit.h', 'common.h'), sha1='d08d8047b1b8c4977796a3d75174dee298cd7cee'),
    'image|gemm_bf16[bias_gelu,256x256 persistent stream]': dict(bytes_per_launch=654394143, sources=('gemm_bf16_stream.hip', 'gemm_epilogue.h', 'dit.h', 'common.h'), sha1='d08d8047b1b8c4977796a3d75174dee298cd7cee'),
    'image|gemm_bf16[bias,256x256 persistent stream]': dict(bytes_per_launch=502440038, sources=('gemm_bf16_stream.hip', 'gemm_epilogue.h', 'dit.h', 'common.h'), sha1='d08d8047b1b8c4977796a3d75174dee298cd7cee'),
    'image|attn_bf16[d64]': dict(bytes_per_launch=258966323, sources=('attn_bf16.hip',), sha1='deb7cb68be1bb871d37e9d8f4121d812368a0ff2'),
    'image|ln_modulate': dict(bytes_per_launch=193824737, sources=('dit_kernels.hip', 'common.h'), sha1='123bdb315659e2bc89a1f7bd3071b9530aa623d9'),
}


def measured_traffic(workload, label):
    """Counter-measured HBM bytes per launch, or None if there are none for this workload and kernel
    or the kernel sources changed since the counters were taken."""
    t = TRAFFIC.get("%s|%s" % (workload, label))
    if t is None:
        return None
    return round(t["bytes_per_launch"]) if source_hash(t["sources"]) == t["sha1"] else None


def source_hash(files):
    """SHA-1 over the code of the given kernel sources: `//` comments and blank lines do not count."""
    import hashlib
    import re
    h = hashlib.sha1()
    for f in files:
        for line in open(os.path.join(ROOT, "paper_2509_06040_amd", "csrc", f), encoding="utf-8"):
            code = re.sub(r"//.*", "", line).rstrip()
            if code:
                h.update(code.encode() + b"\n")
    return h.hexdigest()


HBM_KERNELS = {200: "sde_step", 201: "logp_eval", 300: "ln_modulate", 301: "adaln_gemv"}


def kernel_label(kid):
    if kid in HBM_KERNELS:
        return HBM_KERNELS[kid]
    if kid < 100:
        return "gemm_bf16[%s,%s]" % (GEMM_NAMES[kid // 8], TILE_NAMES[kid % 8])
    return "attn_bf16[d%d]" % (kid - 100)


def progress(msg):
    print("[bench] " + msg, file=sys.stderr, flush=True)


class Ticker:
    """A progress line on stderr at most every `every` seconds (a long run must not fall silent)."""

    def __init__(self, what, every=30.0):
        self.what, self.every, self.last = what, every, time.perf_counter()

    def tick(self, i, n):
        now = time.perf_counter()
        if now - self.last >= self.every:
            self.last = now
            progress("%s: %d of %d" % (self.what, i, n))


def bench_workload(name, steps, warmup, args, want_flat, want_cpu):
    """Times `steps` steps of workload `name` (after `warmup` untimed ones) and returns its figures."""
    import torch
    from paper_2509_06040_amd import binding as br
    from paper_2509_06040_amd import synth
    dev = "cuda"
    wl = dict(synth.WORKLOADS[name])
    if args.splits is not None:
        wl["splits"] = tuple(int(x) for x in args.splits.split(",") if x != "")
    if args.branch is not None:
        wl["K"] = args.branch
    if args.prompts is not None:
        wl["n_cond"] = args.prompts
    cfg, T, C = wl["model"], wl["T"], wl["n_cond"]
    sz = synth.model_sizes(cfg)
    D, L, H, NB = sz["D"], sz["L"], cfg["hidden"], cfg["n_blocks"]
    latent = (cfg["latent_c"], cfg["latent_t"], cfg["latent_h"], cfg["latent_w"])
    tdt = torch.bfloat16 if cfg["dtype"] == synth.BF16 else torch.float32

    # weights: the small networks are drawn on the host (the same arrays feed the oracle below), the
    # multi-billion-parameter ones on the device
    W = None
    if name in ("image", "tiny"):
        W = synth.make_weights(cfg, 0)
        model = br.Model(cfg, br.upload_weights(cfg, W))
        model2 = br.Model(cfg, br.upload_weights(cfg, synth.perturb_weights(cfg, W, 11, 0.002)))
    else:
        Wd = synth.device_weights(cfg, 0, dev)
        model = br.Model(cfg, Wd)
        model2 = br.Model(cfg, synth.device_perturb_weights(cfg, Wd, 11, 0.002, dev))
        del Wd
    cond_np = synth.cond_tokens(cfg, C)
    cond = torch.from_numpy(cond_np).to(dev).to(tdt)
    sched = synth.schedule(T, wl["kappa"], logp_mean=True)
    tree = br.Tree(T, wl["splits"], wl["K"], n_tree=C).upload()
    n_leaves = C * tree.n_leaves
    n = C * tree.n_nodes
    groups = list(range(C))
    kind = {"linear": br.REWARD_LINEAR, "tanh": br.REWARD_TANH, "video": br.REWARD_VIDEO}[wl["reward"]]
    lam = 0.1 if kind == br.REWARD_VIDEO else 0.0
    w_rew = torch.from_numpy(synth.reward_vector(latent[0] * latent[1] if kind == br.REWARD_VIDEO else D, 7)).to(dev)
    depth_mask = br.depth_mask_seeded(T, min(4, T), synth.DATA_SEED)
    b_extreme = max(1, tree.n_leaves // 4)

    z = torch.empty((n, D), device=dev)
    logp = torch.empty(n, device=dev)
    rew = torch.empty(n_leaves, device=dev)
    rbar, adv = torch.empty(n, device=dev), torch.empty(n, device=dev)
    kept = torch.empty(C * tree.n_edges, dtype=torch.int32, device=dev)
    n_kept = torch.zeros(1, dtype=torch.int32, device=dev)
    logp_new = torch.empty(C * tree.n_edges, device=dev)
    J = torch.empty(1, device=dev)
    ws = torch.empty(br.workspace_bytes(tree, model, n_leaves), dtype=torch.uint8, device=dev)
    rs = torch.empty(max(256, br.reward_scratch_bytes(tree, kind, latent)), dtype=torch.uint8, device=dev)

    phase_ms = {}

    def step(seed, timed):
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)] if timed else None
        if timed:
            ev[0].record()
        br.rollout(tree, model, sched, seed, groups, cond, z, logp, None, ws)
        if timed:
            ev[1].record()
        br.leaf_reward(tree, z, kind, w_rew, lam, latent, rew, rs)
        br.fuse_advantage(tree, rew, logp, 1.0, 1e-8, 0, synth.ADV_CLIP, rbar, adv)
        br.prune(tree, rew, br.PRUNE_EXTREME, b_extreme, depth_mask, kept, n_kept)
        nk = int(n_kept.cpu()[0])                       # the only host round trip of a step
        ids = kept[:nk].cpu().numpy()
        if timed:
            ev[2].record()
        br.logprob(tree, model2, sched, cond, z, ids, logp_new, ws)
        br.grpo_objective(logp_new, logp, adv, kept, nk, synth.CLIP_RANGE, J)
        if timed:
            ev[3].record()
        return ev, nk

    tick = Ticker("%s steps" % name)
    for i in range(warmup):
        step(synth.SAMPLER_SEED + i, False)
        tick.tick(i + 1, warmup + steps)
    torch.cuda.synchronize()
    if not args.no_kernel_events:
        br.profile_enable(True)
        br.profile_read()
    t0 = time.perf_counter()
    evs = []
    for i in range(steps):
        evs.append(step(synth.SAMPLER_SEED + 100 + i, True))
        tick.tick(warmup + i + 1, warmup + steps)     # (the step has just waited for its kept-edge count: no extra stall)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    prof = {}
    if not args.no_kernel_events:
        prof = br.profile_read()
        br.profile_enable(False)
    ms_per_step = (t1 - t0) * 1e3 / steps
    nk = evs[-1][1]
    for pname, a, b in (("rollout", 0, 1), ("reward_fuse_prune", 1, 2), ("logprob_objective", 2, 3)):
        phase_ms[pname] = float(np.mean([e[0][a].elapsed_time(e[0][b]) for e in evs]))
    value = n_leaves / (ms_per_step * 1e-3)
    progress("%s: %d steps, %.1f ms/step" % (name, steps, ms_per_step))

    # ---- roofline of the dominant kernel (largest total time among the instrumented ones)
    kernels = {}
    for kid, (work, ms, cnt) in prof.items():
        mfma = kid not in HBM_KERNELS
        ach = work / (ms * 1e-3) / (1e12 if mfma else 1e9) if ms > 0 else 0.0
        peak = PEAK_BF16_TFLOPS if mfma else PEAK_HBM_GBS
        kernels[kernel_label(kid)] = dict(bound="mfma" if mfma else "hbm", launches=int(cnt), total_ms=round(ms, 3),
                                          avg_us=round(ms * 1e3 / cnt, 2), achieved=round(ach, 2),
                                          unit="TFLOP/s" if mfma else "GB/s", frac=round(ach / peak, 4))
    roofline = None
    if kernels:
        dom = max(kernels, key=lambda k: kernels[k]["total_ms"])
        k = kernels[dom]
        roofline = dict(kernel=dom, bound=k["bound"], achieved=k["achieved"], peak=PEAK_BF16_TFLOPS if k["bound"] == "mfma" else PEAK_HBM_GBS,
                        unit=k["unit"], frac=k["frac"], traffic=measured_traffic(name, dom), avg_launch_us=k["avg_us"], launches=k["launches"])
        mf = [v for v in kernels.values() if v["bound"] == "mfma"]
        tot_flop = sum(v["achieved"] * v["total_ms"] for v in mf)
        tot_ms = sum(v["total_ms"] for v in mf)
        roofline["network_mfma_frac"] = round(tot_flop / tot_ms / PEAK_BF16_TFLOPS, 4) if tot_ms else None

    # ---- the memory-bound and latency-bound calls alone, after the timed region: the fused SDE step on the
    # largest plain frontier and on the last split step, the leaf rewards, fusion + advantages, pruning
    def timed_us(fn, reps=20):
        fn()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) * 1e3 / reps

    def sde_kernel_us(fn, reps=20):
        """Average duration of the fused step kernel alone: a HIP event pair on the launch stream around
        that kernel (the pair itself costs a few microseconds, see `event_pair_floor_us`)."""
        fn()
        torch.cuda.synchronize()
        br.profile_enable(True)
        br.profile_read()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        work, ms, cnt = br.profile_read()[200]
        br.profile_enable(False)
        return ms * 1e3 / cnt

    small_calls = {}
    sde_scratch = torch.empty(max(256, br.sde_scratch_bytes(tree, D)), dtype=torch.uint8, device=dev)
    # what the event pair reads around the same kernel when it has next to nothing to do (one parent, 4 KB)
    ftree = br.Tree(T, (), 1, n_tree=1)
    fz, flp = torch.zeros((ftree.n_nodes, 1024), device=dev), torch.zeros(ftree.n_nodes, device=dev)
    fv = torch.zeros((1, 1024), device=dev)
    floor_us = sde_kernel_us(lambda: br.sde_step(ftree, sched, 5, 0, 1024, fv, fz, flp, sde_scratch))
    small_calls["event_pair_floor_us"] = round(floor_us, 2)
    del ftree, fz, flp, fv
    split_steps = [s_ for s_ in wl["splits"] if s_ < T] if wl["K"] > 1 else []
    sde_steps = [T - 1] + ([max(split_steps)] if split_steps else [])
    for cname, i in zip(("sde_step_largest_frontier", "sde_step_last_split"), sde_steps):
        parents, children = C * int(tree.width[i]), C * int(tree.width[i + 1])
        vpar = torch.randn((parents, D), device=dev)
        call = lambda: br.sde_step(tree, sched, 5, i, D, vpar, z, logp, sde_scratch)
        us, kus = timed_us(call), sde_kernel_us(call)
        nbytes = (2 * parents + children) * 4.0 * D + 4.0 * children          # read z, v per parent; write children
        small_calls[cname] = dict(step=int(i), parents=parents, children=children, D=int(D), call_us=round(us, 2),
                                  kernel_us=round(kus, 2), algorithmic_bytes=int(nbytes),
                                  achieved_GBps=round(nbytes / kus / 1e3, 1),
                                  frac_of_hbm_peak=round(nbytes / kus / 1e3 / PEAK_HBM_GBS, 4))
        del vpar
    us = timed_us(lambda: br.leaf_reward(tree, z, kind, w_rew, lam, latent, rew, rs))
    nbytes = 4.0 * D * n_leaves + 4.0 * D
    small_calls["leaf_reward"] = dict(leaves=n_leaves, us=round(us, 2), algorithmic_bytes=int(nbytes),
                                      achieved_GBps=round(nbytes / us / 1e3, 1),
                                      frac_of_hbm_peak=round(nbytes / us / 1e3 / PEAK_HBM_GBS, 4))
    small_calls["fuse_advantage"] = dict(us=round(timed_us(
        lambda: br.fuse_advantage(tree, rew, logp, 1.0, 1e-8, 0, synth.ADV_CLIP, rbar, adv)), 2), bound="launch latency")
    small_calls["prune"] = dict(us=round(timed_us(
        lambda: br.prune(tree, rew, br.PRUNE_EXTREME, b_extreme, depth_mask, kept, n_kept)), 2), bound="launch latency")
    step(synth.SAMPLER_SEED + 100 + steps - 1, False)     # leave the arena as the last timed step left it

    # ---- model FLOPs of a step (2MNK per GEMM, 4 L^2 H per attention block) / wall time
    fwd_flop = NB * (24.0 * L * H * H + 4.0 * L * L * H) + 4.0 * sz["n_img"] * sz["patch_dim"] * H
    n_eval_roll = C * int(sum(tree.width[:T]))
    par = set()
    for g in (kept[:nk].cpu().numpy() if nk else []):
        cc, nn_ = divmod(int(g), tree.n_nodes)
        par.add(cc * tree.n_nodes + int(tree.parent[nn_]))
    n_eval_lp = len(par)
    step_mfma_util = (n_eval_roll + n_eval_lp) * fwd_flop / (ms_per_step * 1e-3) / (PEAK_BF16_TFLOPS * 1e12)
    rollout_mfma_util = n_eval_roll * fwd_flop / (phase_ms["rollout"] * 1e-3) / (PEAK_BF16_TFLOPS * 1e12)

    # ---- flat N*T sequential rollout on the same GPU, same kernels (K = 1 trees)
    flat = None
    if want_flat:
        ftree = br.Tree(T, (), 1, n_tree=n_leaves)
        fz = torch.empty((n_leaves * ftree.n_nodes, D), device=dev)
        flp = torch.empty(n_leaves * ftree.n_nodes, device=dev)
        fcond = cond.repeat_interleave(tree.n_leaves, dim=0).contiguous()
        fgroups = [c for c in range(C) for _ in range(tree.n_leaves)]     # "init same noise" per prompt
        fws = torch.empty(br.workspace_bytes(ftree, model, n_leaves), dtype=torch.uint8, device=dev)
        cheap = name in ("image", "tiny")
        if cheap:                                                         # a warm-up run where it costs little
            br.rollout(ftree, model, sched, 1, fgroups, fcond, fz, flp, None, fws)
        torch.cuda.synchronize()
        f0 = time.perf_counter()
        reps = 2 if cheap else 1
        for i in range(reps):
            br.rollout(ftree, model, sched, 2 + i, fgroups, fcond, fz, flp, None, fws)
        torch.cuda.synchronize()
        fms = (time.perf_counter() - f0) * 1e3 / reps
        flat = dict(ms=round(fms, 2), leaf_traj_per_s=round(n_leaves / (fms * 1e-3), 3),
                    tree_rollout_ms=round(phase_ms["rollout"], 2),
                    tree_rollout_leaf_traj_per_s=round(n_leaves / (phase_ms["rollout"] * 1e-3), 3),
                    speedup_tree_vs_flat=round(fms / phase_ms["rollout"], 3), network_evals_flat=n_leaves * T,
                    network_evals_tree=n_eval_roll)
        del fz, flp, fws, fcond
        progress("%s: flat rollout %.1f ms" % (name, fms))

    # ---- the CPU oracle on a bounded sample, extrapolated to a step
    cpu = None
    if want_cpu:
        from oracle import dit as odit
        from oracle import philox as ophilox
        from oracle import sde as osde
        threads = os.cpu_count()
        try:
            from threadpoolctl import threadpool_info
            threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [threads])
        except Exception:
            pass
        rnd = odit.round_bf16 if cfg["dtype"] == synth.BF16 else odit.identity
        if W is not None:          # whole network evaluations at full size
            n_sample, ocfg, oW, scale = (3 if name == "image" else 1), cfg, W, 1.0
            what = "%d oracle network evaluations"
        else:                      # one block of the network at full size, times the number of blocks
            ocfg = dict(cfg)
            ocfg["n_blocks"] = 1
            n_sample, oW, scale = 1, synth.make_weights(ocfg, 0), float(NB)
            what = "%d oracle evaluation of ONE of the " + str(NB) + " blocks (with the embedding and final layers; x" + str(NB) + ")"
        zs = synth.random_latents(n_sample, D, 3)
        c0 = time.perf_counter()
        for i in range(n_sample):
            v = odit.forward(ocfg, oW, zs[i:i + 1], float(sched["t"][3 + i]), cond_np, [i % C], act_round=rnd)
        c1 = time.perf_counter()
        mu = osde.drift_mean(zs[0].astype(np.float64), v[0], sched["t"][3], sched["t"][4], sched["sigma"][3])
        _, std = osde.step_coefficients(sched["t"][3], sched["t"][4], sched["sigma"][3])
        xi = ophilox.normals(1, 5, 3, ophilox.TAG_ETA, D)
        osde.transition_logp(mu + std * xi, mu, std, True)
        c2 = time.perf_counter()
        per_eval, per_sde = (c1 - c0) / n_sample * scale, c2 - c1
        est = (n_eval_roll + n_eval_lp) * per_eval + (n - C + nk) * per_sde
        cpu = dict(value=round(n_leaves / est, 6), unit="leaf trajectories/s", cores=int(threads), kind="oracle",
                   sample=(what % n_sample) + " (%.2f s per whole evaluation) + 1 oracle SDE step/log-prob (%.3f s) at "
                          "full size, extrapolated to the %d evaluations and %d transitions of one step"
                          % (per_eval, per_sde, n_eval_roll + n_eval_lp, n - C + nk))
        progress("%s: oracle sample %.1f s" % (name, c2 - c0))

    out = dict(value=round(value, 4), unit="leaf trajectories/s", steps=steps, warmup=warmup,
               ms_per_step=round(ms_per_step, 3),
               dtype="bf16" if cfg["dtype"] == synth.BF16 else "f32",
               config=dict(workload="%s tree: DiT %d blocks hidden %d, L=%d, D=%d, T=%d splits %s K=%d, %d prompts x %d "
                                    "leaves; Extreme-%d width pruning + %d seeded dropped depths, log-prob "
                                    "re-evaluation of %d kept edges under perturbed weights"
                                    % (name, NB, H, L, D, T, list(wl["splits"]), wl["K"], C, tree.n_leaves,
                                       b_extreme, int(depth_mask.sum()), nk),
                           prompts=C, leaves_per_prompt=int(tree.n_leaves), n_nodes=int(tree.n_nodes)),
               phase_ms={k: round(v, 3) for k, v in phase_ms.items()},
               mfma_util_step=round(step_mfma_util, 4), mfma_util_rollout=round(rollout_mfma_util, 4),
               network_evals=dict(rollout=n_eval_roll, logprob=n_eval_lp, flop_per_eval=fwd_flop),
               roofline=roofline, kernels=kernels, small_calls=small_calls, flat_rollout=flat, cpu_baseline=cpu)
    del model, model2, z, ws, cond
    gc.collect()
    torch.cuda.empty_cache()
    return out


OPS = ("gemm_qkv", "gemm_proj", "gemm_fc1", "gemm_fc2", "attention", "ln_modulate", "sde_step")


def run_op(args):
    """One kernel of the network alone, at a workload's shape and a given batch: the target of
    `rocprofv3 --pmc ... -- python3 bench.py --op NAME --workload W --op-batch B` (counter runs want few
    dispatches).  Inputs are N(0, 1) activations and N(0, 0.02) weights."""
    import torch
    from paper_2509_06040_amd import binding as br
    from paper_2509_06040_amd import synth
    dev = "cuda"
    wl = synth.WORKLOADS[args.workload]
    cfg = wl["model"]
    sz = synth.model_sizes(cfg)
    L, H, NH, D = sz["L"], cfg["hidden"], cfg["n_heads"], sz["D"]
    B = args.op_batch or wl["n_cond"] * 2 ** len(wl["splits"])
    M = B * L
    g = torch.Generator(device=dev)
    g.manual_seed(1)
    rnd = lambda *shape: torch.randn(shape, generator=g, device=dev)
    bf = torch.bfloat16
    name = args.op
    if name.startswith("gemm_"):
        N, K, mode = {"gemm_qkv": (3 * H, H, 0), "gemm_proj": (H, H, 2), "gemm_fc1": (4 * H, H, 1), "gemm_fc2": (H, 4 * H, 2)}[name]
        A, W, bias = rnd(M, K).to(bf), (rnd(N, K) * 0.02).to(bf), rnd(N)
        if mode == 2:
            out, mods = rnd(M, N), rnd(wl["n_cond"], N)
            cond = (torch.arange(B, device=dev) % wl["n_cond"]).to(torch.int32)
            call = lambda: br.op_gemm(br.BF16, 2, A, W, bias, out, mods=mods, gate_off=0, cond=cond, L=L)
        else:
            out = torch.empty((M, N), dtype=bf, device=dev)
            call = lambda: br.op_gemm(br.BF16, mode, A, W, bias, out)
        work, unit = 2.0 * M * N * K, "TFLOP/s"
    elif name == "attention":
        # the layout the network's QKV projection writes: q carries log2(e) / sqrt(head dim)
        x = rnd(B, L, 3 * H)
        x[..., :H] *= math.log2(math.e) / math.sqrt(H // NH)
        qkv, out = x.to(bf), torch.empty((B, L, H), dtype=bf, device=dev)
        del x
        call = lambda: br.op_attention(br.BF16, qkv, out, NH, q_prescaled=1)
        work, unit = 4.0 * B * L * L * H, "TFLOP/s"
    elif name == "ln_modulate":
        x, out, mods = rnd(M, H), torch.empty((M, H), dtype=bf, device=dev), rnd(wl["n_cond"], 2 * H)
        cond = (torch.arange(B, device=dev) % wl["n_cond"]).to(torch.int32)
        call = lambda: br.op_ln_modulate(br.BF16, x, out, L, L, mods, 0, H, cond)
        work, unit = 6.0 * M * H, "GB/s"
    else:  # the fused SDE step on the widest frontier
        tree = br.Tree(wl["T"], wl["splits"], wl["K"], n_tree=wl["n_cond"])
        i = wl["T"] - 1
        P = wl["n_cond"] * int(tree.width[i])
        z, lp, v = rnd(wl["n_cond"] * tree.n_nodes, D), torch.empty(wl["n_cond"] * tree.n_nodes, device=dev), rnd(P, D)
        sched = synth.schedule(wl["T"], wl["kappa"])
        scr = torch.empty(max(256, br.sde_scratch_bytes(tree, D)), dtype=torch.uint8, device=dev)
        call = lambda: br.sde_step(tree, sched, 5, i, D, v, z, lp, scr)
        work, unit, B = 12.0 * P * D, "GB/s", P
    call()
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(args.op_reps):
        call()
    b.record()
    torch.cuda.synchronize()
    us = a.elapsed_time(b) * 1e3 / args.op_reps
    if args.copy_calibration:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)                       # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
    print(json.dumps(dict(op=name, workload=args.workload, batch=B, rows=M, launches=args.op_reps + 1, avg_us=round(us, 2),
                          achieved=round(work / us / (1e6 if unit == "TFLOP/s" else 1e3), 2), unit=unit)))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="all", choices=["all", "image", "tiny", "image_large", "video"],
                    help="all: image, video and image_large in one run, image_large being the headline; "
                         "a single name: only that workload, as the headline")
    ap.add_argument("--video-steps", type=int, default=1, help="timed steps of the video workload when it is not the headline")
    ap.add_argument("--splits", default=None, help="comma-separated split steps replacing the workload's (extra shapes: "
                    "the paper's Dense 0,3,6,9 / Mixed 0,4,8,12 / Sparse 0,5,10,15 presets, five splits, ...)")
    ap.add_argument("--branch", type=int, default=None, help="branching factor K replacing the workload's (3 -> 81, 4 -> 256 leaves)")
    ap.add_argument("--prompts", type=int, default=None, help="number of prompts (independent trees) replacing the workload's")
    ap.add_argument("--no-kernel-events", action="store_true", help="do not time single launches in the timed region")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-flat", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 1 GiB device copy (reference for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    ap.add_argument("--op", default=None, choices=OPS, help="run one kernel alone at the shape of --workload (default "
                    "image) and --op-batch samples instead of the benchmark; for counter collection")
    ap.add_argument("--op-batch", type=int, default=0, help="samples in the batch of --op (default: the workload's widest frontier)")
    ap.add_argument("--op-reps", type=int, default=3)
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: the measurement covers one GPU only (conditions are independent trees and would shard "
                 "across GPUs without collectives); run with --gpus 1")

    import torch
    from paper_2509_06040_amd import binding as br
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    br.load()
    if args.op:
        if args.workload == "all":
            args.workload = "image"
        return run_op(args)

    names = ORDER if args.workload == "all" else (args.workload,)
    head = HEADLINE if args.workload == "all" else args.workload
    results = {}
    for name in names:
        is_head = name == head
        if is_head or name == "image":
            steps, warmup = args.steps, args.warmup
        else:                                   # video beside the headline: a step takes 15-20 s
            steps, warmup = args.video_steps, 1
        results[name] = bench_workload(name, steps, warmup, args,
                                       want_flat=not args.no_flat and (is_head or name == "image"),
                                       want_cpu=not args.no_cpu_baseline and is_head)

    if args.copy_calibration:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)                       # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst

    h = results[head]
    out = dict(metric="leaf trajectories/sec (tree vs flat N*T rollout); DiT-fwd MFMA util %", value=h["value"],
               unit="leaf trajectories/s", n_gpus=1, steps=h["steps"], warmup=h["warmup"], ms_per_step=h["ms_per_step"],
               higher_is_better=True, scaling="weak", vs_baseline=None, dtype=h["dtype"], data="synthetic",
               config=h["config"], phase_ms=h["phase_ms"], mfma_util_step=h["mfma_util_step"],
               mfma_util_rollout=h["mfma_util_rollout"], network_evals=h["network_evals"], roofline=h["roofline"],
               kernels=h["kernels"], small_calls=h["small_calls"], flat_rollout=h["flat_rollout"],
               cpu_baseline=h["cpu_baseline"],
               workloads={k: {f: v[f] for f in ("value", "unit", "steps", "warmup", "ms_per_step", "config", "phase_ms",
                                                "mfma_util_step", "mfma_util_rollout", "network_evals", "roofline",
                                                "kernels", "small_calls", "flat_rollout")}
                          for k, v in results.items() if k != head})
    print(json.dumps(out))


if __name__ == "__main__":
    main()
