/*
 * libbranchrollout -- C ABI of the BranchGRPO tree rollout (arXiv 2509.06040)
 * for AMD MI355X (gfx950).
 *
 * Conventions
 *   - "host" / "dev" on every pointer says where the memory lives.  The library
 *     never allocates, frees or keeps caller tensors: weights, latents, outputs
 *     and the workspace are caller-owned device allocations passed as raw
 *     pointers.  Only the opaque handles (br_tree, br_model) are library-owned
 *     and are released by their *_free call.
 *   - Every call validates its arguments on the host before any launch and
 *     returns BR_OK or a negative code; br_last_error() then holds a message
 *     (thread-local, static storage, never freed).
 *   - Device work is enqueued on `stream` (a hipStream_t passed as void*; NULL is
 *     the default stream).  Calls do not synchronise unless stated.
 *   - All arrays are dense, row-major, with the last index fastest.
 *   - Node numbering: level order inside a tree; node (d, j), j in [0, width[d]),
 *     has local id off[d] + j; global id = tree_index * n_nodes + local id.  The
 *     children of (i, j) are (i+1, j*K + b), b in [0, K), when step i is a split
 *     step and (i+1, j) otherwise.  Edges are named by their child node.
 *   - Step i (0-based, i = 0 is the first, noisiest step) is the transition from
 *     depth i to depth i+1 over h_i = t[i] - t[i+1] > 0.
 */
#ifndef BRANCHROLLOUT_H
#define BRANCHROLLOUT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t br_status;
enum {
  BR_OK = 0,
  BR_EINVAL = -1,     /* null pointer, value out of range, inconsistent arguments   */
  BR_ENOMEM = -2,     /* host or device allocation of a handle failed               */
  BR_ESHAPE = -3,     /* a shape the kernels do not support (see br_model_create)    */
  BR_EWORKSPACE = -4, /* workspace smaller than br_workspace_bytes()                 */
  BR_EDEVICE = -5     /* a HIP runtime call failed; message holds the HIP error      */
};

/* Message of the last failing call on this thread ("" if none). */
const char* br_last_error(void);

/* ------------------------------------------------------------------------- *
 * Topology  (Sec. 3.2 "Preliminaries": depth T, width w, branching steps B,
 * branching factor K; Alg. 1, tree-building loop).  Host-only, integer,
 * deterministic; needs no GPU.
 * ------------------------------------------------------------------------- */
typedef struct br_tree br_tree;

/* T >= 1 steps (T <= 1024); split_steps host [n_splits], strictly ascending,
 * each in [0, T); K >= 1 (K == 1: splits ignored); n_tree >= 1 identical trees
 * (one per prompt).  n_tree * n_nodes must fit in int32.  *out is set on
 * success only. */
br_status br_tree_build(int32_t T, const int32_t* split_steps, int32_t n_splits, int32_t K,
                        int32_t n_tree, br_tree** out);

/* Sizes and borrowed host arrays (valid until br_tree_free); any out pointer may
 * be NULL.  width [T+1]; off [T+2] (off[T+1] = n_nodes); parent (root: -1),
 * depth, branch, leaf_lo, leaf_hi: [n_nodes] for one tree; the leaves below node
 * n are leaf indices [leaf_lo[n], leaf_hi[n]). */
br_status br_tree_info(const br_tree* tree, int32_t* n_nodes, int32_t* n_edges, int32_t* n_leaves,
                       int32_t* n_tree, const int32_t** width, const int32_t** off,
                       const int32_t** parent, const int32_t** depth, const int32_t** branch,
                       const int32_t** leaf_lo, const int32_t** leaf_hi);
/* Copies the topology arrays to the current GPU (a few KB, one blocking copy; BR_ENOMEM /
 * BR_EDEVICE on failure).  br_fuse_advantage, br_prune and br_fusion_ess need that copy and
 * make it themselves on their first call for a tree that has none; after br_tree_upload they
 * only enqueue kernels.  Safe to call again. */
br_status br_tree_upload(const br_tree* tree);
void br_tree_free(br_tree* tree);

/* ------------------------------------------------------------------------- *
 * Velocity network.  The paper evaluates a denoiser mu_theta(z_i, t_i) once per
 * tree node (Eq. 2; NFE columns of Table 1) but its backbones are pretrained
 * models; here it is a DiT given entirely by the caller's weights:
 *   tokens = [patch_embed(z) + pos ; cond_embed(c)],  L = N_img + n_cond_tokens
 *   cvec   = t_mlp(sinusoid_256(1000 t)) + pool_lin(mean over condition tokens)
 *   mods   = ada_lin(silu(cvec)): per block (shift1, scale1, gate1, shift2,
 *            scale2, gate2), then (shift, scale) of the final layer, each [hidden]
 *   block:   x += gate1 * proj(attention(LN(x)(1+scale1)+shift1))
 *            x += gate2 * fc2(gelu_tanh(fc1(LN(x)(1+scale2)+shift2)))
 *   v      = unpatchify(final_lin(LN(x_img)(1+scale)+shift))
 * LayerNorm: no affine, eps 1e-6.  Attention: full softmax(QK^T/sqrt(d_h))V over
 * all L tokens; q, k, v are rows [0,H), [H,2H), [2H,3H) of qkv, head h owning
 * columns [h d_h, (h+1) d_h) of each.  Latent element order [C, T, H, W]; token
 * order (t, h, w) raster; patch-vector order (c, dt, dh, dw).
 * ------------------------------------------------------------------------- */
typedef struct {
  int32_t n_blocks, hidden, n_heads, mlp_ratio;
  int32_t latent_c, latent_t, latent_h, latent_w;
  int32_t patch_t, patch_h, patch_w;
  int32_t n_cond_tokens, cond_dim;
  int32_t dtype; /* BR_F32: fp32 weights and activations; BR_BF16: bf16 matrices and
                    GEMM/attention operands, fp32 accumulation and residual stream */
} br_model_cfg;
enum { BR_F32 = 0, BR_BF16 = 1 };

/* Order of weight_ptrs (all dev).  Matrices are [out, in] in the model dtype;
 * biases and `pos` are always fp32.  Per-block tensors are stacked on a leading
 * n_blocks axis.  pd = latent_c*patch_t*patch_h*patch_w, R = mlp_ratio,
 * A = n_blocks*6*hidden + 2*hidden. */
enum {
  BR_W_PATCH_W = 0, /* [H, pd]   */ BR_W_PATCH_B, /* [H]        */ BR_W_POS,    /* [N_img, H] */
  BR_W_COND_W,      /* [H, cd]   */ BR_W_COND_B,  /* [H]        */
  BR_W_T1_W,        /* [H, 256]  */ BR_W_T1_B,    /* [H]        */
  BR_W_T2_W,        /* [H, H]    */ BR_W_T2_B,    /* [H]        */
  BR_W_POOL_W,      /* [H, cd]   */ BR_W_POOL_B,  /* [H]        */
  BR_W_ADA_W,       /* [A, H]    */ BR_W_ADA_B,   /* [A]        */
  BR_W_QKV_W,       /* [N,3H,H]  */ BR_W_QKV_B,   /* [N,3H]     */
  BR_W_PROJ_W,      /* [N,H,H]   */ BR_W_PROJ_B,  /* [N,H]      */
  BR_W_FC1_W,       /* [N,RH,H]  */ BR_W_FC1_B,   /* [N,RH]     */
  BR_W_FC2_W,       /* [N,H,RH]  */ BR_W_FC2_B,   /* [N,H]      */
  BR_W_FINAL_W,     /* [pd, H]   */ BR_W_FINAL_B, /* [pd]       */
  BR_W_COUNT
};

typedef struct br_model br_model;

/* Records the configuration and the BR_W_COUNT device pointers (not copied; they
 * must stay valid and 16-byte aligned while the model is used).
 * BR_ESHAPE unless: hidden % n_heads == 0; latent dims divisible by the patch;
 * D = latent_c*latent_t*latent_h*latent_w divisible by 4; hidden % 8 == 0,
 * cond_dim % 8 == 0, pd % 4 == 0; head dim in
 * {16, 32, 64, 128} for BR_F32; for BR_BF16 additionally head dim in {64, 128},
 * hidden % 64 == 0, cond_dim % 64 == 0 and pd % 64 == 0. */
br_status br_model_create(const br_model_cfg* cfg, const void* const* weight_ptrs, int32_t n_ptrs,
                          br_model** out);
void br_model_free(br_model* model);

/* Sampler schedule (App. B.1: reverse grid t_0 > t_1 > ... > t_T, h_i = t_i -
 * t_{i+1}; Eq. 2: branch correlation s).  Caller-owned host memory. */
typedef struct {
  int32_t T;
  const float* t;     /* host [T+1], strictly decreasing, 0 < t[i] <= 1 for i < T, t[T] >= 0 */
  const float* sigma; /* host [T], >= 0: diffusion coefficient eps_t g_t of Eq. 1 on step i;
                         0 makes step i a deterministic (ODE) step without log-prob       */
  float s;            /* >= 0; xi_b = (xi_0 + s eta_b)/sqrt(1+s^2)                         */
  int32_t logp_reduce; /* BR_LOGP_SUM: log-density; BR_LOGP_MEAN: divided by D            */
} br_sched;
enum { BR_LOGP_SUM = 0, BR_LOGP_MEAN = 1 };

/* Bytes of workspace br_rollout / br_logprob / br_velocity need when at most
 * max_batch samples go through the network at once (larger frontiers are
 * processed in chunks).  tree may be NULL for br_velocity (then n_tree is taken
 * as max_batch).  Returns 0 on invalid arguments. */
size_t br_workspace_bytes(const br_tree* tree, const br_model* model, int32_t max_batch);

/* ------------------------------------------------------------------------- *
 * The five calls.
 * ------------------------------------------------------------------------- */

/* Tree rollout under the behaviour policy (Alg. 1, tree-building loop; Eq. 2;
 * App. B.1).  Root of tree c: z_0 ~ N(0, I) drawn from noise stream
 * (seed, noise_group[c]); trees with equal group share z_0.  For every step i
 * the depth-i frontier of all trees is batched through the network once
 * (one evaluation per parent), then every child c of parent p gets
 *   mu   = z_p - h_i v_p - h_i sigma_i^2/(2 t_i) (z_p + (1 - t_i) v_p)
 *   z_c  = mu + sigma_i sqrt(h_i) xi_c
 *   xi_c = eta_c at a non-split step, (xi_0(p) + s eta_c)/sqrt(1+s^2) at a split
 *   logp_c = -|xi_c|^2/2 - D ln(sigma_i sqrt(h_i)) - D/2 ln(2 pi)   (/D if MEAN)
 * with eta, xi_0 standard normals from Philox4x32-10 keyed by seed, counter
 * (element/4, global node id of child resp. parent, i, stream tag), Box-Muller.
 *   noise_group  host [n_tree]
 *   cond_tokens  dev  [n_tree, n_cond_tokens, cond_dim], model dtype
 *   z_nodes      dev out [n_tree*n_nodes, D] fp32
 *   logp_edges   dev out [n_tree*n_nodes] fp32, indexed by child; roots and
 *                sigma = 0 edges get 0
 *   v_nodes      dev out [n_tree*n_nodes, D] fp32 or NULL: velocity at every
 *                non-leaf node (leaf rows are not written)
 * Asynchronous; outputs are complete when `stream` reaches this point. */
br_status br_rollout(const br_tree* tree, const br_model* model, const br_sched* sched, uint64_t seed,
                     const int32_t* noise_group, const void* cond_tokens, float* z_nodes,
                     float* logp_edges, float* v_nodes, void* workspace, size_t workspace_bytes,
                     void* stream);

/* Log-density of stored transitions under another policy (numerator of rho_e,
 * Eq. 5): for edge e with child c = edge_ids[e], parent p, step i = depth(c)-1:
 *   logp_out[e] = -|z_c - mu'|^2/(2 sigma_i^2 h_i) - D ln(sigma_i sqrt(h_i)) - D/2 ln(2 pi)
 * with mu' from the model's velocity at the stored z_p (/D if MEAN; 0 when
 * sigma_i = 0).  Siblings share one network evaluation of their parent, and
 * parents of different steps are batched into one network launch (the network
 * takes a time per sample group), so sparse kept-edge sets still fill the batch.
 *   edge_ids  host [n_edges], strictly ascending global child ids, none a root
 *   logp_out  dev out [n_edges]
 * Asynchronous.  The launch plan built from edge_ids travels through a pinned staging buffer of the
 * tree handle (allocated on first use); a second call on the same tree first waits, on the host, until
 * the previous call's plan has left that buffer. */
br_status br_logprob(const br_tree* tree, const br_model* model, const br_sched* sched,
                     const void* cond_tokens, const float* z_nodes, const int32_t* edge_ids,
                     int32_t n_edges, float* logp_out, void* workspace, size_t workspace_bytes,
                     void* stream);

/* Reward fusion (Eq. 3) and depth-wise normalisation (Eq. 4).
 *   rbar(n) = sum_{l in L(n)} softmax_l(beta s_l) r_l, s_l = sum of logp_edges on
 *   the path n -> l; A(n) = (rbar(n) - mean_d)/(std_d + eps) over the nodes of
 *   n's depth in its tree (std with divisor width_d - ddof; a depth with
 *   width_d <= ddof, or with std_d + eps == 0, gets A = 0); clipped to
 *   [-a_max, a_max] when a_max > 0.  An edge's advantage is its child's.
 *   leaf_rewards dev [n_tree*w]; logp_edges dev [n_tree*n_nodes];
 *   rbar_nodes, adv_nodes dev out [n_tree*n_nodes].  ddof in {0, 1}. */
br_status br_fuse_advantage(const br_tree* tree, const float* leaf_rewards, const float* logp_edges,
                            float beta, float eps, int32_t ddof, float a_max, float* rbar_nodes,
                            float* adv_nodes, void* stream);

/* Width and depth pruning (Sec. 3.4): which edges take part in the update.
 *   width_mode BR_PRUNE_NONE; BR_PRUNE_PARENT_TOP1: of the children of each
 *   parent at the last split step keep the one with the highest reward (tie:
 *   lowest branch index); BR_PRUNE_EXTREME: per tree keep the b lowest and the b
 *   highest leaves in the order (reward, leaf index) (2b >= w keeps all).
 *   depth_pruned host [T] or NULL: nonzero drops every edge of that step.
 * Edge (p -> c) is kept iff c has a kept leaf below it (or is one) and step
 * depth(c)-1 is not dropped.  Rewards must be finite.
 *   leaf_rewards dev [n_tree*w]
 *   kept_edges   dev out [n_tree*n_edges]: ascending global child ids
 *   n_kept       dev out [1] */
enum { BR_PRUNE_NONE = 0, BR_PRUNE_PARENT_TOP1 = 1, BR_PRUNE_EXTREME = 2 };
br_status br_prune(const br_tree* tree, const float* leaf_rewards, int32_t width_mode, int32_t b,
                   const uint8_t* depth_pruned, int32_t* kept_edges, int32_t* n_kept, void* stream);

/* ------------------------------------------------------------------------- *
 * Around the five calls.
 * ------------------------------------------------------------------------- */

/* Synthetic leaf rewards standing in for the reward models of Alg. 1 ("evaluate
 * rewards for leaves").  z_T is the leaf latent of z_nodes.
 *   BR_REWARD_LINEAR  r = <w, z_T>/sqrt(D)                w dev [D]
 *   BR_REWARD_TANH    r = tanh(<w, z_T>/sqrt(D))           w dev [D]
 *   BR_REWARD_VIDEO   m[f,c] = mean over (h,w) of channel c, frame f;
 *                     r = sum w[f,c] m[f,c]/sqrt(F C) - lam/(F-1) sum_f |m[f+1]-m[f]|^2
 *                     w dev [F, C]; latent dims from the four size arguments
 *   rewards dev out [n_tree*w].  For LINEAR/TANH only the product of the four
 *   size arguments (= D) matters.  scratch dev: br_reward_scratch_bytes() bytes
 *   of partial sums (two deterministic stages, no atomics). */
enum { BR_REWARD_LINEAR = 0, BR_REWARD_TANH = 1, BR_REWARD_VIDEO = 2 };
size_t br_reward_scratch_bytes(const br_tree* tree, int32_t kind, int32_t latent_c, int32_t latent_t,
                               int32_t latent_h, int32_t latent_w);
br_status br_leaf_reward(const br_tree* tree, const float* z_nodes, int32_t kind, const float* w,
                         float lam, int32_t latent_c, int32_t latent_t, int32_t latent_h,
                         int32_t latent_w, float* rewards, void* scratch, size_t scratch_bytes,
                         void* stream);

/* Clipped GRPO objective value over a set of edges (Eq. 5):
 *   J = 1/n sum_e min(rho_e A_e, clip(rho_e, 1-clip_eps, 1+clip_eps) A_e),
 *   rho_e = exp(logp_new[e] - logp_old_nodes[edge_ids[e]]), A_e = adv_nodes[edge_ids[e]].
 *   edge_ids dev [n_edges]; logp_new dev [n_edges]; J dev out [1] (0 if n_edges = 0);
 *   clipped dev out [n_edges] or NULL: 1 where the clipped term is the smaller one (the edge
 *   then contributes no gradient), else 0. */
br_status br_grpo_objective(const float* logp_new, const float* logp_old_nodes, const float* adv_nodes,
                            const int32_t* edge_ids, int32_t n_edges, float clip_eps, float* J,
                            uint8_t* clipped, void* stream);

/* Effective sample size of the fusion weights (appendix on the self-normalised importance
 * sampling view of Eq. 3): ESS(n) = (sum_l w_l)^2 / sum_l w_l^2 over the leaves l under node n
 * with the weights of Eq. 3 (1 for a leaf, the number of leaves under n for uniform weights).
 *   logp_edges dev [n_tree*n_nodes]; ess_nodes dev out [n_tree*n_nodes]. */
br_status br_fusion_ess(const br_tree* tree, const float* logp_edges, float beta, float* ess_nodes,
                        void* stream);

/* Velocity of a batch at one time (the network alone; used for teacher-forced
 * checks).  z dev [B, D] fp32; cond_index host [B] -> row of cond_tokens
 * (dev [n_cond, n_cond_tokens, cond_dim]); v_out dev [B, D] fp32.
 * Asynchronous (cond_index travels through a pinned staging buffer of the library, as in br_logprob). */
br_status br_velocity(const br_model* model, const float* z, float t, const void* cond_tokens,
                      int32_t n_cond, const int32_t* cond_index, int32_t B, float* v_out,
                      void* workspace, size_t workspace_bytes, void* stream);

/* One SDE step of the rollout with a caller-given velocity (the fused
 * step/noise/log-prob/expand kernel alone): advances the depth-`step` frontier
 * stored in z_nodes to depth step+1.  v_parents dev [n_tree*width[step], D],
 * row = tree*width[step] + j.  scratch dev, 8-byte aligned: br_sde_scratch_bytes() bytes (one 64-bit
 * word per leaf, in which the blocks working on a child accumulate its log-prob; contents on entry
 * do not matter). */
size_t br_sde_scratch_bytes(const br_tree* tree, int64_t D);
br_status br_sde_step(const br_tree* tree, const br_sched* sched, uint64_t seed, int32_t step,
                      int64_t D, const float* v_parents, float* z_nodes, float* logp_edges,
                      void* scratch, size_t scratch_bytes, void* stream);

/* br_sde_step for callers that cannot allocate device memory (code under HIP graph capture,
 * serving loops, harnesses that forbid hipMalloc): same arguments and results, but the scratch
 * is an array built into the library (one copy per GPU, held until the process ends) and the
 * call itself allocates nothing.  BR_EWORKSPACE when br_sde_scratch_bytes(tree, D) exceeds
 * br_sde_static_scratch_limit() (64 KiB = 8192 leaves over all trees).  All calls
 * on one GPU share that array: calls that overlap on one GPU (different streams or threads)
 * race; calls on one stream are safe. */
size_t br_sde_static_scratch_limit(void);
br_status br_sde_step_static(const br_tree* tree, const br_sched* sched, uint64_t seed, int32_t step,
                             int64_t D, const float* v_parents, float* z_nodes, float* logp_edges,
                             void* stream);

/* Root latents alone: z_nodes rows of all roots <- N(0, I) of (seed, noise_group). */
br_status br_root_noise(const br_tree* tree, uint64_t seed, const int32_t* noise_group, int64_t D,
                        float* z_nodes, void* stream);

/* Raw generator output for checks: words dev out [n_quads, 4] uint32 of counter
 * (q, node_id, step, tag); normals dev out [4*n_quads] fp32 (either may be NULL). */
br_status br_noise_stream(uint64_t seed, uint32_t node_id, uint32_t step, uint32_t tag,
                          int64_t n_quads, uint32_t* words, float* normals, void* stream);

/* Depth-pruning masks (host).  Window (Sec. 3.4 / Sec. 4.4): steps
 * [start, start+window) with start = min(last_split + iter/every, stop - window),
 * clamped to >= 0.  Seeded subset: the n_drop steps with the smallest
 * (Philox word 0 of counter (0, 0, step, 3), step).  mask_out host [T]. */
br_status br_depth_mask_window(int32_t T, int32_t last_split, int32_t window, int32_t iter,
                               int32_t every, int32_t stop, uint8_t* mask_out);
br_status br_depth_mask_seeded(int32_t T, int32_t n_drop, uint64_t seed, uint8_t* mask_out);

/* Hybrid ODE-SDE schedule (ablation "Hybrid ODE-SDE"): every split step stays an SDE step, the
 * steps of a sliding window (window_mask[i] != 0, e.g. from br_depth_mask_window) too, all
 * other steps become deterministic.  sigma_out[i] = eta on SDE steps, 0 on ODE steps;
 * ode_mask_out[i] = 1 on ODE steps -- OR it into the depth mask of br_prune so that the edges
 * of ODE steps, which carry no log-probability, stay out of the update.  Host memory only. */
br_status br_mix_schedule(int32_t T, const int32_t* split_steps, int32_t n_splits, const uint8_t* window_mask,
                          float eta, float* sigma_out, uint8_t* ode_mask_out);

#ifdef __cplusplus
}
#endif
#endif /* BRANCHROLLOUT_H */
