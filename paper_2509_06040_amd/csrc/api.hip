// C-ABI entry points and the frontier scheduler: per step, all nodes of one depth
// (over all trees) go through the network as one batch, so a prefix shared by
// several leaves is evaluated once (Sec. 1; Alg. 1, tree-building loop).
#include <algorithm>
#include <cstring>
#include <cmath>

#include "common.h"
#include "dit.h"
#include "kernels.h"

using namespace br;

namespace {

br_status check_sched(const br_tree* tree, const br_sched* s, const char* who) {
  BR_REQUIRE(s && s->t && s->sigma, BR_EINVAL, std::string(who) + ": schedule or its arrays are NULL");
  BR_REQUIRE(s->T == tree->T, BR_EINVAL, std::string(who) + ": schedule T differs from the tree's");
  for (int i = 0; i < s->T; ++i) {
    BR_REQUIRE(std::isfinite(s->t[i]) && s->t[i] > 0.f && s->t[i] > s->t[i + 1], BR_EINVAL,
               std::string(who) + ": t must be strictly decreasing and positive before the last entry");
    BR_REQUIRE(std::isfinite(s->sigma[i]) && s->sigma[i] >= 0.f, BR_EINVAL, std::string(who) + ": sigma must be >= 0");
  }
  BR_REQUIRE(std::isfinite(s->t[s->T]) && s->t[s->T] >= 0.f, BR_EINVAL, std::string(who) + ": t[T] must be >= 0");
  BR_REQUIRE(std::isfinite(s->s) && s->s >= 0.f, BR_EINVAL, std::string(who) + ": branch correlation s must be >= 0");
  BR_REQUIRE(s->logp_reduce == BR_LOGP_SUM || s->logp_reduce == BR_LOGP_MEAN, BR_EINVAL,
             std::string(who) + ": unknown logp_reduce");
  return BR_OK;
}

int max_frontier(const br_tree* t) {  // widest batch that ever goes through the network
  int w = 1;
  for (int i = 0; i < t->T; ++i) w = std::max(w, t->width[i]);
  return w * t->n_tree;
}

struct Sizes {
  int n_cond;
  long long v_rows, partial_floats, plan_ints;
};

Sizes sizes_for(const br_tree* t, const br_model* m, int max_batch) {
  Sizes s;
  if (t) {
    s.n_cond = t->n_tree;
    s.v_rows = max_frontier(t);
    s.partial_floats = (long long)sde_scratch_floats((long long)t->n_tree * t->n_leaves, m->D);
    s.plan_ints = 9LL * t->n_tree * t->n_nodes + max_batch;
  } else {
    s.n_cond = max_batch;
    s.v_rows = 0;
    s.partial_floats = 0;
    s.plan_ints = max_batch;
  }
  return s;
}

// Largest batch (<= want) whose plan fits into `bytes`; 0 if none.
int fit_batch(const br_tree* t, const br_model* m, int want, size_t bytes, int n_cond_override) {
  int lo = 0, hi = want;
  while (lo < hi) {
    const int mid = (lo + hi + 1) / 2;
    Sizes s = sizes_for(t, m, t ? mid : want);
    if (n_cond_override > 0) s.n_cond = n_cond_override;
    if (plan_workspace(m, s.n_cond, mid, s.v_rows, s.partial_floats, s.plan_ints, nullptr, nullptr) <= bytes) lo = mid;
    else hi = mid - 1;
  }
  return lo;
}

}  // namespace

extern "C" size_t br_workspace_bytes(const br_tree* tree, const br_model* model, int32_t max_batch) {
  if (!model || max_batch < 1) return 0;
  const Sizes s = sizes_for(tree, model, max_batch);
  return plan_workspace(model, s.n_cond, max_batch, s.v_rows, s.partial_floats, s.plan_ints, nullptr, nullptr);
}

extern "C" br_status br_rollout(const br_tree* tree, const br_model* model, const br_sched* sched, uint64_t seed,
                                const int32_t* noise_group, const void* cond_tokens, float* z_nodes, float* logp_edges,
                                float* v_nodes, void* workspace, size_t workspace_bytes, void* stream) {
  BR_REQUIRE(tree && model && noise_group && cond_tokens && z_nodes && logp_edges && workspace, BR_EINVAL,
             "br_rollout: NULL argument");
  br_status s;
  if ((s = check_sched(tree, sched, "br_rollout")) != BR_OK) return s;
  hipStream_t st = (hipStream_t)stream;
  const int mb = fit_batch(tree, model, max_frontier(tree), workspace_bytes, 0);
  BR_REQUIRE(mb >= 1, BR_EWORKSPACE, "br_rollout: workspace too small (see br_workspace_bytes)");
  FwdBuffers fb;
  const Sizes sz = sizes_for(tree, model, mb);
  plan_workspace(model, sz.n_cond, mb, sz.v_rows, sz.partial_floats, sz.plan_ints, &fb, workspace);
  const long long D = model->D;
  if ((s = launch_fill_zero(logp_edges, (long long)tree->n_tree * tree->n_nodes, st)) != BR_OK) return s;
  if ((s = launch_root_noise(tree, seed, noise_group, D, z_nodes, st)) != BR_OK) return s;
  if ((s = launch_sde_scratch_reset(fb.sde_partials, (long long)tree->n_tree * tree->n_leaves, D, st)) != BR_OK) return s;
  if ((s = embed_cond(model, fb, cond_tokens, tree->n_tree, st)) != BR_OK) return s;
  float* v = v_nodes ? v_nodes : fb.v;
  for (int i = 0; i < tree->T; ++i) {
    const int Bi = tree->n_tree * tree->width[i];
    const SampleMap sm{nullptr, nullptr, tree->n_nodes, tree->off[i], tree->width[i]};
    for (int b0 = 0; b0 < Bi; b0 += mb) {
      const int Bc = std::min(mb, Bi - b0);
      if ((s = fill_sample_maps(fb, sm, b0, Bc, v_nodes != nullptr, st)) != BR_OK) return s;
      if ((s = forward_uniform_t(model, fb, z_nodes, Bc, sched->t[i], tree->n_tree, v, st)) != BR_OK) return s;
    }
    if ((s = launch_sde_step(tree, sched, seed, i, D, v, v_nodes == nullptr, z_nodes, logp_edges, fb.sde_partials,
                             st)) != BR_OK)
      return s;
  }
  return BR_OK;
}

extern "C" br_status br_logprob(const br_tree* tree, const br_model* model, const br_sched* sched,
                                const void* cond_tokens, const float* z_nodes, const int32_t* edge_ids, int32_t n_edges,
                                float* logp_out, void* workspace, size_t workspace_bytes, void* stream) {
  BR_REQUIRE(tree && model && cond_tokens && z_nodes && workspace, BR_EINVAL, "br_logprob: NULL argument");
  BR_REQUIRE(n_edges >= 0 && (n_edges == 0 || (edge_ids && logp_out)), BR_EINVAL, "br_logprob: bad edge list");
  br_status s;
  if ((s = check_sched(tree, sched, "br_logprob")) != BR_OK) return s;
  if (n_edges == 0) return BR_OK;
  hipStream_t st = (hipStream_t)stream;
  const int nn = tree->n_nodes;
  const long long total_nodes = (long long)tree->n_tree * nn;
  BR_REQUIRE(n_edges <= total_nodes, BR_EINVAL, "br_logprob: more edges than the forest has");
  for (int e = 0; e < n_edges; ++e) {
    const int g = edge_ids[e];
    BR_REQUIRE(g >= 0 && g < total_nodes && g % nn != 0, BR_EINVAL, "br_logprob: edge id out of range or a root");
    BR_REQUIRE(e == 0 || g > edge_ids[e - 1], BR_EINVAL, "br_logprob: edge ids must be strictly ascending");
  }
  const int mb = fit_batch(tree, model, max_frontier(tree), workspace_bytes, 0);
  BR_REQUIRE(mb >= 1, BR_EWORKSPACE, "br_logprob: workspace too small (see br_workspace_bytes)");
  FwdBuffers fb;
  const Sizes sz = sizes_for(tree, model, mb);
  plan_workspace(model, sz.n_cond, mb, sz.v_rows, sz.partial_floats, sz.plan_ints, &fb, workspace);

  // Launch plan.  Parents of kept edges on stochastic steps are evaluated once each (siblings
  // share the evaluation), ordered by (step, row) and cut into batches of up to mb samples that
  // may span several steps: the network takes one time per modulation group (condition, step),
  // so shallow steps with few kept parents do not cost a poorly filled launch each.
  struct Edge { int step, crow, prow, par, slot; };
  std::vector<Edge> edges(n_edges);
  for (int e = 0; e < n_edges; ++e) {
    const int g = edge_ids[e], c = g / nn, n = g - c * nn;
    edges[e] = {tree->depth[n] - 1, g, c * nn + tree->parent[n], -1, e};
  }
  std::stable_sort(edges.begin(), edges.end(), [](const Edge& a, const Edge& b) { return a.step < b.step; });
  std::vector<int> p_row, p_cond, p_step;  // unique parents on stochastic steps
  for (Edge& ed : edges) {                // ascending ids inside a step: parents ascend too
    if (!(sched->sigma[ed.step] > 0.f)) continue;
    if (p_row.empty() || p_row.back() != ed.prow || p_step.back() != ed.step) {
      p_row.push_back(ed.prow);
      p_cond.push_back(ed.prow / nn);
      p_step.push_back(ed.step);
    }
    ed.par = (int)p_row.size() - 1;
  }
  const int n_par = (int)p_row.size();
  // host image of the plan: [rows | cond | group] per parent, then per batch its group tables,
  // then [crow | prow | vrow | slot] per edge in (step, id) order
  std::vector<int> host;
  const int o_rows = 0, o_cond = n_par, o_group = 2 * n_par;
  host.resize(3 * (size_t)n_par);
  struct Batch { int b0, B, o_gcond, o_gt, G; };
  std::vector<Batch> batches;
  for (int b0 = 0; b0 < n_par; b0 += mb) {
    Batch bt{b0, std::min(mb, n_par - b0), 0, 0, 0};
    std::vector<int> gcond, gstep;
    for (int i = b0; i < b0 + bt.B; ++i) {
      int g = -1;
      for (int k = (int)gcond.size() - 1; k >= 0 && g < 0; --k)
        if (gcond[k] == p_cond[i] && gstep[k] == p_step[i]) g = k;
      if (g < 0) {
        gcond.push_back(p_cond[i]);
        gstep.push_back(p_step[i]);
        g = (int)gcond.size() - 1;
      }
      host[o_rows + i] = p_row[i];
      host[o_cond + i] = p_cond[i];
      host[o_group + i] = g;
    }
    bt.G = (int)gcond.size();
    bt.o_gcond = (int)host.size();
    host.insert(host.end(), gcond.begin(), gcond.end());
    bt.o_gt = (int)host.size();
    for (int k = 0; k < bt.G; ++k) {
      const float tv = sched->t[gstep[k]];
      int bits;
      std::memcpy(&bits, &tv, sizeof(bits));
      host.push_back(bits);
    }
    batches.push_back(bt);
  }
  const int o_crow = (int)host.size(), o_prow = o_crow + n_edges, o_vrow = o_prow + n_edges, o_slot = o_vrow + n_edges;
  host.resize(host.size() + 4 * (size_t)n_edges);
  for (int e = 0; e < n_edges; ++e) {
    host[o_crow + e] = edges[e].crow;
    host[o_prow + e] = edges[e].prow;
    host[o_vrow + e] = edges[e].par >= 0 ? edges[e].par % mb : 0;  // row of the batch's velocity buffer
    host[o_slot + e] = edges[e].slot;
  }
  BR_REQUIRE((long long)host.size() <= sz.plan_ints, BR_EWORKSPACE, "br_logprob: plan does not fit the workspace");
  if ((s = tree->plan_stage.upload(host.data(), host.size(), fb.plan, st)) != BR_OK) return s;

  if ((s = embed_cond(model, fb, cond_tokens, tree->n_tree, st)) != BR_OK) return s;
  const long long D = model->D;
  if ((s = launch_sde_scratch_reset(fb.sde_partials, (long long)tree->n_tree * tree->n_leaves, D, st)) != BR_OK) return s;
  auto eval_range = [&](int e0, int e1) {  // edges [e0, e1): one step, velocities (if any) in fb.v
    return launch_logp_eval(sched, edges[e0].step, D, z_nodes, fb.v, fb.plan + o_crow + e0, fb.plan + o_prow + e0,
                            fb.plan + o_vrow + e0, fb.plan + o_slot + e0, e1 - e0, (long long)tree->n_tree * tree->n_leaves,
                            logp_out, fb.sde_partials, st);
  };
  // deterministic steps: no evaluation, log-prob 0
  for (int e0 = 0; e0 < n_edges;) {
    int e1 = e0 + 1;
    while (e1 < n_edges && edges[e1].step == edges[e0].step) ++e1;
    if (edges[e0].par < 0 && (s = eval_range(e0, e1)) != BR_OK) return s;
    e0 = e1;
  }
  int e_next = 0;  // edges are in (step, parent) order, so each batch owns a contiguous range
  for (const Batch& bt : batches) {
    SampleMap sm{fb.plan + o_rows, fb.plan + o_cond, 0, 0, 1};
    sm.group = fb.plan + o_group;
    if ((s = fill_sample_maps(fb, sm, bt.b0, bt.B, 2, st)) != BR_OK) return s;
    if ((s = forward(model, fb, z_nodes, bt.B, fb.plan + bt.o_gcond, reinterpret_cast<const float*>(fb.plan + bt.o_gt),
                     bt.G, fb.v, st)) != BR_OK)
      return s;
    while (e_next < n_edges && edges[e_next].par < bt.b0 + bt.B) {
      if (edges[e_next].par < 0) {  // deterministic step, done above
        ++e_next;
        continue;
      }
      int e1 = e_next + 1;
      while (e1 < n_edges && edges[e1].step == edges[e_next].step && edges[e1].par >= 0 &&
             edges[e1].par < bt.b0 + bt.B)
        ++e1;
      if ((s = eval_range(e_next, e1)) != BR_OK) return s;
      e_next = e1;
    }
  }
  return BR_OK;
}

extern "C" br_status br_velocity(const br_model* model, const float* z, float t, const void* cond_tokens,
                                 int32_t n_cond, const int32_t* cond_index, int32_t B, float* v_out, void* workspace,
                                 size_t workspace_bytes, void* stream) {
  BR_REQUIRE(model && z && cond_tokens && cond_index && v_out && workspace, BR_EINVAL, "br_velocity: NULL argument");
  BR_REQUIRE(B >= 1 && n_cond >= 1, BR_EINVAL, "br_velocity: B and n_cond must be >= 1");
  BR_REQUIRE(std::isfinite(t), BR_EINVAL, "br_velocity: t must be finite");
  for (int b = 0; b < B; ++b)
    BR_REQUIRE(cond_index[b] >= 0 && cond_index[b] < n_cond, BR_EINVAL, "br_velocity: cond_index out of range");
  hipStream_t st = (hipStream_t)stream;
  // the plan holds cond_index [B]; conditioning buffers are sized for n_cond
  int lo = 0, hi = B;
  while (lo < hi) {
    const int mid = (lo + hi + 1) / 2;
    if (plan_workspace(model, n_cond, mid, 0, 0, B, nullptr, nullptr) <= workspace_bytes) lo = mid;
    else hi = mid - 1;
  }
  const int mb = lo;
  BR_REQUIRE(mb >= 1, BR_EWORKSPACE, "br_velocity: workspace too small");
  FwdBuffers fb;
  plan_workspace(model, n_cond, mb, 0, 0, B, &fb, workspace);
  static PinnedStage cond_stage;  // (shared by all callers of br_velocity; uploads are serialised)
  br_status s;
  if ((s = cond_stage.upload(cond_index, (size_t)B, fb.plan, st)) != BR_OK) return s;
  if ((s = embed_cond(model, fb, cond_tokens, n_cond, st)) != BR_OK) return s;
  const SampleMap sm{nullptr, fb.plan, 0, 0, B};  // row = b
  for (int b0 = 0; b0 < B; b0 += mb) {
    const int Bc = std::min(mb, B - b0);
    if ((s = fill_sample_maps(fb, sm, b0, Bc, 0, st)) != BR_OK) return s;
    if ((s = forward_uniform_t(model, fb, z, Bc, t, n_cond, v_out, st)) != BR_OK) return s;
  }
  return BR_OK;
}

extern "C" br_status br_fuse_advantage(const br_tree* tree, const float* leaf_rewards, const float* logp_edges,
                                       float beta, float eps, int32_t ddof, float a_max, float* rbar_nodes,
                                       float* adv_nodes, void* stream) {
  BR_REQUIRE(tree && leaf_rewards && logp_edges && rbar_nodes && adv_nodes, BR_EINVAL, "br_fuse_advantage: NULL argument");
  BR_REQUIRE(std::isfinite(beta) && std::isfinite(eps) && eps >= 0.f && !std::isnan(a_max), BR_EINVAL,
             "br_fuse_advantage: beta / eps / a_max out of range");
  BR_REQUIRE(ddof == 0 || ddof == 1, BR_EINVAL, "br_fuse_advantage: ddof must be 0 or 1");
  TreeDev td;
  br_status s;
  if ((s = tree_device(tree, &td)) != BR_OK) return s;
  return launch_fuse_advantage(tree, td, leaf_rewards, logp_edges, beta, eps, ddof, a_max, rbar_nodes, adv_nodes,
                               (hipStream_t)stream);
}

extern "C" br_status br_prune(const br_tree* tree, const float* leaf_rewards, int32_t width_mode, int32_t b,
                              const uint8_t* depth_pruned, int32_t* kept_edges, int32_t* n_kept, void* stream) {
  BR_REQUIRE(tree && leaf_rewards && kept_edges && n_kept, BR_EINVAL, "br_prune: NULL argument");
  BR_REQUIRE(width_mode >= BR_PRUNE_NONE && width_mode <= BR_PRUNE_EXTREME, BR_EINVAL, "br_prune: unknown width mode");
  BR_REQUIRE(b >= 0, BR_EINVAL, "br_prune: b must be >= 0");
  DepthMask dm{};
  if (depth_pruned)
    for (int i = 0; i < tree->T; ++i)
      if (depth_pruned[i]) dm.bits[i >> 5] |= 1u << (i & 31);
  TreeDev td;
  br_status s;
  if ((s = tree_device(tree, &td)) != BR_OK) return s;
  if (tree->n_nodes == 1) {  // no edges at all (cannot happen with T >= 1, kept for safety)
    return fail(BR_EINVAL, "br_prune: tree has no edges");
  }
  return launch_prune(tree, td, leaf_rewards, width_mode, b, dm, kept_edges, n_kept, (hipStream_t)stream);
}

extern "C" size_t br_reward_scratch_bytes(const br_tree* tree, int32_t kind, int32_t latent_c, int32_t latent_t,
                                          int32_t latent_h, int32_t latent_w) {
  if (!tree || latent_c < 1 || latent_t < 1 || latent_h < 1 || latent_w < 1) return 0;
  const long long D = (long long)latent_c * latent_t * latent_h * latent_w;
  return reward_scratch_floats(tree, kind, D, latent_c, latent_t) * sizeof(float);
}

extern "C" br_status br_leaf_reward(const br_tree* tree, const float* z_nodes, int32_t kind, const float* w, float lam,
                                    int32_t latent_c, int32_t latent_t, int32_t latent_h, int32_t latent_w,
                                    float* rewards, void* scratch, size_t scratch_bytes, void* stream) {
  BR_REQUIRE(tree && z_nodes && w && rewards && scratch, BR_EINVAL, "br_leaf_reward: NULL argument");
  BR_REQUIRE(kind >= BR_REWARD_LINEAR && kind <= BR_REWARD_VIDEO, BR_EINVAL, "br_leaf_reward: unknown kind");
  BR_REQUIRE(latent_c >= 1 && latent_t >= 1 && latent_h >= 1 && latent_w >= 1, BR_EINVAL,
             "br_leaf_reward: latent sizes must be positive");
  const long long D = (long long)latent_c * latent_t * latent_h * latent_w;
  BR_REQUIRE(D % 4 == 0, BR_ESHAPE, "br_leaf_reward: latent size must be a multiple of 4");
  BR_REQUIRE(scratch_bytes >= br_reward_scratch_bytes(tree, kind, latent_c, latent_t, latent_h, latent_w),
             BR_EWORKSPACE, "br_leaf_reward: scratch too small (see br_reward_scratch_bytes)");
  return launch_leaf_reward(tree, z_nodes, kind, w, lam, latent_c, latent_t, latent_h, latent_w, rewards,
                            (float*)scratch, (hipStream_t)stream);
}

extern "C" br_status br_fusion_ess(const br_tree* tree, const float* logp_edges, float beta, float* ess_nodes,
                                   void* stream) {
  BR_REQUIRE(tree && logp_edges && ess_nodes, BR_EINVAL, "br_fusion_ess: NULL argument");
  BR_REQUIRE(std::isfinite(beta), BR_EINVAL, "br_fusion_ess: beta must be finite");
  TreeDev td;
  br_status s;
  if ((s = tree_device(tree, &td)) != BR_OK) return s;
  return launch_fusion_ess(tree, td, logp_edges, beta, ess_nodes, (hipStream_t)stream);
}

extern "C" br_status br_grpo_objective(const float* logp_new, const float* logp_old_nodes, const float* adv_nodes,
                                       const int32_t* edge_ids, int32_t n_edges, float clip_eps, float* J,
                                       uint8_t* clipped, void* stream) {
  BR_REQUIRE(J != nullptr && n_edges >= 0, BR_EINVAL, "br_grpo_objective: J is NULL or n_edges < 0");
  BR_REQUIRE(n_edges == 0 || (logp_new && logp_old_nodes && adv_nodes && edge_ids), BR_EINVAL,
             "br_grpo_objective: NULL argument");
  BR_REQUIRE(std::isfinite(clip_eps) && clip_eps >= 0.f, BR_EINVAL, "br_grpo_objective: clip_eps must be >= 0");
  return launch_grpo_objective(logp_new, logp_old_nodes, adv_nodes, edge_ids, n_edges, clip_eps, J, clipped,
                               (hipStream_t)stream);
}

extern "C" size_t br_sde_scratch_bytes(const br_tree* tree, int64_t D) {
  if (!tree || D < 4) return 0;
  return sde_scratch_floats((long long)tree->n_tree * tree->n_leaves, D) * sizeof(float);
}

extern "C" br_status br_sde_step(const br_tree* tree, const br_sched* sched, uint64_t seed, int32_t step, int64_t D,
                                 const float* v_parents, float* z_nodes, float* logp_edges, void* scratch,
                                 size_t scratch_bytes, void* stream) {
  BR_REQUIRE(tree && v_parents && z_nodes && logp_edges && scratch, BR_EINVAL, "br_sde_step: NULL argument");
  br_status s;
  if ((s = check_sched(tree, sched, "br_sde_step")) != BR_OK) return s;
  BR_REQUIRE(step >= 0 && step < tree->T, BR_EINVAL, "br_sde_step: step outside [0, T)");
  BR_REQUIRE(D >= 4 && D % 4 == 0, BR_ESHAPE, "br_sde_step: D must be a positive multiple of 4");
  BR_REQUIRE(scratch_bytes >= br_sde_scratch_bytes(tree, D), BR_EWORKSPACE, "br_sde_step: scratch too small");
  BR_REQUIRE(((uintptr_t)scratch & 7) == 0, BR_EINVAL, "br_sde_step: scratch must be 8-byte aligned");
  if ((s = launch_sde_scratch_reset((float*)scratch, (long long)tree->n_tree * tree->n_leaves, D, (hipStream_t)stream)) != BR_OK)
    return s;
  return launch_sde_step(tree, sched, seed, step, D, v_parents, 1, z_nodes, logp_edges, (float*)scratch,
                         (hipStream_t)stream);
}

// ---- br_sde_step for callers that cannot allocate: the scratch of the step (the 64-bit
// words the blocks of a child accumulate its log-prob in) lives in a device array of the library instead of a caller buffer.
namespace {
constexpr size_t kStaticScratchBytes = 1u << 16;  // one 64-bit word per child of a step: 8192 children
static __device__ __align__(256) unsigned char g_sde_scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
void* g_sde_scratch_ptr[kMaxDevices] = {nullptr};  // device address of the array on each device

br_status static_scratch(float** out) {
  int dev = 0;
  BR_HIP(hipGetDevice(&dev));
  BR_REQUIRE(dev >= 0 && dev < kMaxDevices, BR_EDEVICE, "br_sde_step_static: device index out of range");
  void* p = __atomic_load_n(&g_sde_scratch_ptr[dev], __ATOMIC_ACQUIRE);
  if (!p) {  // every device holds its own copy of the array at its own address
    BR_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(g_sde_scratch)));
    BR_REQUIRE(p != nullptr, BR_EDEVICE, "br_sde_step_static: the scratch array has no device address");
    __atomic_store_n(&g_sde_scratch_ptr[dev], p, __ATOMIC_RELEASE);
  }
  *out = static_cast<float*>(p);
  return BR_OK;
}
}  // namespace

extern "C" size_t br_sde_static_scratch_limit(void) { return kStaticScratchBytes; }

extern "C" br_status br_sde_step_static(const br_tree* tree, const br_sched* sched, uint64_t seed, int32_t step,
                                        int64_t D, const float* v_parents, float* z_nodes, float* logp_edges,
                                        void* stream) {
  BR_REQUIRE(tree && v_parents && z_nodes && logp_edges, BR_EINVAL, "br_sde_step_static: NULL argument");
  br_status s;
  if ((s = check_sched(tree, sched, "br_sde_step_static")) != BR_OK) return s;
  BR_REQUIRE(step >= 0 && step < tree->T, BR_EINVAL, "br_sde_step_static: step outside [0, T)");
  BR_REQUIRE(D >= 4 && D % 4 == 0, BR_ESHAPE, "br_sde_step_static: D must be a positive multiple of 4");
  BR_REQUIRE(br_sde_scratch_bytes(tree, D) <= kStaticScratchBytes, BR_EWORKSPACE,
             "br_sde_step_static: the tree needs more than the 64 KiB of built-in scratch (br_sde_scratch_bytes: "
             "8 bytes per leaf); use br_sde_step with a caller buffer");
  float* scratch = nullptr;
  if ((s = static_scratch(&scratch)) != BR_OK) return s;
  const long long n_items = (long long)tree->n_tree * tree->n_leaves;
  if ((s = launch_sde_scratch_reset(scratch, n_items, D, (hipStream_t)stream)) != BR_OK) return s;
  return launch_sde_step(tree, sched, seed, step, D, v_parents, 1, z_nodes, logp_edges, scratch, (hipStream_t)stream);
}

extern "C" br_status br_root_noise(const br_tree* tree, uint64_t seed, const int32_t* noise_group, int64_t D,
                                   float* z_nodes, void* stream) {
  BR_REQUIRE(tree && noise_group && z_nodes, BR_EINVAL, "br_root_noise: NULL argument");
  BR_REQUIRE(D >= 4 && D % 4 == 0, BR_ESHAPE, "br_root_noise: D must be a positive multiple of 4");
  return launch_root_noise(tree, seed, noise_group, D, z_nodes, (hipStream_t)stream);
}

extern "C" br_status br_noise_stream(uint64_t seed, uint32_t node_id, uint32_t step, uint32_t tag, int64_t n_quads,
                                     uint32_t* words, float* normals, void* stream) {
  BR_REQUIRE(n_quads >= 0 && n_quads <= 0xFFFFFFFFLL, BR_EINVAL, "br_noise_stream: n_quads out of range");
  BR_REQUIRE(words || normals, BR_EINVAL, "br_noise_stream: both outputs are NULL");
  return launch_noise_stream(seed, node_id, step, tag, n_quads, words, normals, (hipStream_t)stream);
}
