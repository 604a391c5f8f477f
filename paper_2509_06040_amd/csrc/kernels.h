// Launch wrappers of the HIP kernels (one translation unit each); internal.
#pragma once
#include "common.h"

namespace br {

// ---- sde_kernels.hip
struct StepCoef {
  float a_z, a_v;   // mu = a_z z + a_v v   (App. B.1 Euler-Maruyama mean of step i)
  float std;        // sigma_i sqrt(h_i)
  float ca, cb;     // xi_b = ca xi_0 + cb eta_b  (Eq. 2)
  int noise;        // 0: deterministic step, no log-prob
  double c0;        // -D ln std - D/2 ln 2 pi
  double inv_div;   // 1 or 1/D
  float inv_std;    // 1/std (0 on a deterministic step)
};
StepCoef step_coef(const br_sched* s, int i, long long D);
br_status launch_root_noise(const br_tree* t, uint64_t seed, const int* noise_group, long long D, float* z,
                            hipStream_t st);
// `scratch` of the two launchers below: sde_scratch_floats(n_items, D) floats = one 64-bit word per child
// / edge of a launch (at most n_items), 8-byte aligned; the words must be zero (launch_sde_scratch_reset)
// before the first launch and are left at zero by every launch.
size_t sde_scratch_floats(long long n_items, long long D);
br_status launch_sde_scratch_reset(float* scratch, long long n_items, long long D, hipStream_t st);
br_status launch_sde_step(const br_tree* t, const br_sched* s, uint64_t seed, int i, long long D, const float* v,
                          int v_compact, float* z, float* logp, float* scratch, hipStream_t st);
br_status launch_logp_eval(const br_sched* s, int i, long long D, const float* z, const float* v, const int* crow,
                           const int* prow, const int* vrow, const int* out_slot, int n_edges, long long n_items,
                           float* logp_out, float* scratch, hipStream_t st);
br_status launch_fill_zero(float* p, long long n, hipStream_t st);
br_status launch_noise_stream(uint64_t seed, uint32_t node, uint32_t step, uint32_t tag, long long nq, uint32_t* words,
                              float* normals, hipStream_t st);

// ---- tree_kernels.hip
struct DepthMask {
  uint32_t bits[32];  // step i dropped iff bit i set (T <= 1024)
};
size_t reward_scratch_floats(const br_tree* t, int kind, long long D, int lc, int lt);
br_status launch_leaf_reward(const br_tree* t, const float* z, int kind, const float* w, float lam, int lc, int lt,
                             int lh, int lw, float* rewards, float* scratch, hipStream_t st);
br_status launch_fuse_advantage(const br_tree* t, const TreeDev& td, const float* r, const float* logp, float beta,
                                float eps, int ddof, float a_max, float* rbar, float* adv, hipStream_t st);
br_status launch_prune(const br_tree* t, const TreeDev& td, const float* r, int mode, int b, const DepthMask& dm,
                       int* kept, int* n_kept, hipStream_t st);
br_status launch_grpo_objective(const float* logp_new, const float* logp_old_nodes, const float* adv_nodes,
                                const int* edge_ids, int n, float clip_eps, float* J, unsigned char* clipped,
                                hipStream_t st);
br_status launch_fusion_ess(const br_tree* t, const TreeDev& td, const float* logp, float beta, float* ess,
                            hipStream_t st);

}  // namespace br
