// Tree post-processing: synthetic leaf rewards, reward fusion (Eq. 3), depth-wise
// normalisation (Eq. 4), width/depth pruning (Sec. 3.4) and the clipped objective
// value (Eq. 5).  A tree has at most a few thousand nodes, so one wavefront (or
// one workgroup) owns a whole tree and reduces with lane shuffles in a fixed
// order; results are deterministic.
#include "common.h"
#include "kernels.h"

namespace br {

__device__ inline float wsum_f(float x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x += __shfl_down(x, o, 64);
  return x;
}
__device__ inline double wsum_d(double x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x += __shfl_down(x, o, 64);
  return __shfl(x, 0, 64);
}
__device__ inline double wmax_d(double x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x = fmax(x, __shfl_down(x, o, 64));
  return __shfl(x, 0, 64);
}

// ------------------------------------------------------------------ rewards
// Stage 1 (linear / tanh): slice sums of <w, z_leaf>; grid (S, n_leaves_total).
__global__ __launch_bounds__(256) void reward_dot_kernel(const float* __restrict__ z, const float* __restrict__ w,
                                                         long long D, int n_nodes, int leaf_off, int n_leaves,
                                                         float* __restrict__ partials) {
  __shared__ float red[4];
  const int g = blockIdx.y, c = g / n_leaves, l = g - c * n_leaves;
  const float4* zp = reinterpret_cast<const float4*>(z + ((size_t)c * n_nodes + leaf_off + l) * D);
  const float4* wp = reinterpret_cast<const float4*>(w);
  const long long nq = D >> 2;
  float acc = 0.f;
  for (long long q = (long long)blockIdx.x * 256 + threadIdx.x; q < nq; q += (long long)gridDim.x * 256) {
    const float4 a = zp[q], b = wp[q];
    acc += (a.x * b.x + a.y * b.y) + (a.z * b.z + a.w * b.w);
  }
  acc = wsum_f(acc);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = acc;
  __syncthreads();
  if (threadIdx.x == 0) partials[(size_t)g * gridDim.x + blockIdx.x] = (red[0] + red[1]) + (red[2] + red[3]);
}

__global__ __launch_bounds__(64) void reward_dot_finish_kernel(const float* __restrict__ partials, int S, double inv_sqrt_d,
                                                               int use_tanh, float* __restrict__ out) {
  const int g = blockIdx.x;
  double s = 0.0;
  for (int i = threadIdx.x; i < S; i += 64) s += (double)partials[(size_t)g * S + i];
  s = wsum_d(s);
  if (threadIdx.x == 0) {
    const double r = s * inv_sqrt_d;
    out[g] = (float)(use_tanh ? tanh(r) : r);
  }
}

// Stage 1 (video): mean of one (channel, frame) plane; grid (C*F, n_leaves_total).
__global__ __launch_bounds__(256) void reward_plane_mean_kernel(const float* __restrict__ z, long long D, int n_nodes,
                                                                int leaf_off, int n_leaves, int plane,
                                                                float* __restrict__ means) {
  __shared__ float red[4];
  const int g = blockIdx.y, c = g / n_leaves, l = g - c * n_leaves;
  const float* p = z + ((size_t)c * n_nodes + leaf_off + l) * D + (size_t)blockIdx.x * plane;
  float acc = 0.f;
  for (int i = threadIdx.x; i < plane; i += 256) acc += p[i];
  acc = wsum_f(acc);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = acc;
  __syncthreads();
  if (threadIdx.x == 0)
    means[(size_t)g * gridDim.x + blockIdx.x] = ((red[0] + red[1]) + (red[2] + red[3])) / (float)plane;
}

// Stage 2 (video): m is stored [C, F] per leaf; w is [F, C].
__global__ __launch_bounds__(64) void reward_video_finish_kernel(const float* __restrict__ means,
                                                                 const float* __restrict__ w, int C, int F, float lam,
                                                                 float* __restrict__ out) {
  const int g = blockIdx.x;
  const float* m = means + (size_t)g * C * F;
  double lin = 0.0, pen = 0.0;
  for (int i = threadIdx.x; i < C * F; i += 64) {
    const int c = i / F, f = i - c * F;
    lin += (double)w[f * C + c] * (double)m[i];
    if (f + 1 < F) {
      const double d = (double)m[i + 1] - (double)m[i];
      pen += d * d;
    }
  }
  lin = wsum_d(lin);
  pen = wsum_d(pen);
  if (threadIdx.x == 0) {
    double r = lin / sqrt((double)F * C);
    if (F > 1) r -= (double)lam * pen / (double)(F - 1);
    out[g] = (float)r;
  }
}

// ------------------------------------------------- fusion + depth-wise advantages
// One wavefront per tree.  S(l) = sum of edge log-probs from the root to leaf l;
// because the softmax of Eq. 3 is shift-invariant, the weights of node n are
// softmax over its leaf interval of beta * S(l).
struct FuseCtx {
  const double* S;  // LDS [w]
  const float* r;   // global leaf rewards of this tree
  double beta;
};

// rbar of the node whose leaves are [lo, hi), computed by one lane.
__device__ inline double rbar_lane(const FuseCtx& cx, int lo, int hi) {
  double m = -INFINITY;
  for (int l = lo; l < hi; ++l) m = fmax(m, cx.beta * cx.S[l]);
  double num = 0.0, den = 0.0;
  for (int l = lo; l < hi; ++l) {
    const double e = exp(cx.beta * cx.S[l] - m);
    num += e * (double)cx.r[l];
    den += e;
  }
  return num / den;
}
// The same by the whole wavefront (result in every lane).
__device__ inline double rbar_wave(const FuseCtx& cx, int lo, int hi) {
  const int lane = threadIdx.x & 63;
  double m = -INFINITY;
  for (int l = lo + lane; l < hi; l += 64) m = fmax(m, cx.beta * cx.S[l]);
  m = wmax_d(m);
  double num = 0.0, den = 0.0;
  for (int l = lo + lane; l < hi; l += 64) {
    const double e = exp(cx.beta * cx.S[l] - m);
    num += e * (double)cx.r[l];
    den += e;
  }
  return wsum_d(num) / wsum_d(den);
}

__global__ __launch_bounds__(64) void fuse_advantage_kernel(TreeDev td, int T, int n_nodes, int w,
                                                            const float* __restrict__ rewards,
                                                            const float* __restrict__ logp, double beta, double eps,
                                                            int ddof, double a_max, float* __restrict__ rbar_out,
                                                            float* __restrict__ adv_out) {
  extern __shared__ double S[];
  const int c = blockIdx.x, lane = threadIdx.x;
  const float* lp = logp + (size_t)c * n_nodes;
  const int leaf0 = td.off[T];
  for (int l = lane; l < w; l += 64) {
    double s = 0.0;
    for (int n = leaf0 + l; td.parent[n] >= 0; n = td.parent[n]) s += (double)lp[n];
    S[l] = s;
  }
  __syncthreads();
  FuseCtx cx{S, rewards + (size_t)c * w, beta};
  for (int d = 0; d <= T; ++d) {
    const int lo_n = td.off[d], wd = td.off[d + 1] - lo_n, span = w / wd;
    const bool by_wave = span >= 32;
    // three sweeps over the depth: mean, spread, output; rbar is recomputed each time
    double mean = 0.0, inv = 0.0;
    for (int pass = 0; pass < 3; ++pass) {
      double acc = 0.0;
      if (by_wave) {
        for (int j = 0; j < wd; ++j) {
          const double rb = rbar_wave(cx, j * span, (j + 1) * span);
          if (pass == 0) acc += rb;
          else if (pass == 1) acc += (rb - mean) * (rb - mean);
          else if (lane == 0) {
            double a = (rb - mean) * inv;
            if (a_max > 0.0) a = fmin(fmax(a, -a_max), a_max);
            rbar_out[(size_t)c * n_nodes + lo_n + j] = (float)rb;
            adv_out[(size_t)c * n_nodes + lo_n + j] = (float)a;
          }
        }
      } else {
        for (int j = lane; j < wd; j += 64) {
          const double rb = rbar_lane(cx, j * span, (j + 1) * span);
          if (pass == 0) acc += rb;
          else if (pass == 1) acc += (rb - mean) * (rb - mean);
          else {
            double a = (rb - mean) * inv;
            if (a_max > 0.0) a = fmin(fmax(a, -a_max), a_max);
            rbar_out[(size_t)c * n_nodes + lo_n + j] = (float)rb;
            adv_out[(size_t)c * n_nodes + lo_n + j] = (float)a;
          }
        }
        if (pass < 2) acc = wsum_d(acc);
      }
      if (pass == 0) mean = acc / (double)wd;
      else if (pass == 1) {
        const int dof = wd - ddof;
        const double sd = dof > 0 ? sqrt(acc / (double)dof) : 0.0;
        inv = (dof > 0 && sd + eps > 0.0) ? 1.0 / (sd + eps) : 0.0;
      }
    }
  }
}

// The same for trees whose leaf path sums and fused rewards fit in LDS (every tree of the
// paper's presets does): one workgroup of four wavefronts per tree.  Every node's fused reward is
// computed once -- nodes with 64 or more leaves by a whole wavefront, the others by one lane each,
// all in parallel -- and kept in LDS; the depths are then normalised from there, one wavefront
// per depth.  Summation orders are fixed, so the result does not depend on timing.
__global__ __launch_bounds__(256) void fuse_advantage_lds_kernel(TreeDev td, int T, int n_nodes, int w,
                                                                 const float* __restrict__ rewards,
                                                                 const float* __restrict__ logp, double beta,
                                                                 double eps, int ddof, double a_max,
                                                                 float* __restrict__ rbar_out,
                                                                 float* __restrict__ adv_out) {
  extern __shared__ double sh[];
  double* S = sh;        // [w] leaf path sums
  double* RB = sh + w;   // [n_nodes] fused rewards
  const int c = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const float* lp = logp + (size_t)c * n_nodes;
  const int leaf0 = td.off[T];
  for (int l = tid; l < w; l += 256) {
    double s = 0.0;
    for (int n = leaf0 + l; td.parent[n] >= 0; n = td.parent[n]) s += (double)lp[n];
    S[l] = s;
  }
  __syncthreads();
  FuseCtx cx{S, rewards + (size_t)c * w, beta};
  // nodes with many leaves: depth by depth, one wavefront per node
  int first_small = 0;  // first node (level order) with fewer than 64 leaves
  for (int d = 0; d <= T; ++d) {
    const int lo_n = td.off[d], wd = td.off[d + 1] - lo_n, span = w / wd;
    if (span < 64) break;
    for (int j = wv; j < wd; j += 4) {
      const double rb = rbar_wave(cx, j * span, (j + 1) * span);
      if (lane == 0) RB[lo_n + j] = rb;
    }
    first_small = lo_n + wd;
  }
  for (int n = first_small + tid; n < n_nodes; n += 256) RB[n] = rbar_lane(cx, td.leaf_lo[n], td.leaf_hi[n]);
  __syncthreads();
  for (int d = wv; d <= T; d += 4) {
    const int lo_n = td.off[d], wd = td.off[d + 1] - lo_n;
    double acc = 0.0;
    for (int j = lane; j < wd; j += 64) acc += RB[lo_n + j];
    const double mean = wsum_d(acc) / (double)wd;
    acc = 0.0;
    for (int j = lane; j < wd; j += 64) acc += (RB[lo_n + j] - mean) * (RB[lo_n + j] - mean);
    acc = wsum_d(acc);
    const int dof = wd - ddof;
    const double sd = dof > 0 ? sqrt(acc / (double)dof) : 0.0;
    const double inv = (dof > 0 && sd + eps > 0.0) ? 1.0 / (sd + eps) : 0.0;
    for (int j = lane; j < wd; j += 64) {
      const double rb = RB[lo_n + j];
      double a = (rb - mean) * inv;
      if (a_max > 0.0) a = fmin(fmax(a, -a_max), a_max);
      rbar_out[(size_t)c * n_nodes + lo_n + j] = (float)rb;
      adv_out[(size_t)c * n_nodes + lo_n + j] = (float)a;
    }
  }
}

// Effective sample size of the fusion weights of every node (App., self-normalised importance
// sampling view of Eq. 3): ESS(n) = (sum_l w_l)^2 / sum_l w_l^2 over the leaves under n, with
// w_l = exp(beta S(l) - max).  One wavefront per tree, same leaf path sums as the fusion.
__global__ __launch_bounds__(64) void fusion_ess_kernel(TreeDev td, int T, int n_nodes, int w,
                                                        const float* __restrict__ logp, double beta,
                                                        float* __restrict__ ess_out) {
  extern __shared__ double S[];
  const int c = blockIdx.x, lane = threadIdx.x;
  const float* lp = logp + (size_t)c * n_nodes;
  const int leaf0 = td.off[T];
  for (int l = lane; l < w; l += 64) {
    double s = 0.0;
    for (int n = leaf0 + l; td.parent[n] >= 0; n = td.parent[n]) s += (double)lp[n];
    S[l] = s;
  }
  __syncthreads();
  for (int d = 0; d <= T; ++d) {
    const int lo_n = td.off[d], wd = td.off[d + 1] - lo_n, span = w / wd;
    if (span >= 32) {
      for (int j = 0; j < wd; ++j) {
        const int lo = j * span, hi = lo + span;
        double m = -INFINITY;
        for (int l = lo + lane; l < hi; l += 64) m = fmax(m, beta * S[l]);
        m = wmax_d(m);
        double s1 = 0.0, s2 = 0.0;
        for (int l = lo + lane; l < hi; l += 64) {
          const double e = exp(beta * S[l] - m);
          s1 += e;
          s2 += e * e;
        }
        s1 = wsum_d(s1);
        s2 = wsum_d(s2);
        if (lane == 0) ess_out[(size_t)c * n_nodes + lo_n + j] = (float)(s1 * s1 / s2);
      }
    } else {
      for (int j = lane; j < wd; j += 64) {
        const int lo = j * span, hi = lo + span;
        double m = -INFINITY;
        for (int l = lo; l < hi; ++l) m = fmax(m, beta * S[l]);
        double s1 = 0.0, s2 = 0.0;
        for (int l = lo; l < hi; ++l) {
          const double e = exp(beta * S[l] - m);
          s1 += e;
          s2 += e * e;
        }
        ess_out[(size_t)c * n_nodes + lo_n + j] = (float)(s1 * s1 / s2);
      }
    }
  }
}

// ------------------------------------------------------------------ pruning
__device__ inline bool dm_get(const DepthMask& dm, int i) { return (dm.bits[i >> 5] >> (i & 31)) & 1u; }

// One workgroup per tree: leaf selection, then per-edge flags written to
// flags[c*n_edges + (n-1)].
__global__ __launch_bounds__(256) void prune_flags_kernel(TreeDev td, int T, int K, int n_nodes, int w, int last_split,
                                                          const float* __restrict__ rewards, int mode, int b,
                                                          DepthMask dm, int* __restrict__ flags) {
  extern __shared__ int pre[];  // [w + 1] exclusive prefix of kept-leaf flags
  __shared__ int chunk_sum[256];
  const int c = blockIdx.x, tid = threadIdx.x;
  const float* r = rewards + (size_t)c * w;
  for (int l = tid; l < w; l += 256) {
    int keep = 1;
    if (mode == BR_PRUNE_EXTREME && 2 * b < w) {
      const float rl = r[l];
      int rank = 0;
      for (int m = 0; m < w; ++m) {
        const float rm = r[m];
        rank += (rm < rl || (rm == rl && m < l)) ? 1 : 0;
      }
      keep = (rank < b || rank >= w - b) ? 1 : 0;
    } else if (mode == BR_PRUNE_PARENT_TOP1 && last_split >= 0) {
      // after the last split every node has one leaf: leaf l is child l of that depth
      const int first = l - l % K;
      int best = first;
      for (int m = first + 1; m < first + K; ++m)
        if (r[m] > r[best]) best = m;
      keep = best == l ? 1 : 0;
    }
    pre[l + 1] = keep;
  }
  if (tid == 0) pre[0] = 0;
  __syncthreads();
  // inclusive scan of pre[1..w] in place: per-thread chunks, then chunk offsets
  const int per = (w + 255) / 256, lo = 1 + tid * per, hi = min(lo + per, w + 1);
  int s = 0;
  for (int i = lo; i < hi; ++i) s += pre[i];
  chunk_sum[tid] = s;
  __syncthreads();
  int base = 0;
  for (int i = 0; i < tid; ++i) base += chunk_sum[i];
  for (int i = lo; i < hi; ++i) {
    base += pre[i];
    pre[i] = base;
  }
  __syncthreads();
  const int n_edges = n_nodes - 1;
  for (int n = 1 + tid; n < n_nodes; n += 256) {
    const bool has = pre[td.leaf_hi[n]] - pre[td.leaf_lo[n]] > 0;
    flags[(size_t)c * n_edges + (n - 1)] = (has && !dm_get(dm, td.depth[n] - 1)) ? 1 : 0;
  }
}

// Single workgroup: in-place ordered compaction of the flags into global child ids.
__global__ __launch_bounds__(1024) void prune_compact_kernel(int* __restrict__ buf, int n_tree, int n_nodes,
                                                             int* __restrict__ n_kept) {
  __shared__ int wsums[16];
  __shared__ int running;
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int n_edges = n_nodes - 1;
  const long long total = (long long)n_tree * n_edges;
  if (tid == 0) running = 0;
  __syncthreads();
  for (long long base = 0; base < total; base += 1024) {
    const long long i = base + tid;
    const int f = i < total ? buf[i] : 0;
    // inclusive scan inside the wavefront, then across the 16 wavefronts
    int x = f;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int y = __shfl_up(x, o, 64);
      if (lane >= o) x += y;
    }
    if (lane == 63) wsums[wv] = x;
    __syncthreads();  // all flags of this chunk are read; wave totals visible
    int before = running;
    for (int k = 0; k < wv; ++k) before += wsums[k];
    if (f) {
      const int c = (int)(i / n_edges), e = (int)(i - (long long)c * n_edges);
      buf[before + x - 1] = c * n_nodes + e + 1;
    }
    __syncthreads();
    if (tid == 0) {
      int t = running;
      for (int k = 0; k < 16; ++k) t += wsums[k];
      running = t;
    }
    __syncthreads();
  }
  if (tid == 0) *n_kept = running;
}

// ------------------------------------------------------------------ objective
__global__ __launch_bounds__(256) void grpo_objective_kernel(const float* __restrict__ logp_new,
                                                             const float* __restrict__ logp_old,
                                                             const float* __restrict__ adv,
                                                             const int* __restrict__ ids, int n, double clip_eps,
                                                             float* __restrict__ J,
                                                             unsigned char* __restrict__ clipped) {
  __shared__ double red[4];
  double acc = 0.0;
  for (int e = threadIdx.x; e < n; e += 256) {
    const int g = ids[e];
    const double rho = exp((double)logp_new[e] - (double)logp_old[g]), a = adv[g];
    const double cl = fmin(fmax(rho, 1.0 - clip_eps), 1.0 + clip_eps);
    acc += fmin(rho * a, cl * a);
    if (clipped) clipped[e] = cl * a < rho * a ? 1 : 0;  // the clipped term is the one taken
  }
  acc = wsum_d(acc);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = acc;
  __syncthreads();
  if (threadIdx.x == 0) J[0] = n > 0 ? (float)(((red[0] + red[1]) + (red[2] + red[3])) / (double)n) : 0.f;
}

// ---------------------------------------------------------------- host side

static int reward_slices(long long D) {
  long long s = (D / 4 + 1023) / 1024;
  return (int)(s < 1 ? 1 : (s > 64 ? 64 : s));
}

size_t reward_scratch_floats(const br_tree* t, int kind, long long D, int lc, int lt) {
  const size_t nl = (size_t)t->n_tree * t->n_leaves;
  return kind == BR_REWARD_VIDEO ? nl * (size_t)lc * lt : nl * (size_t)reward_slices(D);
}

br_status launch_leaf_reward(const br_tree* t, const float* z, int kind, const float* w, float lam, int lc, int lt,
                             int lh, int lw, float* rewards, float* scratch, hipStream_t st) {
  const long long D = (long long)lc * lt * lh * lw;
  const int nl = t->n_tree * t->n_leaves;
  BR_REQUIRE(nl <= 65535, BR_ESHAPE, "leaf reward: more than 65535 leaves are not supported");
  if (kind == BR_REWARD_VIDEO) {
    BR_REQUIRE(lc * lt <= 65535 * 32, BR_ESHAPE, "leaf reward: too many planes");
    hipLaunchKernelGGL(reward_plane_mean_kernel, dim3(lc * lt, nl), dim3(256), 0, st, z, D, t->n_nodes, t->off[t->T],
                       t->n_leaves, lh * lw, scratch);
    BR_LAUNCH_CHECK();
    hipLaunchKernelGGL(reward_video_finish_kernel, dim3(nl), dim3(64), 0, st, scratch, w, lc, lt, lam, rewards);
  } else {
    const int S = reward_slices(D);
    hipLaunchKernelGGL(reward_dot_kernel, dim3(S, nl), dim3(256), 0, st, z, w, D, t->n_nodes, t->off[t->T],
                       t->n_leaves, scratch);
    BR_LAUNCH_CHECK();
    hipLaunchKernelGGL(reward_dot_finish_kernel, dim3(nl), dim3(64), 0, st, scratch, S, 1.0 / sqrt((double)D),
                       kind == BR_REWARD_TANH ? 1 : 0, rewards);
  }
  BR_LAUNCH_CHECK();
  return BR_OK;
}

br_status launch_fuse_advantage(const br_tree* t, const TreeDev& td, const float* r, const float* logp, float beta,
                                float eps, int ddof, float a_max, float* rbar, float* adv, hipStream_t st) {
  BR_REQUIRE(t->n_leaves <= 4096, BR_ESHAPE, "fuse: more than 4096 leaves per tree are not supported");
  const size_t cached = ((size_t)t->n_leaves + (size_t)t->n_nodes) * sizeof(double);
  if (cached <= 48 * 1024) {
    hipLaunchKernelGGL(fuse_advantage_lds_kernel, dim3(t->n_tree), dim3(256), cached, st, td, t->T, t->n_nodes,
                       t->n_leaves, r, logp, (double)beta, (double)eps, ddof, (double)a_max, rbar, adv);
    BR_LAUNCH_CHECK();
    return BR_OK;
  }
  hipLaunchKernelGGL(fuse_advantage_kernel, dim3(t->n_tree), dim3(64), (size_t)t->n_leaves * sizeof(double), st, td,
                     t->T, t->n_nodes, t->n_leaves, r, logp, (double)beta, (double)eps, ddof, (double)a_max, rbar, adv);
  BR_LAUNCH_CHECK();
  return BR_OK;
}

br_status launch_fusion_ess(const br_tree* t, const TreeDev& td, const float* logp, float beta, float* ess,
                            hipStream_t st) {
  BR_REQUIRE(t->n_leaves <= 4096, BR_ESHAPE, "ess: more than 4096 leaves per tree are not supported");
  hipLaunchKernelGGL(fusion_ess_kernel, dim3(t->n_tree), dim3(64), (size_t)t->n_leaves * sizeof(double), st, td, t->T,
                     t->n_nodes, t->n_leaves, logp, (double)beta, ess);
  BR_LAUNCH_CHECK();
  return BR_OK;
}

br_status launch_prune(const br_tree* t, const TreeDev& td, const float* r, int mode, int b, const DepthMask& dm,
                       int* kept, int* n_kept, hipStream_t st) {
  BR_REQUIRE(t->n_leaves <= 8191, BR_ESHAPE, "prune: more than 8191 leaves per tree are not supported");
  const int last_split = t->splits.empty() ? -1 : t->splits.back();
  hipLaunchKernelGGL(prune_flags_kernel, dim3(t->n_tree), dim3(256), (size_t)(t->n_leaves + 1) * sizeof(int), st, td,
                     t->T, t->K, t->n_nodes, t->n_leaves, last_split, r, mode, b, dm, kept);
  BR_LAUNCH_CHECK();
  hipLaunchKernelGGL(prune_compact_kernel, dim3(1), dim3(1024), 0, st, kept, t->n_tree, t->n_nodes, n_kept);
  BR_LAUNCH_CHECK();
  return BR_OK;
}

br_status launch_grpo_objective(const float* logp_new, const float* logp_old_nodes, const float* adv_nodes,
                                const int* edge_ids, int n, float clip_eps, float* J, unsigned char* clipped,
                                hipStream_t st) {
  hipLaunchKernelGGL(grpo_objective_kernel, dim3(1), dim3(256), 0, st, logp_new, logp_old_nodes, adv_nodes, edge_ids, n,
                     (double)clip_eps, J, clipped);
  BR_LAUNCH_CHECK();
  return BR_OK;
}

}  // namespace br
