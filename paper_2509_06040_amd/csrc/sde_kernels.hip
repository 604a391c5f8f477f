// Fused reverse-SDE step + counter-based noise + transition log-prob + branch
// expansion (Eq. 1, Eq. 2, App. B.1), the log-prob re-evaluation of stored
// transitions (ratio of Eq. 5) and the root noise (Alg. 1 "sample root noise").
// HBM-bound: a parent's z and v are read once, every child is written once; the
// noise lives in registers only.
#include "common.h"
#include "kernels.h"
#include "philox.h"
#include "prof.h"

namespace br {

__device__ inline float wave_sum(float x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x += __shfl_down(x, o, 64);
  return x;
}

// Sum over a 256-thread block in a fixed order; result valid in thread 0.
__device__ inline float block_sum_256(float x, float* lds4) {
  x = wave_sum(x);
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  __syncthreads();
  if (lane == 0) lds4[wv] = x;
  __syncthreads();
  return (lds4[0] + lds4[1]) + (lds4[2] + lds4[3]);
}

struct RootArgs {
  int group[256];
};

__global__ __launch_bounds__(256) void root_noise_kernel(float* __restrict__ z, long long D, int n_nodes, int tree0,
                                                         RootArgs ga, PhiloxKey key) {
  const int c = blockIdx.y;
  const long long nq = D >> 2;
  float4* dst = reinterpret_cast<float4*>(z + (size_t)(tree0 + c) * n_nodes * D);
  for (long long q = (long long)blockIdx.x * 256 + threadIdx.x; q < nq; q += (long long)gridDim.x * 256) {
    float n[4];
    philox_normal4(key, (uint32_t)q, (uint32_t)ga.group[c], 0u, TAG_ROOT, n);
    dst[q] = make_float4(n[0], n[1], n[2], n[3]);
  }
}

// One block column per parent (blockIdx.y); KC = children per parent handled in
// registers.  partials[(b*KC + k) * gridDim.x + blockIdx.x] = block sum of xi^2.
template <int KC>
__global__ __launch_bounds__(256) void sde_step_kernel(float* __restrict__ z, const float* __restrict__ v, int v_compact,
                                                       long long D, int n_nodes, int off_p, int off_c, int width_p,
                                                       int is_split, StepCoef cf, PhiloxKey key, int step,
                                                       float* __restrict__ partials) {
  __shared__ float red[4];
  const int b = blockIdx.y;
  const int c = b / width_p, j = b - c * width_p;
  const int prow = c * n_nodes + off_p + j;
  const int crow0 = c * n_nodes + off_c + (is_split ? j * KC : j);
  const float4* zp = reinterpret_cast<const float4*>(z + (size_t)prow * D);
  const float4* vp = reinterpret_cast<const float4*>(v + (size_t)(v_compact ? b : prow) * D);
  const long long nq = D >> 2;
  float acc[KC];
#pragma unroll
  for (int k = 0; k < KC; ++k) acc[k] = 0.f;
  for (long long q = (long long)blockIdx.x * 256 + threadIdx.x; q < nq; q += (long long)gridDim.x * 256) {
    const float4 zz = zp[q], vv = vp[q];
    float mu[4] = {fmaf(cf.a_z, zz.x, cf.a_v * vv.x), fmaf(cf.a_z, zz.y, cf.a_v * vv.y),
                   fmaf(cf.a_z, zz.z, cf.a_v * vv.z), fmaf(cf.a_z, zz.w, cf.a_v * vv.w)};
    float x0[4] = {0.f, 0.f, 0.f, 0.f};
    if (cf.noise && is_split) philox_normal4(key, (uint32_t)q, (uint32_t)prow, (uint32_t)step, TAG_XI0, x0);
#pragma unroll
    for (int k = 0; k < KC; ++k) {
      float xi[4] = {0.f, 0.f, 0.f, 0.f};
      if (cf.noise) {
        philox_normal4(key, (uint32_t)q, (uint32_t)(crow0 + k), (uint32_t)step, TAG_ETA, xi);
        if (is_split) {
#pragma unroll
          for (int e = 0; e < 4; ++e) xi[e] = cf.ca * x0[e] + cf.cb * xi[e];
        }
      }
      float4 o;
      o.x = fmaf(cf.std, xi[0], mu[0]);
      o.y = fmaf(cf.std, xi[1], mu[1]);
      o.z = fmaf(cf.std, xi[2], mu[2]);
      o.w = fmaf(cf.std, xi[3], mu[3]);
      reinterpret_cast<float4*>(z + (size_t)(crow0 + k) * D)[q] = o;
      acc[k] += (xi[0] * xi[0] + xi[1] * xi[1]) + (xi[2] * xi[2] + xi[3] * xi[3]);
    }
  }
#pragma unroll
  for (int k = 0; k < KC; ++k) {
    const float s = block_sum_256(acc[k], red);
    if (threadIdx.x == 0) partials[((size_t)b * KC + k) * gridDim.x + blockIdx.x] = s;
  }
}

// Any K: one child per blockIdx.z, the parent is re-read per child.
__global__ __launch_bounds__(256) void sde_step_kernel_anyk(float* __restrict__ z, const float* __restrict__ v,
                                                            int v_compact, long long D, int n_nodes, int off_p,
                                                            int off_c, int width_p, int K, StepCoef cf, PhiloxKey key,
                                                            int step, float* __restrict__ partials) {
  __shared__ float red[4];
  const int b = blockIdx.y, k = blockIdx.z;
  const int c = b / width_p, j = b - c * width_p;
  const int prow = c * n_nodes + off_p + j;
  const int crow = c * n_nodes + off_c + j * K + k;
  const float4* zp = reinterpret_cast<const float4*>(z + (size_t)prow * D);
  const float4* vp = reinterpret_cast<const float4*>(v + (size_t)(v_compact ? b : prow) * D);
  const long long nq = D >> 2;
  float acc = 0.f;
  for (long long q = (long long)blockIdx.x * 256 + threadIdx.x; q < nq; q += (long long)gridDim.x * 256) {
    const float4 zz = zp[q], vv = vp[q];
    float xi[4] = {0.f, 0.f, 0.f, 0.f};
    if (cf.noise) {
      float x0[4];
      philox_normal4(key, (uint32_t)q, (uint32_t)prow, (uint32_t)step, TAG_XI0, x0);
      philox_normal4(key, (uint32_t)q, (uint32_t)crow, (uint32_t)step, TAG_ETA, xi);
#pragma unroll
      for (int e = 0; e < 4; ++e) xi[e] = cf.ca * x0[e] + cf.cb * xi[e];
    }
    float4 o;
    o.x = fmaf(cf.std, xi[0], fmaf(cf.a_z, zz.x, cf.a_v * vv.x));
    o.y = fmaf(cf.std, xi[1], fmaf(cf.a_z, zz.y, cf.a_v * vv.y));
    o.z = fmaf(cf.std, xi[2], fmaf(cf.a_z, zz.z, cf.a_v * vv.z));
    o.w = fmaf(cf.std, xi[3], fmaf(cf.a_z, zz.w, cf.a_v * vv.w));
    reinterpret_cast<float4*>(z + (size_t)crow * D)[q] = o;
    acc += (xi[0] * xi[0] + xi[1] * xi[1]) + (xi[2] * xi[2] + xi[3] * xi[3]);
  }
  const float s = block_sum_256(acc, red);
  if (threadIdx.x == 0) partials[((size_t)b * K + k) * gridDim.x + blockIdx.x] = s;
}

// logp of child (b, k): -scale * sum(partials) + c0, one wave per child.
// out index: explicit ids[] (global rows or edge slots) or the frontier formula.
__global__ __launch_bounds__(64) void logp_finalize_kernel(const float* __restrict__ partials, int nblk, int n_items,
                                                           double scale, double c0, double inv_div, int noise,
                                                           float* __restrict__ out, const int* __restrict__ ids,
                                                           int n_nodes, int off_c, int width_c) {
  const int item = blockIdx.x;
  if (item >= n_items) return;
  float s = 0.f;
  for (int i = threadIdx.x; i < nblk; i += 64) s += partials[(size_t)item * nblk + i];
  s = wave_sum(s);
  if (threadIdx.x == 0) {
    const int dst = ids ? ids[item] : (item / width_c) * n_nodes + off_c + item % width_c;
    out[dst] = noise ? (float)((c0 - scale * (double)s) * inv_div) : 0.f;
  }
}

// Re-evaluation: squared distance of the stored child to the new mean.
// edge e: child row crow[e], parent row prow[e], velocity row vrow[e] of v.
__global__ __launch_bounds__(256) void logp_eval_kernel(const float* __restrict__ z, const float* __restrict__ v,
                                                        long long D, const int* __restrict__ crow,
                                                        const int* __restrict__ prow, const int* __restrict__ vrow,
                                                        StepCoef cf, float* __restrict__ partials) {
  __shared__ float red[4];
  const int e = blockIdx.y;
  const float4* zc = reinterpret_cast<const float4*>(z + (size_t)crow[e] * D);
  const float4* zp = reinterpret_cast<const float4*>(z + (size_t)prow[e] * D);
  const float4* vp = reinterpret_cast<const float4*>(v + (size_t)vrow[e] * D);
  const long long nq = D >> 2;
  float acc = 0.f;
  for (long long q = (long long)blockIdx.x * 256 + threadIdx.x; q < nq; q += (long long)gridDim.x * 256) {
    const float4 a = zc[q], zz = zp[q], vv = vp[q];
    const float d0 = a.x - fmaf(cf.a_z, zz.x, cf.a_v * vv.x);
    const float d1 = a.y - fmaf(cf.a_z, zz.y, cf.a_v * vv.y);
    const float d2 = a.z - fmaf(cf.a_z, zz.z, cf.a_v * vv.z);
    const float d3 = a.w - fmaf(cf.a_z, zz.w, cf.a_v * vv.w);
    acc += (d0 * d0 + d1 * d1) + (d2 * d2 + d3 * d3);
  }
  const float s = block_sum_256(acc, red);
  if (threadIdx.x == 0) partials[(size_t)e * gridDim.x + blockIdx.x] = s;
}

__global__ void noise_stream_kernel(PhiloxKey key, uint32_t node, uint32_t step, uint32_t tag, long long nq,
                                    uint32_t* __restrict__ words, float* __restrict__ normals) {
  for (long long q = (long long)blockIdx.x * blockDim.x + threadIdx.x; q < nq; q += (long long)gridDim.x * blockDim.x) {
    if (words) {
      uint32_t w[4];
      philox4x32_10(key, (uint32_t)q, node, step, tag, w);
      reinterpret_cast<uint4*>(words)[q] = make_uint4(w[0], w[1], w[2], w[3]);
    }
    if (normals) {
      float n[4];
      philox_normal4(key, (uint32_t)q, node, step, tag, n);
      reinterpret_cast<float4*>(normals)[q] = make_float4(n[0], n[1], n[2], n[3]);
    }
  }
}

__global__ void fill_zero_kernel(float* __restrict__ p, long long n) {
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (long long)gridDim.x * blockDim.x)
    p[i] = 0.f;
}

// ---------------------------------------------------------------- host side

int sde_nblk(long long D) {
  long long nb = (D / 4 + 255) / 256;
  return (int)(nb < 1 ? 1 : (nb > 1024 ? 1024 : nb));
}

StepCoef step_coef(const br_sched* s, int i, long long D) {
  StepCoef c;
  const double ti = s->t[i], h = (double)s->t[i] - (double)s->t[i + 1], sg = s->sigma[i];
  const double g = h * sg * sg / (2.0 * ti);
  c.a_z = (float)(1.0 - g);
  c.a_v = (float)(-h - g * (1.0 - ti));
  const double sd = sg * sqrt(h);
  c.std = (float)sd;
  const double ss = s->s;
  c.ca = (float)(1.0 / sqrt(1.0 + ss * ss));
  c.cb = (float)(ss / sqrt(1.0 + ss * ss));
  c.noise = sd > 0.0 ? 1 : 0;
  c.c0 = c.noise ? -(double)D * log(sd) - 0.5 * (double)D * log(2.0 * M_PI) : 0.0;
  c.inv_div = s->logp_reduce == BR_LOGP_MEAN ? 1.0 / (double)D : 1.0;
  c.inv_2var = c.noise ? 1.0 / (2.0 * sd * sd) : 0.0;
  return c;
}

br_status launch_root_noise(const br_tree* t, uint64_t seed, const int* noise_group, long long D, float* z,
                            hipStream_t st) {
  const PhiloxKey key = philox_key(seed);
  const int nblk = sde_nblk(D);
  for (int c0 = 0; c0 < t->n_tree; c0 += 256) {
    RootArgs ga;
    const int n = std::min(256, t->n_tree - c0);
    for (int i = 0; i < n; ++i) ga.group[i] = noise_group[c0 + i];
    hipLaunchKernelGGL(root_noise_kernel, dim3(nblk, n), dim3(256), 0, st, z, D, t->n_nodes, c0, ga, key);
    BR_LAUNCH_CHECK();
  }
  return BR_OK;
}

br_status launch_sde_step(const br_tree* t, const br_sched* s, uint64_t seed, int i, long long D, const float* v,
                          int v_compact, float* z, float* logp, float* partials, hipStream_t st) {
  const StepCoef cf = step_coef(s, i, D);
  const PhiloxKey key = philox_key(seed);
  const int nblk = sde_nblk(D);
  const int n_par = t->n_tree * t->width[i];
  const int split = t->is_split[i];
  const int K = split ? t->K : 1;
  const int off_p = t->off[i], off_c = t->off[i + 1];
  BR_REQUIRE(n_par <= 65535, BR_ESHAPE, "sde step: more than 65535 parents in one depth are not supported");
  dim3 grid(nblk, n_par);
  // algorithmic bytes: z and v of every parent read once, every child written once
  ProfScope ps(st, PROF_SDE_STEP, (double)n_par * (2.0 + K) * 4.0 * (double)D);
#define BR_SDE_ARGS z, v, v_compact, (long long)D, t->n_nodes, off_p, off_c, t->width[i], split, cf, key, i, partials
  if (K == 1) hipLaunchKernelGGL(sde_step_kernel<1>, grid, dim3(256), 0, st, BR_SDE_ARGS);
  else if (K == 2) hipLaunchKernelGGL(sde_step_kernel<2>, grid, dim3(256), 0, st, BR_SDE_ARGS);
  else if (K == 3) hipLaunchKernelGGL(sde_step_kernel<3>, grid, dim3(256), 0, st, BR_SDE_ARGS);
  else if (K == 4) hipLaunchKernelGGL(sde_step_kernel<4>, grid, dim3(256), 0, st, BR_SDE_ARGS);
  else {
    BR_REQUIRE(K <= 65535, BR_ESHAPE, "sde step: K too large");
    hipLaunchKernelGGL(sde_step_kernel_anyk, dim3(nblk, n_par, K), dim3(256), 0, st, z, v, v_compact, (long long)D,
                       t->n_nodes, off_p, off_c, t->width[i], K, cf, key, i, partials);
  }
#undef BR_SDE_ARGS
  BR_LAUNCH_CHECK();
  if (ps.on) { prof_end(st); ps.on = false; }
  const int n_child = n_par * K;
  hipLaunchKernelGGL(logp_finalize_kernel, dim3(n_child), dim3(64), 0, st, partials, nblk, n_child, 0.5, cf.c0,
                     cf.inv_div, cf.noise, logp, (const int*)nullptr, t->n_nodes, off_c, t->width[i + 1]);
  BR_LAUNCH_CHECK();
  return BR_OK;
}

br_status launch_logp_eval(const br_sched* s, int i, long long D, const float* z, const float* v, const int* crow,
                           const int* prow, const int* vrow, const int* out_slot, int n_edges, float* logp_out,
                           float* partials, hipStream_t st) {
  if (n_edges == 0) return BR_OK;
  const StepCoef cf = step_coef(s, i, D);
  const int nblk = sde_nblk(D);
  BR_REQUIRE(n_edges <= 65535, BR_ESHAPE, "logprob: more than 65535 kept edges in one depth are not supported");
  ProfScope ps(st, PROF_LOGP_EVAL, (double)n_edges * 3.0 * 4.0 * (double)D);
  hipLaunchKernelGGL(logp_eval_kernel, dim3(nblk, n_edges), dim3(256), 0, st, z, v, (long long)D, crow, prow, vrow, cf,
                     partials);
  BR_LAUNCH_CHECK();
  if (ps.on) { prof_end(st); ps.on = false; }
  hipLaunchKernelGGL(logp_finalize_kernel, dim3(n_edges), dim3(64), 0, st, partials, nblk, n_edges, cf.inv_2var, cf.c0,
                     cf.inv_div, cf.noise, logp_out, out_slot, 0, 0, 1);
  BR_LAUNCH_CHECK();
  return BR_OK;
}

br_status launch_fill_zero(float* p, long long n, hipStream_t st) {
  if (n <= 0) return BR_OK;
  const int nb = (int)std::min<long long>((n + 255) / 256, 4096);
  hipLaunchKernelGGL(fill_zero_kernel, dim3(nb), dim3(256), 0, st, p, n);
  BR_LAUNCH_CHECK();
  return BR_OK;
}

br_status launch_noise_stream(uint64_t seed, uint32_t node, uint32_t step, uint32_t tag, long long nq, uint32_t* words,
                              float* normals, hipStream_t st) {
  if (nq <= 0) return BR_OK;
  const int nb = (int)std::min<long long>((nq + 255) / 256, 4096);
  hipLaunchKernelGGL(noise_stream_kernel, dim3(nb), dim3(256), 0, st, philox_key(seed), node, step, tag, nq, words,
                     normals);
  BR_LAUNCH_CHECK();
  return BR_OK;
}

}  // namespace br
