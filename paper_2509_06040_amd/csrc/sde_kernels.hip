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

// Sum over a block of NT threads in a fixed order; result valid in thread 0.
template <int NT>
__device__ inline float block_sum(float x, float* lds) {
  x = wave_sum(x);
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  __syncthreads();
  if (lane == 0) lds[wv] = x;
  __syncthreads();
  float s = 0.f;
  if (threadIdx.x == 0) {
#pragma unroll
    for (int w = 0; w < NT / 64; w += 2) s += lds[w] + lds[w + 1];
  }
  return s;
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

// ---- log-prob reduction inside the producing kernel.  The sum over a child's D elements is
// spread over the blocks of one grid row.  Every block adds its share to one 64-bit word per
// child with a single device-scope atomic: bits 11..63 hold the sum in fixed point (2^-12
// units; integer addition, so the total does not depend on the order in which blocks arrive),
// bits 0..10 count the blocks that have arrived (at most 1024 per child).  The atomic returns
// the word as it was, so the block that arrives last knows it is last and knows the complete
// sum: it writes the log-prob and stores 0 back, which leaves the word ready for the next
// launch.  Words must be zero before the first launch.  No block reads what another block
// wrote except through that atomic, so no fence is needed (a device-scope release would write
// back every dirty L2 line of the compute die, i.e. the child latents just stored: measured
// 3x the kernel time).
constexpr int kSumShift = 11;
constexpr double kSumScale = 4096.0;

// s >= 0: the block's share; returns true (thread 0 only) when this block is the last of nblk,
// with the complete sum in *total.
__device__ inline bool accumulate_share(unsigned long long* word, float s, int nblk, double* total) {
  const unsigned long long cap = ((1ull << 53) - 1) / (unsigned)nblk;  // a saturated total cannot wrap
  const double f = (double)s * kSumScale + 0.5;
  unsigned long long q = f < 9.0e15 ? (unsigned long long)f : cap;     // (NaN compares false: saturates)
  q = q < cap ? q : cap;
  const unsigned long long mine = (q << kSumShift) | 1ull;
  const unsigned long long old = __hip_atomic_fetch_add(word, mine, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  if ((int)(old & ((1u << kSumShift) - 1)) != nblk - 1) return false;
  *total = (double)((old + mine) >> kSumShift) * (1.0 / kSumScale);
  __hip_atomic_store(word, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  return true;
}

// One grid row per parent (blockIdx.y); KC = children per parent handled in registers; a thread
// has UNR quads of z and of v in flight and walks the row with the grid's stride.  The last
// block of a row writes logp of the parent's KC children: (c0 - sum xi^2 / 2) * inv_div, 0 on
// a deterministic step.  words: one per child, index b*KC + k.
template <int KC, int UNR, int NT>
__global__ __launch_bounds__(NT) void sde_step_kernel(float* __restrict__ z, const float* __restrict__ v, int v_compact,
                                                       long long D, int n_nodes, int off_p, int off_c, int width_p,
                                                       int is_split, StepCoef cf, PhiloxKey key, int step,
                                                       unsigned long long* __restrict__ words, float* __restrict__ logp) {
  __shared__ float red[NT / 64];
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
  for (long long q0 = (long long)blockIdx.x * (NT * UNR) + threadIdx.x; q0 < nq; q0 += (long long)gridDim.x * (NT * UNR)) {
    float4 zz[UNR], vv[UNR];
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      const long long q = q0 + u * NT;
      if (q < nq) {
        zz[u] = zp[q];
        vv[u] = vp[q];
      }
    }
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      const long long q = q0 + u * NT;
      if (q >= nq) break;
      float mu[4] = {fmaf(cf.a_z, zz[u].x, cf.a_v * vv[u].x), fmaf(cf.a_z, zz[u].y, cf.a_v * vv[u].y),
                     fmaf(cf.a_z, zz[u].z, cf.a_v * vv[u].z), fmaf(cf.a_z, zz[u].w, cf.a_v * vv[u].w)};
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
  }
  float s[KC];
#pragma unroll
  for (int k = 0; k < KC; ++k) s[k] = block_sum<NT>(acc[k], red);
  if (threadIdx.x == 0) {
#pragma unroll
    for (int k = 0; k < KC; ++k) {
      double tot;
      if (accumulate_share(words + (size_t)b * KC + k, s[k], gridDim.x, &tot))
        logp[crow0 + k] = cf.noise ? (float)((cf.c0 - 0.5 * tot) * cf.inv_div) : 0.f;
    }
  }
}

// Any K: one child per blockIdx.z, the parent is re-read per child.
__global__ __launch_bounds__(256) void sde_step_kernel_anyk(float* __restrict__ z, const float* __restrict__ v,
                                                            int v_compact, long long D, int n_nodes, int off_p,
                                                            int off_c, int width_p, int K, StepCoef cf, PhiloxKey key,
                                                            int step, unsigned long long* __restrict__ words,
                                                            float* __restrict__ logp) {
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
  const float s = block_sum<256>(acc, red);
  double tot;
  if (threadIdx.x == 0 && accumulate_share(words + (size_t)b * K + k, s, gridDim.x, &tot))
    logp[crow] = cf.noise ? (float)((cf.c0 - 0.5 * tot) * cf.inv_div) : 0.f;
}

// Re-evaluation: distance of the stored child to the new mean in units of the step's standard
// deviation; the last block of an edge writes logp_out[slot[e]] = (c0 - sum / 2) * inv_div
// (0 on a deterministic step).  edge e: child row crow[e], parent row prow[e], velocity row
// vrow[e] of v.
template <int UNR, int NT>
__global__ __launch_bounds__(NT) void logp_eval_kernel(const float* __restrict__ z, const float* __restrict__ v,
                                                        long long D, const int* __restrict__ crow,
                                                        const int* __restrict__ prow, const int* __restrict__ vrow,
                                                        const int* __restrict__ slot, StepCoef cf,
                                                        unsigned long long* __restrict__ words,
                                                        float* __restrict__ logp_out) {
  __shared__ float red[NT / 64];
  const int e = blockIdx.y;
  const float4* zc = reinterpret_cast<const float4*>(z + (size_t)crow[e] * D);
  const float4* zp = reinterpret_cast<const float4*>(z + (size_t)prow[e] * D);
  const float4* vp = reinterpret_cast<const float4*>(v + (size_t)vrow[e] * D);
  const long long nq = D >> 2;
  const float is = cf.inv_std;
  float acc = 0.f;
  for (long long q0 = (long long)blockIdx.x * (NT * UNR) + threadIdx.x; q0 < nq; q0 += (long long)gridDim.x * (NT * UNR)) {
    float4 a[UNR], zz[UNR], vv[UNR];
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      const long long q = q0 + u * NT;
      if (q < nq) {
        a[u] = zc[q];
        zz[u] = zp[q];
        vv[u] = vp[q];
      }
    }
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      if (q0 + u * NT >= nq) break;
      const float d0 = (a[u].x - fmaf(cf.a_z, zz[u].x, cf.a_v * vv[u].x)) * is;
      const float d1 = (a[u].y - fmaf(cf.a_z, zz[u].y, cf.a_v * vv[u].y)) * is;
      const float d2 = (a[u].z - fmaf(cf.a_z, zz[u].z, cf.a_v * vv[u].z)) * is;
      const float d3 = (a[u].w - fmaf(cf.a_z, zz[u].w, cf.a_v * vv[u].w)) * is;
      acc += (d0 * d0 + d1 * d1) + (d2 * d2 + d3 * d3);
    }
  }
  const float s = block_sum<NT>(acc, red);
  double tot;
  if (threadIdx.x == 0 && accumulate_share(words + e, s, gridDim.x, &tot))
    logp_out[slot[e]] = cf.noise ? (float)((cf.c0 - 0.5 * tot) * cf.inv_div) : 0.f;
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
  c.inv_std = c.noise ? (float)(1.0 / sd) : 0.f;
  return c;
}

br_status launch_root_noise(const br_tree* t, uint64_t seed, const int* noise_group, long long D, float* z,
                            hipStream_t st) {
  const PhiloxKey key = philox_key(seed);
  const int nblk = (int)std::max<long long>(1, std::min<long long>((D / 4 + 255) / 256, 1024));
  for (int c0 = 0; c0 < t->n_tree; c0 += 256) {
    RootArgs ga;
    const int n = std::min(256, t->n_tree - c0);
    for (int i = 0; i < n; ++i) ga.group[i] = noise_group[c0 + i];
    hipLaunchKernelGGL(root_noise_kernel, dim3(nblk, n), dim3(256), 0, st, z, D, t->n_nodes, c0, ga, key);
    BR_LAUNCH_CHECK();
  }
  return BR_OK;
}

// Launch shape of the row kernels: blocks of BR_SDE_THREADS threads, BR_SDE_UNROLL quads in
// flight per thread, and as many blocks per row as give the whole grid about
// BR_SDE_BLOCKS_PER_CU blocks per compute unit.  Few, large, long-lived blocks: every block ends
// with one atomic round trip, and the blocks of a row all hit one word -- atomics of different
// compute dies on one address take about 50 ns each, one after the other (measured: 512 blocks
// per row cost 28 us at the video shape).  Block sizes 256..1024, 1..4 blocks per unit and 1..2
// quads in flight all measure within 10 % of each other at the three workload shapes.
#ifndef BR_SDE_BLOCKS_PER_CU
#define BR_SDE_BLOCKS_PER_CU 1
#endif
#ifndef BR_SDE_UNROLL
#define BR_SDE_UNROLL 1
#endif
#ifndef BR_SDE_THREADS
#define BR_SDE_THREADS 512
#endif
static int sde_grid_x(long long D, long long n_rows) {
  const long long nq = D / 4, per = (long long)BR_SDE_THREADS * BR_SDE_UNROLL;
  const long long max_x = std::min<long long>((nq + per - 1) / per, 1024);
  const long long want = ((long long)BR_SDE_BLOCKS_PER_CU * device_cu_count() + n_rows - 1) / n_rows;
  return (int)std::max<long long>(1, std::min(max_x, want));
}

size_t sde_scratch_floats(long long n_items, long long D) { (void)D; return (size_t)n_items * 2; }

br_status launch_sde_step(const br_tree* t, const br_sched* s, uint64_t seed, int i, long long D, const float* v,
                          int v_compact, float* z, float* logp, float* scratch, hipStream_t st) {
  const StepCoef cf = step_coef(s, i, D);
  const PhiloxKey key = philox_key(seed);
  const int n_par = t->n_tree * t->width[i];
  const int split = t->is_split[i];
  const int K = split ? t->K : 1;
  const int off_p = t->off[i], off_c = t->off[i + 1];
  BR_REQUIRE(n_par <= 65535, BR_ESHAPE, "sde step: more than 65535 parents in one depth are not supported");
  unsigned long long* words = reinterpret_cast<unsigned long long*>(scratch);  // one per child of the step
  dim3 grid(sde_grid_x(D, n_par), n_par);
  // algorithmic bytes: z and v of every parent read once, every child written once
  ProfScope ps(st, PROF_SDE_STEP, (double)n_par * (2.0 + K) * 4.0 * (double)D);
#define BR_SDE_ARGS z, v, v_compact, (long long)D, t->n_nodes, off_p, off_c, t->width[i], split, cf, key, i, words, logp
#define BR_SDE_LAUNCH(KC) \
  hipLaunchKernelGGL((sde_step_kernel<KC, BR_SDE_UNROLL, BR_SDE_THREADS>), grid, dim3(BR_SDE_THREADS), 0, st, BR_SDE_ARGS)
  if (K == 1) BR_SDE_LAUNCH(1);
  else if (K == 2) BR_SDE_LAUNCH(2);
  else if (K == 3) BR_SDE_LAUNCH(3);
  else if (K == 4) BR_SDE_LAUNCH(4);
  else {
    BR_REQUIRE(K <= 65535, BR_ESHAPE, "sde step: K too large");
    const long long nb = std::min<long long>((D / 4 + 255) / 256, 1024);
    const int gx = (int)std::max<long long>(1, std::min(nb, (2LL * device_cu_count() + (long long)n_par * K - 1) / ((long long)n_par * K)));
    hipLaunchKernelGGL(sde_step_kernel_anyk, dim3(gx, n_par, K), dim3(256), 0, st, z, v, v_compact, (long long)D,
                       t->n_nodes, off_p, off_c, t->width[i], K, cf, key, i, words, logp);
  }
#undef BR_SDE_LAUNCH
#undef BR_SDE_ARGS
  BR_LAUNCH_CHECK();
  return BR_OK;
}

br_status launch_logp_eval(const br_sched* s, int i, long long D, const float* z, const float* v, const int* crow,
                           const int* prow, const int* vrow, const int* out_slot, int n_edges, long long n_items,
                           float* logp_out, float* scratch, hipStream_t st) {
  if (n_edges == 0) return BR_OK;
  const StepCoef cf = step_coef(s, i, D);
  BR_REQUIRE(n_edges <= 65535 && n_edges <= n_items, BR_ESHAPE, "logprob: too many kept edges in one depth");
  unsigned long long* words = reinterpret_cast<unsigned long long*>(scratch);
  ProfScope ps(st, PROF_LOGP_EVAL, (double)n_edges * 3.0 * 4.0 * (double)D);
  hipLaunchKernelGGL((logp_eval_kernel<BR_SDE_UNROLL, BR_SDE_THREADS>), dim3(sde_grid_x(D, n_edges), n_edges),
                     dim3(BR_SDE_THREADS), 0, st, z, v, (long long)D, crow, prow, vrow, out_slot, cf, words, logp_out);
  BR_LAUNCH_CHECK();
  return BR_OK;
}

// Zeroes the words of a scratch area laid out for n_items (once per call of an entry point).
br_status launch_sde_scratch_reset(float* scratch, long long n_items, long long D, hipStream_t st) {
  return launch_fill_zero(scratch, (long long)sde_scratch_floats(n_items, D), st);
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
