// Velocity network: the memory-bound and small kernels (sample maps, patchify,
// condition broadcast, conditioning path, LayerNorm-modulate) and the fp32 GEMM /
// attention used by BR_F32 models.  The bf16 MFMA GEMM and flash attention live in
// gemm_bf16.hip and attn_bf16.hip.
#include "common.h"
#include "dit.h"
#include "prof.h"

namespace br {

template <typename T>
__device__ inline float to_f(T v) { return (float)v; }

// ------------------------------------------------------------- sample maps
__global__ void sample_map_kernel(SampleMap sm, int b0, int B, int v_rows_mode, int* __restrict__ rowmap,
                                  int* __restrict__ condmap, int* __restrict__ modmap, int* __restrict__ vrows) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= B) return;
  const int b = b0 + i;
  const int row = sm.rows ? sm.rows[b] : (b / sm.width) * sm.n_nodes + sm.off + b % sm.width;
  const int c = sm.cond ? sm.cond[b] : b / sm.width;
  rowmap[i] = row;
  condmap[i] = c;
  modmap[i] = sm.group ? sm.group[b] : c;
  vrows[i] = v_rows_mode == 1 ? row : (v_rows_mode == 2 ? i : b);  // arena row / row of this batch / frontier index
}

// One modulation group per condition, all at time t.
__global__ void uniform_groups_kernel(float t, int n_cond, int* __restrict__ gcond, float* __restrict__ gt) {
  const int g = blockIdx.x * blockDim.x + threadIdx.x;
  if (g >= n_cond) return;
  gcond[g] = g;
  gt[g] = t;
}

// ---------------------------------------------------------------- patchify
// patches[(b n_img + tok) pd + el] = z[rowmap[b]][latent index]; tokens in (t,h,w)
// raster order, patch vector in (c, dt, dh, dw) order.
template <typename T>
__global__ __launch_bounds__(256) void patchify_kernel(const float* __restrict__ z, const int* __restrict__ rowmap,
                                                       long long D, int n_img, int pd, int lt, int lh, int lw, int pt,
                                                       int ph, int pw, int gh, int gw, long long total,
                                                       T* __restrict__ out) {
  for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < total; i += (long long)gridDim.x * 256) {
    const int el = (int)(i % pd);
    const long long bt = i / pd;
    const int tok = (int)(bt % n_img), b = (int)(bt / n_img);
    const int tw = tok % gw, th = (tok / gw) % gh, tt = tok / (gw * gh);
    const int dw = el % pw, dh = (el / pw) % ph, dt = (el / (pw * ph)) % pt, c = el / (pw * ph * pt);
    const long long idx = (((long long)c * lt + tt * pt + dt) * lh + th * ph + dh) * lw + tw * pw + dw;
    out[i] = (T)z[(size_t)rowmap[b] * D + idx];
  }
}

// x[b, n_img + j, :] = cond_emb[condmap[b], j, :]
__global__ __launch_bounds__(256) void cond_broadcast_kernel(const float* __restrict__ cond_emb,
                                                             const int* __restrict__ condmap, int L, int n_img, int Nc,
                                                             int H, long long total4, float* __restrict__ x) {
  const int H4 = H >> 2;
  for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < total4; i += (long long)gridDim.x * 256) {
    const int h4 = (int)(i % H4);
    const long long bj = i / H4;
    const int j = (int)(bj % Nc), b = (int)(bj / Nc);
    const float4 v = reinterpret_cast<const float4*>(cond_emb)[((size_t)condmap[b] * Nc + j) * H4 + h4];
    reinterpret_cast<float4*>(x)[((size_t)b * L + n_img + j) * H4 + h4] = v;
  }
}

// ------------------------------------------------------- conditioning path
// temb = [cos(1000 t f_k), sin(1000 t f_k)], f_k = 10000^(-k/128).  The angle (up to 1000 rad)
// is formed and reduced to [-pi, pi] in fp64, then fp32 sin/cos suffice.
__device__ inline float silu_f(float x) { return x / (1.f + __expf(-x)); }

__global__ __launch_bounds__(128) void temb_kernel(const float* __restrict__ gt, float* __restrict__ temb) {
  const int k = threadIdx.x, g = blockIdx.x;
  const double f = exp(-9.210340371976184 * (double)k / 128.0);  // ln 10000
  double a = 1000.0 * (double)gt[g] * f;
  a -= 6.283185307179586 * rint(a * 0.15915494309189535);
  float sn, cs;
  sincosf((float)a, &sn, &cs);
  temb[(size_t)g * 256 + k] = cs;
  temb[(size_t)g * 256 + 128 + k] = sn;
}

// cvec[g, :] = silu(pool_lin[gcond[g], :] + ct[g, :])
__global__ __launch_bounds__(256) void group_cvec_kernel(const float* __restrict__ pool_lin,
                                                         const float* __restrict__ ct, const int* __restrict__ gcond,
                                                         int H, float* __restrict__ cvec) {
  const int g = blockIdx.y, h = blockIdx.x * 256 + threadIdx.x;
  if (h >= H) return;
  cvec[(size_t)g * H + h] = silu_f(pool_lin[(size_t)gcond[g] * H + h] + ct[(size_t)g * H + h]);
}

// pooled[c, :] = mean over the condition tokens of condition c (depends on the prompt only)
template <typename T>
__global__ __launch_bounds__(256) void pool_kernel(const T* __restrict__ cond, int Nc, int cd,
                                                   float* __restrict__ pooled) {
  const int c = blockIdx.y, d = blockIdx.x * 256 + threadIdx.x;
  if (d >= cd) return;
  float s = 0.f;
  for (int j = 0; j < Nc; ++j) s += to_f(cond[((size_t)c * Nc + j) * cd + d]);
  pooled[(size_t)c * cd + d] = s / (float)Nc;
}

template <typename TW>
struct WChunk;  // eight consecutive weights as floats
template <>
struct WChunk<float> {
  static __device__ inline void load(const float* p, float* w) {
    const float4 a = *reinterpret_cast<const float4*>(p), b = *reinterpret_cast<const float4*>(p + 4);
    w[0] = a.x; w[1] = a.y; w[2] = a.z; w[3] = a.w; w[4] = b.x; w[5] = b.y; w[6] = b.z; w[7] = b.w;
  }
};
template <>
struct WChunk<bf16> {
  static __device__ inline void load(const bf16* p, float* w) {
    typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
    const bf16x8_t v = *reinterpret_cast<const bf16x8_t*>(p);
#pragma unroll
    for (int e = 0; e < 8; ++e) w[e] = (float)v[e];
  }
};

// out[r, n] = post( sum_k pre(in[r, k]) W[n, k] + bias[n] + add[n] ), r < R <= 8.
// Weight-streaming: one wavefront per output column, lanes along k in 8-element chunks
// (K % 8 == 0, rows 16-byte aligned).
template <typename TW, int R>
__global__ __launch_bounds__(256) void skinny_gemm_kernel(const float* __restrict__ in, int ldi,
                                                          const TW* __restrict__ W, int K, int N,
                                                          const float* __restrict__ bias,
                                                          const float* __restrict__ add, int pre_silu, int post_silu,
                                                          float* __restrict__ out, int ldo) {
  const int lane = threadIdx.x & 63;
  const int n = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (n >= N) return;
  float acc[R];
#pragma unroll
  for (int r = 0; r < R; ++r) acc[r] = 0.f;
  const TW* wr = W + (size_t)n * K;
  for (int k = lane * 8; k < K; k += 512) {
    float w[8];
    WChunk<TW>::load(wr + k, w);
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const float4 a0 = *reinterpret_cast<const float4*>(in + (size_t)r * ldi + k);
      const float4 a1 = *reinterpret_cast<const float4*>(in + (size_t)r * ldi + k + 4);
      float a[8] = {a0.x, a0.y, a0.z, a0.w, a1.x, a1.y, a1.z, a1.w};
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float x = pre_silu ? silu_f(a[e]) : a[e];
        acc[r] = fmaf(x, w[e], acc[r]);
      }
    }
  }
#pragma unroll
  for (int r = 0; r < R; ++r) {
    float s = acc[r];
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) s += __shfl_down(s, o, 64);
    if (lane == 0) {
      s += bias[n] + (add ? add[n] : 0.f);
      out[(size_t)r * ldo + n] = post_silu ? silu_f(s) : s;
    }
  }
}

template <typename TW>
static br_status skinny(const float* in, int ldi, int R, const TW* W, int K, int N, const float* bias, const float* add,
                        int pre, int post, float* out, int ldo, hipStream_t st) {
  for (int r0 = 0; r0 < R; r0 += 8) {
    const int r = std::min(8, R - r0);
    const float* ip = in + (size_t)r0 * ldi;
    float* op = out + (size_t)r0 * ldo;
    dim3 g(cdiv(N, 4)), b(256);
#define BR_SK(RR) hipLaunchKernelGGL((skinny_gemm_kernel<TW, RR>), g, b, 0, st, ip, ldi, W, K, N, bias, add, pre, post, op, ldo)
    switch (r) {
      case 1: BR_SK(1); break;
      case 2: BR_SK(2); break;
      case 3: BR_SK(3); break;
      case 4: BR_SK(4); break;
      case 5: BR_SK(5); break;
      case 6: BR_SK(6); break;
      case 7: BR_SK(7); break;
      default: BR_SK(8); break;
    }
#undef BR_SK
    BR_LAUNCH_CHECK();
  }
  return BR_OK;
}

// Per modulation group g: cvec = silu(t_mlp(temb(gt[g])) + pool_lin[gcond[g]]); mods = ada_lin(cvec).
template <typename T>
static br_status conditioning_t(const br_model* m, const FwdBuffers& fb, const int* gcond, const float* gt, int G,
                                hipStream_t st) {
  const int H = m->H;
  hipLaunchKernelGGL(temb_kernel, dim3(G), dim3(128), 0, st, gt, fb.temb);
  BR_LAUNCH_CHECK();
  br_status s;
  if ((s = skinny<T>(fb.temb, 256, G, (const T*)m->w[BR_W_T1_W], 256, H, (const float*)m->w[BR_W_T1_B], nullptr, 0, 1,
                     fb.h1, H, st)) != BR_OK) return s;
  if ((s = skinny<T>(fb.h1, H, G, (const T*)m->w[BR_W_T2_W], H, H, (const float*)m->w[BR_W_T2_B], nullptr, 0, 0, fb.ct,
                     H, st)) != BR_OK) return s;
  hipLaunchKernelGGL(group_cvec_kernel, dim3(cdiv(H, 256), G), dim3(256), 0, st, fb.pool_lin, fb.ct, gcond, H, fb.cvec);
  BR_LAUNCH_CHECK();
  // the modulation vectors of all blocks: a GEMV that streams the [A, H] weights once per 8 groups
  ProfScope ps(st, PROF_ADALN, (double)cdiv(G, 8) * (double)m->A * H * sizeof(T));
  return skinny<T>(fb.cvec, H, G, (const T*)m->w[BR_W_ADA_W], H, m->A, (const float*)m->w[BR_W_ADA_B], nullptr, 0, 0,
                   fb.mods, m->A, st);
}

// pool_lin[c, :] = W_pool pooled[c, :] + b_pool: the time-independent half of the conditioning vector
br_status launch_pool_linear(const br_model* m, const FwdBuffers& fb, int n_cond, hipStream_t st) {
  if (m->cfg.dtype == BR_BF16)
    return skinny<bf16>(fb.pooled, m->cd, n_cond, (const bf16*)m->w[BR_W_POOL_W], m->cd, m->H,
                        (const float*)m->w[BR_W_POOL_B], nullptr, 0, 0, fb.pool_lin, m->H, st);
  return skinny<float>(fb.pooled, m->cd, n_cond, (const float*)m->w[BR_W_POOL_W], m->cd, m->H,
                       (const float*)m->w[BR_W_POOL_B], nullptr, 0, 0, fb.pool_lin, m->H, st);
}

br_status launch_uniform_groups(const FwdBuffers& fb, float t, int n_cond, hipStream_t st) {
  hipLaunchKernelGGL(uniform_groups_kernel, dim3(cdiv(n_cond, 256)), dim3(256), 0, st, t, n_cond, fb.gcond, fb.gt);
  BR_LAUNCH_CHECK();
  return BR_OK;
}

br_status launch_pool(const br_model* m, const FwdBuffers& fb, const void* cond, int n_cond, hipStream_t st) {
  dim3 g(cdiv(m->cd, 256), n_cond), b(256);
  if (m->cfg.dtype == BR_BF16)
    hipLaunchKernelGGL((pool_kernel<bf16>), g, b, 0, st, (const bf16*)cond, m->Nc, m->cd, fb.pooled);
  else
    hipLaunchKernelGGL((pool_kernel<float>), g, b, 0, st, (const float*)cond, m->Nc, m->cd, fb.pooled);
  BR_LAUNCH_CHECK();
  return BR_OK;
}

br_status conditioning(const br_model* m, const FwdBuffers& fb, const int* gcond, const float* gt, int G,
                       hipStream_t st) {
  return m->cfg.dtype == BR_BF16 ? conditioning_t<bf16>(m, fb, gcond, gt, G, st)
                                 : conditioning_t<float>(m, fb, gcond, gt, G, st);
}

// ------------------------------------------------------- LayerNorm-modulate
// out[r, :] = LN(x[src(r), :]) (1 + scale) + shift; one wavefront per row, the row held in
// registers (VPL float4 per lane; VPL = 0: any H, the row is re-read from cache instead).
// r = b * rows_per_sample + tok, src = b * L_in + tok; LN without affine, eps 1e-6.
template <typename T, int VPL>
__global__ __launch_bounds__(256) void ln_modulate_kernel(const float* __restrict__ x, T* __restrict__ out, int n_rows,
                                                          int rows_per_sample, int L_in, int H,
                                                          const float* __restrict__ mods, int A, int shift_off,
                                                          int scale_off, const int* __restrict__ condmap) {
  const int lane = threadIdx.x & 63;
  const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= n_rows) return;
  const int b = r / rows_per_sample, tok = r - b * rows_per_sample;
  const float4* xr = reinterpret_cast<const float4*>(x + ((size_t)b * L_in + tok) * H);
  const int H4 = H >> 2;
  float4 v[VPL > 0 ? VPL : 1];
  float s = 0.f;
  if (VPL > 0) {
#pragma unroll
    for (int i = 0; i < VPL; ++i) {
      v[i] = xr[lane + 64 * i];
      s += (v[i].x + v[i].y) + (v[i].z + v[i].w);
    }
  } else {
    for (int i = lane; i < H4; i += 64) {
      const float4 u = xr[i];
      s += (u.x + u.y) + (u.z + u.w);
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
  const float mean = s / (float)H;
  float q = 0.f;
  if (VPL > 0) {
#pragma unroll
    for (int i = 0; i < VPL; ++i) {
      const float a = v[i].x - mean, bq = v[i].y - mean, c = v[i].z - mean, d = v[i].w - mean;
      q += (a * a + bq * bq) + (c * c + d * d);
    }
  } else {
    for (int i = lane; i < H4; i += 64) {
      const float4 u = xr[i];
      const float a = u.x - mean, bq = u.y - mean, c = u.z - mean, d = u.w - mean;
      q += (a * a + bq * bq) + (c * c + d * d);
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) q += __shfl_xor(q, o, 64);
  const float rstd = 1.0f / __builtin_sqrtf(q / (float)H + 1e-6f);
  const float* mrow = mods + (size_t)condmap[b] * A;
  const float4* sh = reinterpret_cast<const float4*>(mrow + shift_off);
  const float4* sc = reinterpret_cast<const float4*>(mrow + scale_off);
  T* orow = out + (size_t)r * H;
  if (VPL > 0) {
#pragma unroll
    for (int i = 0; i < VPL; ++i) {
      const int c4 = lane + 64 * i;
      const float4 a = sh[c4], g = sc[c4];
      store4_stream(orow + 4 * c4, fmaf((v[i].x - mean) * rstd, 1.f + g.x, a.x), fmaf((v[i].y - mean) * rstd, 1.f + g.y, a.y),
                fmaf((v[i].z - mean) * rstd, 1.f + g.z, a.z), fmaf((v[i].w - mean) * rstd, 1.f + g.w, a.w));
    }
  } else {
    for (int i = lane; i < H4; i += 64) {
      const float4 u = xr[i], a = sh[i], g = sc[i];
      store4<T>(orow + 4 * i, fmaf((u.x - mean) * rstd, 1.f + g.x, a.x), fmaf((u.y - mean) * rstd, 1.f + g.y, a.y),
                fmaf((u.z - mean) * rstd, 1.f + g.z, a.z), fmaf((u.w - mean) * rstd, 1.f + g.w, a.w));
    }
  }
}

template <typename T>
static void ln_launch(dim3 g, dim3 b, hipStream_t st, const float* x, T* out, int n_rows, int rows_per_sample, int L_in,
                      int H, const float* mods, int A, int shift_off, int scale_off, const int* condmap) {
#define BR_LN(V) hipLaunchKernelGGL((ln_modulate_kernel<T, V>), g, b, 0, st, x, out, n_rows, rows_per_sample, L_in, H, \
                                    mods, A, shift_off, scale_off, condmap)
  switch (H % 256 == 0 ? H / 256 : 0) {
    case 1: BR_LN(1); break;
    case 2: BR_LN(2); break;
    case 3: BR_LN(3); break;
    case 4: BR_LN(4); break;
    case 6: BR_LN(6); break;
    case 8: BR_LN(8); break;
    case 12: BR_LN(12); break;
    default: BR_LN(0); break;
  }
#undef BR_LN
}

br_status launch_ln_modulate(int dtype, const float* x, void* out, int n_rows, int rows_per_sample, int L_in, int H,
                             const float* mods, int A, int shift_off, int scale_off, const int* condmap,
                             hipStream_t st) {
  if (n_rows == 0) return BR_OK;
  dim3 g(cdiv(n_rows, 4)), b(256);
  ProfScope ps(st, PROF_LN_MOD, (double)n_rows * H * (4.0 + (dtype == BR_BF16 ? 2.0 : 4.0)));
  if (dtype == BR_BF16)
    ln_launch<bf16>(g, b, st, x, (bf16*)out, n_rows, rows_per_sample, L_in, H, mods, A, shift_off, scale_off, condmap);
  else
    ln_launch<float>(g, b, st, x, (float*)out, n_rows, rows_per_sample, L_in, H, mods, A, shift_off, scale_off, condmap);
  BR_LAUNCH_CHECK();
  return BR_OK;
}

// --------------------------------------------------------------- fp32 GEMM
// C[m, n] = sum_k A[m, k] W[n, k]; 64x64 tile, 16-deep, 4x4 outputs per thread.
template <int MODE>
__global__ __launch_bounds__(256) void gemm_f32_kernel(const float* __restrict__ A, int lda, const float* __restrict__ W,
                                                       int ldw, int M, int N, int K, Epilogue<MODE, float> epi) {
  __shared__ float sA[16][64 + 4], sW[16][64 + 4];
  const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
  const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += 16) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int e = tid + i * 256, row = e >> 4, kk = e & 15;
      const int gm = m0 + row, gn = n0 + row, gk = k0 + kk;
      sA[kk][row] = (gm < M && gk < K) ? A[(size_t)gm * lda + gk] : 0.f;
      sW[kk][row] = (gn < N && gk < K) ? W[(size_t)gn * ldw + gk] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < 16; ++kk) {
      float a[4], w[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        a[i] = sA[kk][ty * 4 + i];
        w[i] = sW[kk][tx * 4 + i];
      }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], w[j], acc[i][j]);
    }
    __syncthreads();
  }
  const int n = n0 + tx * 4;
  if (n >= N) return;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int m = m0 + ty * 4 + i;
    if (m < M) {
      const auto r = epi.row(m);
      epi.store(r, n, acc[i][0], acc[i][1], acc[i][2], acc[i][3]);
    }
  }
}

template <int MODE>
static br_status gemm_f32_mode(const float* A, int lda, const float* W, int ldw, int M, int N, int K, const EpiArgs& ea,
                               hipStream_t st) {
  Epilogue<MODE, float> epi{ea};
  hipLaunchKernelGGL((gemm_f32_kernel<MODE>), dim3(cdiv(N, 64), cdiv(M, 64)), dim3(256), 0, st, A, lda, W, ldw, M, N, K,
                     epi);
  BR_LAUNCH_CHECK();
  return BR_OK;
}

br_status launch_gemm(int dtype, int mode, const void* A, int lda, const void* W, int ldw, int M, int N, int K,
                      const EpiArgs& ea, hipStream_t st) {
  if (M == 0) return BR_OK;
  BR_REQUIRE(N % 4 == 0, BR_ESHAPE, "gemm: N must be a multiple of 4");
  if (dtype == BR_BF16)
    return launch_gemm_bf16(mode, (const bf16*)A, lda, (const bf16*)W, ldw, M, N, K, ea, -1, st);
  const float* a = (const float*)A;
  const float* w = (const float*)W;
  switch (mode) {
    case EPI_BIAS: return gemm_f32_mode<EPI_BIAS>(a, lda, w, ldw, M, N, K, ea, st);
    case EPI_BIAS_GELU: return gemm_f32_mode<EPI_BIAS_GELU>(a, lda, w, ldw, M, N, K, ea, st);
    case EPI_BIAS_GATE_RES: return gemm_f32_mode<EPI_BIAS_GATE_RES>(a, lda, w, ldw, M, N, K, ea, st);
    case EPI_PATCH_EMBED: return gemm_f32_mode<EPI_PATCH_EMBED>(a, lda, w, ldw, M, N, K, ea, st);
    case EPI_BIAS_F32: return gemm_f32_mode<EPI_BIAS_F32>(a, lda, w, ldw, M, N, K, ea, st);
    case EPI_UNPATCH: return gemm_f32_mode<EPI_UNPATCH>(a, lda, w, ldw, M, N, K, ea, st);
  }
  return fail(BR_EINVAL, "gemm: unknown epilogue");
}

// ---------------------------------------------------------- fp32 attention
// One thread per query, streaming over all keys with an online softmax.
template <int DH>
__global__ __launch_bounds__(64) void attn_f32_kernel(const float* __restrict__ qkv, float* __restrict__ out, int L,
                                                      int H, float scale) {
  const int b = blockIdx.z, h = blockIdx.y, qi = blockIdx.x * 64 + threadIdx.x;
  const float* base = qkv + (size_t)b * L * 3 * H + h * DH;
  const bool live = qi < L;
  float q[DH], o[DH];
#pragma unroll
  for (int d = 0; d < DH; ++d) {
    q[d] = live ? base[(size_t)qi * 3 * H + d] * scale : 0.f;
    o[d] = 0.f;
  }
  float mx = -INFINITY, den = 0.f;
  for (int j = 0; j < L; ++j) {
    const float* kr = base + (size_t)j * 3 * H + H;
    const float* vr = kr + H;
    float s = 0.f;
#pragma unroll
    for (int d = 0; d < DH; ++d) s = fmaf(q[d], kr[d], s);
    const float mn = fmaxf(mx, s);
    const float alpha = __expf(mx - mn), p = __expf(s - mn);
    den = den * alpha + p;
#pragma unroll
    for (int d = 0; d < DH; ++d) o[d] = fmaf(p, vr[d], o[d] * alpha);
    mx = mn;
  }
  if (live) {
    float* orow = out + ((size_t)b * L + qi) * H + h * DH;
    const float inv = 1.f / den;
#pragma unroll
    for (int d = 0; d < DH; ++d) orow[d] = o[d] * inv;
  }
}

br_status launch_attention(int dtype, const void* qkv, void* out, int B, int L, int NH, int DH, int q_prescaled,
                           hipStream_t st) {
  if (B == 0) return BR_OK;
  if (dtype == BR_BF16) return launch_attention_bf16((const bf16*)qkv, (bf16*)out, B, L, NH, DH, q_prescaled, st);
  BR_REQUIRE(!q_prescaled, BR_EINVAL, "attention: prescaled queries are a bf16 layout");
  BR_REQUIRE(NH <= 65535 && B <= 65535, BR_ESHAPE, "attention: too many heads or samples for one launch");
  dim3 g(cdiv(L, 64), NH, B), blk(64);
  const float scale = 1.0f / sqrtf((float)DH);
  const int H = NH * DH;
#define BR_AT(D_) hipLaunchKernelGGL((attn_f32_kernel<D_>), g, blk, 0, st, (const float*)qkv, (float*)out, L, H, scale)
  switch (DH) {
    case 16: BR_AT(16); break;
    case 32: BR_AT(32); break;
    case 64: BR_AT(64); break;
    case 128: BR_AT(128); break;
    default: return fail(BR_ESHAPE, "attention: head dim must be 16, 32, 64 or 128");
  }
#undef BR_AT
  BR_LAUNCH_CHECK();
  return BR_OK;
}

// -------------------------------------------------------------- launchers
br_status fill_sample_maps(const FwdBuffers& fb, const SampleMap& smap, int b0, int B, int v_mode_rows, hipStream_t st) {
  hipLaunchKernelGGL(sample_map_kernel, dim3(cdiv(B, 256)), dim3(256), 0, st, smap, b0, B, v_mode_rows, fb.rowmap,
                     fb.condmap, fb.modmap, fb.vrows);
  BR_LAUNCH_CHECK();
  return BR_OK;
}

br_status launch_patchify(const br_model* m, const FwdBuffers& fb, const float* z, int B, hipStream_t st) {
  const long long total = (long long)B * m->n_img * m->pd;
  const int nb = (int)std::min<long long>((total + 255) / 256, 65535 * 16);
  const br_model_cfg& c = m->cfg;
  if (c.dtype == BR_BF16)
    hipLaunchKernelGGL((patchify_kernel<bf16>), dim3(nb), dim3(256), 0, st, z, fb.rowmap, m->D, m->n_img, m->pd,
                       c.latent_t, c.latent_h, c.latent_w, c.patch_t, c.patch_h, c.patch_w, m->gh, m->gw, total,
                       (bf16*)fb.patches);
  else
    hipLaunchKernelGGL((patchify_kernel<float>), dim3(nb), dim3(256), 0, st, z, fb.rowmap, m->D, m->n_img, m->pd,
                       c.latent_t, c.latent_h, c.latent_w, c.patch_t, c.patch_h, c.patch_w, m->gh, m->gw, total,
                       (float*)fb.patches);
  BR_LAUNCH_CHECK();
  return BR_OK;
}

br_status launch_cond_broadcast(const br_model* m, const FwdBuffers& fb, int B, hipStream_t st) {
  const long long total4 = (long long)B * m->Nc * (m->H / 4);
  if (total4 == 0) return BR_OK;
  const int nb = (int)std::min<long long>((total4 + 255) / 256, 65535 * 16);
  hipLaunchKernelGGL(cond_broadcast_kernel, dim3(nb), dim3(256), 0, st, fb.cond_emb, fb.condmap, m->L, m->n_img, m->Nc,
                     m->H, total4, fb.x);
  BR_LAUNCH_CHECK();
  return BR_OK;
}

}  // namespace br
