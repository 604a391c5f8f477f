// Velocity-network internals: model handle, workspace plan, epilogues, launchers.
#pragma once
#include "common.h"

typedef __bf16 bf16;

struct br_model {
  br_model_cfg cfg;
  const void* w[BR_W_COUNT];
  // derived
  int H, NB, NH, DH, R, n_img, pd, L, Nc, cd, A;  // A = NB*6H + 2H
  long long D;
  int gt, gh, gw;
};

namespace br {

// ---- epilogues of the GEMMs (fused bias / activation / gate / residual / scatter)
enum EpiMode {
  EPI_BIAS = 0,           // out[m, n] = acc + bias[n]                        (T out)
  EPI_BIAS_GELU = 1,      // out[m, n] = gelu_tanh(acc + bias[n])             (T out)
  EPI_BIAS_GATE_RES = 2,  // x[m, n] += gate[cond(m / L)][n] * (acc + bias)   (fp32 in place)
  EPI_PATCH_EMBED = 3,    // x[(m / n_img) L + m % n_img, n] = acc + bias + pos[m % n_img, n]
  EPI_BIAS_F32 = 4,       // out[m, n] = acc + bias[n]                        (fp32 out)
  EPI_UNPATCH = 5         // v[vrow(m / n_img)][latent index of (m % n_img, n)] = acc + bias
};

struct EpiArgs {
  const float* bias;
  void* out;
  int ldo;
  // gate / residual
  const float* mods;   // [n_cond, A]
  int A, gate_off;
  const int* condmap;  // [B]
  int L, n_img;
  const float* pos;    // [n_img, H]
  // unpatchify
  const int* vrows;    // [B] destination row of each sample in v
  long long D;
  int lt, lh, lw, pt, ph, pw, gh, gw;
  // EPI_BIAS: columns n < qcols (a multiple of 4) are multiplied by qscale after the bias.  The QKV
  // projection of the bf16 network writes q * log2(e) / sqrt(head dim) this way, rounded to bf16 once.
  int qcols;
  float qscale;
};

struct FwdBuffers {  // carved from the workspace
  int* rowmap;
  int* condmap;   // sample -> condition (its condition tokens)
  int* modmap;    // sample -> modulation group (its adaLN vectors)
  int* vrows;
  int* gcond;     // modulation group -> condition
  float* gt;      // modulation group -> time
  float *temb, *h1, *ct, *pooled, *pool_lin, *cvec, *mods, *cond_emb, *x, *sde_partials;
  void *patches, *xn, *qkv, *hid;
  float* v;       // compact velocity [max_frontier, D] (rollout only)
  int* plan;      // br_logprob launch plan
  size_t total;
};

size_t plan_workspace(const br_model* m, int n_cond, int max_batch, long long v_rows, long long partial_floats,
                      long long plan_ints, FwdBuffers* fb, void* base);

// One network evaluation of `B` samples (B <= max_batch of the plan).  z_base: latent rows,
// picked by fb.rowmap; v_out rows given by fb.vrows.  The adaLN vectors are computed once per
// modulation group g = (condition gcond[g], time gt[g]), g < n_groups <= max(n_cond, max_batch);
// sample b uses group fb.modmap[b].  gcond / gt are device arrays.
br_status forward(const br_model* m, const FwdBuffers& fb, const float* z_base, int B, const int* gcond,
                  const float* gt, int n_groups, float* v_out, hipStream_t st);
// The same with one time for the whole batch: one group per condition, modmap = condmap.
br_status forward_uniform_t(const br_model* m, const FwdBuffers& fb, const float* z_base, int B, float t, int n_cond,
                            float* v_out, hipStream_t st);
// Fill rowmap/condmap/modmap/vrows for a batch [b0, b0+B) of a frontier.
br_status fill_sample_maps(const FwdBuffers& fb, const SampleMap& smap, int b0, int B, int v_mode_rows, hipStream_t st);
// Condition-token embedding, once per call.
br_status embed_cond(const br_model* m, const FwdBuffers& fb, const void* cond_tokens, int n_cond, hipStream_t st);

// ---- op launchers (dit_kernels.hip, gemm_bf16.hip, attn_bf16.hip)
br_status launch_gemm(int dtype, int mode, const void* A, int lda, const void* W, int ldw, int M, int N, int K,
                      const EpiArgs& ea, hipStream_t st);
// q_prescaled: the q third already carries the factor log2(e) / sqrt(DH) (bf16 only)
br_status launch_attention(int dtype, const void* qkv, void* out, int B, int L, int NH, int DH, int q_prescaled,
                           hipStream_t st);
br_status launch_gemm_bf16(int mode, const bf16* A, int lda, const bf16* W, int ldw, int M, int N, int K,
                           const EpiArgs& ea, int variant, hipStream_t st);
bool gemm_stream_supported(int M, int N, int K, size_t bytes_a, size_t bytes_w);
br_status launch_gemm_bf16_stream(int mode, const bf16* A, int lda, const bf16* W, int ldw, int M, int N, int K,
                                  const EpiArgs& ea, int group_n, int row_block, int stagger_slack, int stagger_crit,
                                  hipStream_t st);
br_status launch_attention_bf16(const bf16* qkv, bf16* out, int B, int L, int NH, int DH, int q_prescaled, hipStream_t st);
br_status launch_ln_modulate(int dtype, const float* x, void* out, int n_rows, int rows_per_sample, int L_in, int H,
                             const float* mods, int A, int shift_off, int scale_off, const int* condmap,
                             hipStream_t st);

// ---- epilogue device code, shared by the fp32 and the MFMA GEMM
__device__ inline float gelu_tanh_f(float x) {
  // 0.5 x (1 + tanh(u)) = x / (1 + exp(-2u)), u = sqrt(2/pi) (x + 0.044715 x^3);
  // exp(-2u) = exp2(x (k1 + k3 x^2)), k1 = -2 sqrt(2/pi) log2(e), k3 = 0.044715 k1
  const float t = x * fmaf(x * x, -0.10294324f, -2.3022082f);
  return x * __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(t));
}

template <typename T>
__device__ inline void store4(T* p, float a, float b, float c, float d);
template <>
__device__ inline void store4<float>(float* p, float a, float b, float c, float d) {
  *reinterpret_cast<float4*>(p) = make_float4(a, b, c, d);
}
template <>
__device__ inline void store4<bf16>(bf16* p, float a, float b, float c, float d) {
  typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
  bf16x4 v = {(bf16)a, (bf16)b, (bf16)c, (bf16)d};
  *reinterpret_cast<bf16x4*>(p) = v;
}

template <int MODE, typename T>
struct Epilogue {
  EpiArgs a;
  struct Row {
    long long o;       // element offset of the output row
    const float* aux;  // gate row / pos row
    int tok;
  };
  __device__ inline Row row(int m) const {
    Row r;
    r.aux = nullptr;
    r.tok = 0;
    if (MODE == EPI_BIAS_GATE_RES) {
      r.o = (long long)m * a.ldo;
      r.aux = a.mods + (size_t)a.condmap[m / a.L] * a.A + a.gate_off;
    } else if (MODE == EPI_PATCH_EMBED) {
      const int b = m / a.n_img, tok = m - b * a.n_img;
      r.o = ((long long)b * a.L + tok) * a.ldo;
      r.aux = a.pos + (size_t)tok * a.ldo;
    } else if (MODE == EPI_UNPATCH) {
      const int b = m / a.n_img;
      r.tok = m - b * a.n_img;
      r.o = (long long)a.vrows[b] * a.D;
    } else {
      r.o = (long long)m * a.ldo;
    }
    return r;
  }
  // rows per sample when the row mapping depends on the sample, else 0
  __device__ inline int rows_per_sample() const {
    return MODE == EPI_BIAS_GATE_RES ? a.L : (MODE == EPI_PATCH_EMBED || MODE == EPI_UNPATCH) ? a.n_img : 0;
  }
  // ---- staged interface of the MFMA GEMM epilogue.  One hardware counter tracks a wave's
  // loads and stores in issue order, so a load issued after a store cannot be waited for
  // without also waiting for the store's write acknowledgement.  Whatever a tile's rows need
  // from memory is therefore fetched ahead of the stores: column constants and per-sample
  // constants once per tile, the per-row addend a few rows ahead.
  struct SampleC {
    float4 gate;  // gate[b, n..n+3] of the gated residual
    long long o;  // output offset of the sample (patch embedding, unpatchify)
  };
  static constexpr bool kHasAddend = MODE == EPI_BIAS_GATE_RES || MODE == EPI_PATCH_EMBED;
  __device__ inline float4 bias4(int n) const { return *reinterpret_cast<const float4*>(a.bias + n); }
  // EPI_BIAS: factor of the four columns n..n+3 (n % 4 == 0)
  __device__ inline float colscale(int n) const { return n < a.qcols ? a.qscale : 1.f; }
  __device__ inline SampleC sample_consts(int b, int n) const {
    SampleC s;
    s.gate = make_float4(0.f, 0.f, 0.f, 0.f);
    s.o = 0;
    if (MODE == EPI_BIAS_GATE_RES)
      s.gate = *reinterpret_cast<const float4*>(a.mods + (size_t)a.condmap[b] * a.A + a.gate_off + n);
    else if (MODE == EPI_PATCH_EMBED)
      s.o = (long long)b * a.L * a.ldo;
    else if (MODE == EPI_UNPATCH)
      s.o = (long long)a.vrows[b] * a.D;
    return s;
  }
  // what is added to row m (token tok of its sample) at columns n..n+3: the residual stream
  // or the position embedding
  __device__ inline float4 addend(int m, int tok, int n) const {
    if (MODE == EPI_BIAS_GATE_RES)
      return *reinterpret_cast<const float4*>(reinterpret_cast<const float*>(a.out) + (long long)m * a.ldo + n);
    if (MODE == EPI_PATCH_EMBED) return *reinterpret_cast<const float4*>(a.pos + (size_t)tok * a.ldo + n);
    return make_float4(0.f, 0.f, 0.f, 0.f);
  }
  // store() on operands already in registers
  __device__ inline void finish(int m, int tok, int n, float v0, float v1, float v2, float v3, const float4& bb,
                                const SampleC& sc, const float4& add) const {
    v0 += bb.x; v1 += bb.y; v2 += bb.z; v3 += bb.w;
    if (MODE == EPI_BIAS) {
      const float cs = colscale(n);
      store4<T>(reinterpret_cast<T*>(a.out) + (long long)m * a.ldo + n, v0 * cs, v1 * cs, v2 * cs, v3 * cs);
    } else if (MODE == EPI_BIAS_GELU) {
      store4<T>(reinterpret_cast<T*>(a.out) + (long long)m * a.ldo + n, gelu_tanh_f(v0), gelu_tanh_f(v1),
                gelu_tanh_f(v2), gelu_tanh_f(v3));
    } else if (MODE == EPI_BIAS_GATE_RES) {
      store4_stream(reinterpret_cast<float*>(a.out) + (long long)m * a.ldo + n, fmaf(sc.gate.x, v0, add.x),
                    fmaf(sc.gate.y, v1, add.y), fmaf(sc.gate.z, v2, add.z), fmaf(sc.gate.w, v3, add.w));
    } else if (MODE == EPI_PATCH_EMBED) {
      store4<float>(reinterpret_cast<float*>(a.out) + sc.o + (long long)tok * a.ldo + n, v0 + add.x, v1 + add.y,
                    v2 + add.z, v3 + add.w);
    } else if (MODE == EPI_BIAS_F32) {
      store4<float>(reinterpret_cast<float*>(a.out) + (long long)m * a.ldo + n, v0, v1, v2, v3);
    } else {
      Row r;
      r.o = sc.o;
      r.aux = nullptr;
      r.tok = tok;
      scatter_unpatch(r, n, v0, v1, v2, v3);
    }
  }
  // EPI_UNPATCH: token (tt, th, tw) raster, element (c, dt, dh, dw)
  __device__ inline void scatter_unpatch(const Row& r, int n, float v0, float v1, float v2, float v3) const {
    float* v = reinterpret_cast<float*>(a.out) + r.o;
    const int tw = r.tok % a.gw, th = (r.tok / a.gw) % a.gh, tt = r.tok / (a.gw * a.gh);
    const float vals[4] = {v0, v1, v2, v3};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int el = n + e;
      const int dw = el % a.pw, dh = (el / a.pw) % a.ph, dt = (el / (a.pw * a.ph)) % a.pt,
                c = el / (a.pw * a.ph * a.pt);
      const long long idx =
          (((long long)c * a.lt + tt * a.pt + dt) * a.lh + th * a.ph + dh) * a.lw + tw * a.pw + dw;
      v[idx] = vals[e];
    }
  }
  // four consecutive output columns n..n+3 (n % 4 == 0)
  __device__ inline void store(const Row& r, int n, float v0, float v1, float v2, float v3) const {
    const float4 bb = *reinterpret_cast<const float4*>(a.bias + n);
    v0 += bb.x; v1 += bb.y; v2 += bb.z; v3 += bb.w;
    if (MODE == EPI_BIAS) {
      const float cs = colscale(n);
      store4<T>(reinterpret_cast<T*>(a.out) + r.o + n, v0 * cs, v1 * cs, v2 * cs, v3 * cs);
    } else if (MODE == EPI_BIAS_GELU) {
      store4<T>(reinterpret_cast<T*>(a.out) + r.o + n, gelu_tanh_f(v0), gelu_tanh_f(v1), gelu_tanh_f(v2),
                gelu_tanh_f(v3));
    } else if (MODE == EPI_BIAS_GATE_RES) {
      float* x = reinterpret_cast<float*>(a.out) + r.o + n;
      const float4 g = *reinterpret_cast<const float4*>(r.aux + n);
      float4 xv = *reinterpret_cast<float4*>(x);
      xv.x = fmaf(g.x, v0, xv.x); xv.y = fmaf(g.y, v1, xv.y); xv.z = fmaf(g.z, v2, xv.z); xv.w = fmaf(g.w, v3, xv.w);
      *reinterpret_cast<float4*>(x) = xv;
    } else if (MODE == EPI_PATCH_EMBED) {
      const float4 p = *reinterpret_cast<const float4*>(r.aux + n);
      store4<float>(reinterpret_cast<float*>(a.out) + r.o + n, v0 + p.x, v1 + p.y, v2 + p.z, v3 + p.w);
    } else if (MODE == EPI_BIAS_F32) {
      store4<float>(reinterpret_cast<float*>(a.out) + r.o + n, v0, v1, v2, v3);
    } else {
      scatter_unpatch(r, n, v0, v1, v2, v3);
    }
  }
};

}  // namespace br
