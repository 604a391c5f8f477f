// bf16 flash attention on the gfx950 matrix cores: softmax(Q K^T / sqrt(d)) V over
// all L tokens of a sample, one workgroup per (128 queries, head, sample), four
// wavefronts of 32 queries each, key/value tiles of 64 staged through LDS.
//
// Scores are computed transposed, S^T = K Q^T: in the 32x32 MFMA accumulator a
// lane then holds 16 keys of ONE query (the other 16 sit in lane ^ 32), so the
// running max / sum / rescale of the online softmax are per-lane scalars and the
// exponentiated tile is already laid out as the column operand of O^T = V^T P^T.
// The contraction order of that product is permuted to match the accumulator
// layout; V is staged transposed ([d][key]) so the row operand is two 8-byte reads.
#include "common.h"
#include "dit.h"
#include "prof.h"

namespace br {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int KV_TILE = 64;
constexpr int VT_STRIDE = 68;  // bf16 elements per row of the transposed V tile (136 B)

template <int DH>
__global__ __launch_bounds__(256) void attn_bf16_kernel(const bf16* __restrict__ qkv, bf16* __restrict__ out, int L,
                                                        int H, int NH, int n_pairs, int grouped, float scale_log2) {
  constexpr int CH = DH / 8;    // 16-byte chunks per K row
  constexpr int KS = DH / 16;   // MFMA k-steps of the score product
  constexpr int DB = DH / 32;   // 32-row blocks of O^T
  constexpr int NKC = KV_TILE * CH / 256;  // K chunks per thread and tile
  constexpr int NVP = 32 * CH / 256;       // V key-pair items per thread and tile
  __shared__ __attribute__((aligned(16))) u32x4 sK[2][KV_TILE * CH];
  __shared__ __attribute__((aligned(16))) bf16 sVt[2][DH * VT_STRIDE];

  // Workgroups are dispatched round-robin over the 8 XCDs.  All query tiles of one
  // (sample, head) read the same keys and values, so they are given to one XCD and run
  // back to back there: K/V then come out of that XCD's L2 instead of being fetched 8 times.
  const int nq = (L + 127) / 128;
  // (With few pairs that would leave XCDs idle: then tiles are simply dealt out in order.)
  int pair, qt;
  if (grouped) {
    const int x = blockIdx.x & 7, slot = blockIdx.x >> 3;
    pair = (slot / nq) * 8 + x;
    qt = slot - (slot / nq) * nq;
  } else {
    pair = blockIdx.x / nq;
    qt = blockIdx.x - pair * nq;
  }
  if (pair >= n_pairs) return;
  const int b = pair / NH, h = pair - b * NH;
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, l32 = lane & 31, lh = lane >> 5;
  const size_t ld = (size_t)3 * H;
  const bf16* base = qkv + (size_t)b * L * ld + (size_t)h * DH;
  const int qi = qt * 128 + wv * 32 + l32;
  const int qc = min(qi, L - 1);

  bf16x8 qf[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks)
    qf[ks] = *reinterpret_cast<const bf16x8*>(base + (size_t)qc * ld + ks * 16 + lh * 8);

  f32x16 o[DB];
#pragma unroll
  for (int d = 0; d < DB; ++d)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[d][r] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  const bf16x2 one2 = {(bf16)1.0f, (bf16)1.0f};

  // The next key/value tile is fetched into registers while the current one is multiplied
  // out of LDS; two LDS buffers, one barrier per tile.
  u32x4 rk[NKC];
  bf16x8 rva[NVP], rvb[NVP];
  // byte offsets of this thread's items from the first key of a tile; a tile's base address is
  // uniform, so a fetch is a scalar base plus these 32-bit offsets
  const unsigned ldb = (unsigned)(ld * 2);
  unsigned koff[NKC], voff[NVP];
#pragma unroll
  for (int i = 0; i < NKC; ++i) {
    const int id = tid + i * 256, row = id / CH, c = id % CH;
    koff[i] = row * ldb + (H + c * 8) * 2;
  }
#pragma unroll
  for (int i = 0; i < NVP; ++i) {
    const int id = tid + i * 256, p = id & 31, c = id >> 5;
    voff[i] = 2 * p * ldb + (2 * H + c * 8) * 2;
  }
  auto fetch = [&](int k0) {
    const char* tile = reinterpret_cast<const char*>(base) + (size_t)k0 * ldb;
    if (k0 + KV_TILE <= L) {
#pragma unroll
      for (int i = 0; i < NKC; ++i) rk[i] = *reinterpret_cast<const u32x4*>(tile + koff[i]);
#pragma unroll
      for (int i = 0; i < NVP; ++i) {
        rva[i] = *reinterpret_cast<const bf16x8*>(tile + voff[i]);
        rvb[i] = *reinterpret_cast<const bf16x8*>(tile + voff[i] + ldb);
      }
    } else {  // ragged last tile: keys past the end read the last key (their scores are masked)
      const int last = L - 1 - k0;
#pragma unroll
      for (int i = 0; i < NKC; ++i) {
        const int id = tid + i * 256, row = id / CH, c = id % CH;
        rk[i] = *reinterpret_cast<const u32x4*>(tile + min(row, last) * ldb + (H + c * 8) * 2);
      }
#pragma unroll
      for (int i = 0; i < NVP; ++i) {
        const int id = tid + i * 256, p = id & 31, c = id >> 5;
        rva[i] = *reinterpret_cast<const bf16x8*>(tile + min(2 * p, last) * ldb + (2 * H + c * 8) * 2);
        rvb[i] = *reinterpret_cast<const bf16x8*>(tile + min(2 * p + 1, last) * ldb + (2 * H + c * 8) * 2);
      }
    }
  };
  auto stash = [&](int buf) {
    // K tile: row-major, chunk c of row r in slot c ^ (r & 7)
#pragma unroll
    for (int i = 0; i < NKC; ++i) {
      const int id = tid + i * 256, row = id / CH, c = id % CH;
      sK[buf][row * CH + (c ^ (row & 7))] = rk[i];
    }
    // V tile transposed: a thread holds two neighbouring keys of one 8-wide d chunk and
    // writes eight (key pair) words
#pragma unroll
    for (int i = 0; i < NVP; ++i) {
      const int id = tid + i * 256, p = id & 31, c = id >> 5;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
        bf16x2 pr = {rva[i][e], rvb[i][e]};
        *reinterpret_cast<bf16x2*>(&sVt[buf][(c * 8 + e) * VT_STRIDE + 2 * p]) = pr;
      }
    }
  };

  const int nkv = (L + KV_TILE - 1) / KV_TILE;
  fetch(0);
  stash(0);
  __syncthreads();
  // Pin the query fragments in registers here.  Left alone, the compiler sinks their loads to
  // just before the loop, and its wait-count bookkeeping at the loop header then makes every
  // iteration wait for the key/value fetch it has just issued.
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) asm volatile("" : "+v"(qf[ks]));
  for (int it = 0; it < nkv; ++it) {
    const int k0 = it * KV_TILE, buf = it & 1;
    if (it + 1 < nkv) fetch(k0 + KV_TILE);

    // S^T tile: s[kb][r] = score of key k0 + 32 kb + 8 (r/4) + 4 lh + r%4 for query l32
    f32x16 s[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
      for (int r = 0; r < 16; ++r) s[kb][r] = 0.f;
      const int row = kb * 32 + l32;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const int c = ks * 2 + lh;
        const bf16x8 kf = *reinterpret_cast<const bf16x8*>(&sK[buf][row * CH + (c ^ (row & 7))]);
        s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], s[kb], 0, 0, 0);
      }
    }
    // keys past the end exist only in the last tile of a ragged sequence
    if (k0 + KV_TILE > L) {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = k0 + kb * 32 + 8 * (r >> 2) + 4 * lh + (r & 3);
          if (key >= L) s[kb][r] = -INFINITY;
        }
    }
    // running maximum in the raw score domain (the scale is positive); the scale is folded
    // into the exponent: p = exp2(s c - m c)
    float mx = -INFINITY;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[kb][r]);
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float m_new = fmaxf(m_run, mx);
    const float mc = m_new * scale_log2;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int r = 0; r < 16; ++r) s[kb][r] = __builtin_amdgcn_exp2f(fmaf(s[kb][r], scale_log2, -mc));
    // the accumulators are rescaled only when some query of this wave saw a new maximum
    if (__builtin_amdgcn_ballot_w64(m_new != m_run) != 0) {
      const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * scale_log2);
      l_run *= alpha;
#pragma unroll
      for (int d = 0; d < DB; ++d)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[d][r] *= alpha;
      m_run = m_new;
    }

    // O^T += V^T P^T; k-slot (lh, e) of step (kb, j) is key 32 kb + 16 j + 8 (e/4) + 4 lh + e%4
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        bf16x8 pf;
#pragma unroll
        for (int e = 0; e < 8; ++e) pf[e] = (bf16)s[kb][8 * j + e];
        // row sum of the rounded probabilities, two per instruction (what the product below sums)
#pragma unroll
        for (int e = 0; e < 8; e += 2) {
          const bf16x2 pr = {pf[e], pf[e + 1]};
          l_run = __builtin_amdgcn_fdot2_f32_bf16(pr, one2, l_run, false);
        }
        const int kofs = kb * 32 + j * 16 + lh * 4;
#pragma unroll
        for (int d = 0; d < DB; ++d) {
          const bf16* vr = &sVt[buf][(d * 32 + l32) * VT_STRIDE + kofs];
          const bf16x4 v0 = *reinterpret_cast<const bf16x4*>(vr);
          const bf16x4 v1 = *reinterpret_cast<const bf16x4*>(vr + 8);
          const bf16x8 vf = {v0[0], v0[1], v0[2], v0[3], v1[0], v1[1], v1[2], v1[3]};
          o[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf, o[d], 0, 0, 0);
        }
      }
    // the other buffer was last read one tile ago, before the previous barrier
    if (it + 1 < nkv) stash(buf ^ 1);
    __syncthreads();
  }

  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  const float inv = 1.f / l_tot;
  if (qi < L) {
    bf16* orow = out + ((size_t)b * L + qi) * H + (size_t)h * DH;
#pragma unroll
    for (int d = 0; d < DB; ++d)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        bf16x4 v = {(bf16)(o[d][4 * g] * inv), (bf16)(o[d][4 * g + 1] * inv), (bf16)(o[d][4 * g + 2] * inv),
                    (bf16)(o[d][4 * g + 3] * inv)};
        *reinterpret_cast<bf16x4*>(orow + d * 32 + g * 8 + lh * 4) = v;
      }
  }
}

br_status launch_attention_bf16(const bf16* qkv, bf16* out, int B, int L, int NH, int DH, hipStream_t st) {
  BR_REQUIRE(L >= 1, BR_EINVAL, "attention: empty sequence");
  const long long n_pairs = (long long)B * NH;
  const int grouped = n_pairs >= 32 ? 1 : 0;
  const long long n_blocks = (grouped ? (n_pairs + 7) / 8 * 8 : n_pairs) * cdiv(L, 128);
  BR_REQUIRE(n_blocks <= 0x7FFFFFFFLL, BR_ESHAPE, "attention: too many workgroups for one launch");
  dim3 g((unsigned)n_blocks), blk(256);
  const float scale_log2 = (float)(1.4426950408889634 / sqrt((double)DH));
  const int H = NH * DH;
  ProfScope ps(st, PROF_ATTN + DH, 4.0 * B * (double)L * L * H);
  if (DH == 64) hipLaunchKernelGGL((attn_bf16_kernel<64>), g, blk, 0, st, qkv, out, L, H, NH, (int)n_pairs, grouped, scale_log2);
  else if (DH == 128) hipLaunchKernelGGL((attn_bf16_kernel<128>), g, blk, 0, st, qkv, out, L, H, NH, (int)n_pairs, grouped, scale_log2);
  else return fail(BR_ESHAPE, "bf16 attention: head dim must be 64 or 128");
  BR_LAUNCH_CHECK();
  return BR_OK;
}

}  // namespace br
