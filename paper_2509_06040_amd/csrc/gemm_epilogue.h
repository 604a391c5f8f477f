// Epilogue of the MFMA GEMM kernels, shared by all tile shapes whose waves own 64 output
// columns.  The 32x32 accumulator layout gives a lane 4 consecutive columns of ONE row, so a
// direct store would touch 32 rows per instruction.  Each wave instead passes its accumulators
// through a private 4 KB LDS buffer (XOR-swizzled, conflict-free for the column-wise writes and
// the row-wise reads) and stores whole row segments of its 64 columns:
//   - bf16 outputs of a full tile: bias / GELU in the accumulator layout, rounded, 32 rows per pass;
//   - everything else: fp32 through LDS, 16 rows per pass, then bias / gate / addend per row.
//
// A wave's loads and stores retire through one in-order counter, so a load issued behind a
// store waits for that store's write acknowledgement.  The pass loops therefore contain no
// load that depends on a recent store: bias and per-sample constants (gate vector, output
// offset) are fetched once before the first store, and the per-row addend (residual stream,
// position embedding) is fetched ADDEND_AHEAD passes ahead of its use.
#pragma once
#include <type_traits>

#include "dit.h"

namespace br {

typedef float f32x16_e __attribute__((ext_vector_type(16)));
typedef float f32x4_e __attribute__((ext_vector_type(4)));

__device__ inline void epilogue_wave_fence() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Moves 16 rows (half `p` of accumulator block j) of the wave's accumulators into its LDS buffer.
template <int TM, int TN>
__device__ inline void epilogue_stage_rows(const f32x16_e (&acc)[TN][TM], char* ebuf, int j, int p, int lane) {
  const int l32 = lane & 31, lh = lane >> 5;
  // Lanes exchange data through the buffer without a workgroup barrier: the hardware keeps one
  // wave's LDS operations in order, and the wavefront-scope fences tell the compiler that the
  // reads on either side see other lanes' writes (it must neither reuse an earlier read of the
  // same address nor move accesses across).
  epilogue_wave_fence();
  if ((l32 >> 4) == p) {
    const int r = l32 & 15;
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int cc = i * 8 + g * 2 + lh;
        f32x4_e v = {acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]};
        *reinterpret_cast<f32x4_e*>(ebuf + r * 256 + ((cc ^ r) << 4)) = v;
      }
  }
  epilogue_wave_fence();
}

// Rows of a wave tile that spans more than two samples (models with fewer than 32 * TM rows
// per sample): every row looks its sample up by itself.
template <int TM, int TN, int MODE, typename TOUT>
__device__ inline void wave_epilogue_rows(const f32x16_e (&acc)[TN][TM], char* ebuf, int m_base, int n_base, int M, int N,
                                          const Epilogue<MODE, TOUT>& epi, int lane) {
  const int c4 = lane & 15, rq = lane >> 4;
  const int n = n_base + c4 * 4;
  const bool n_ok = n < N;
#pragma unroll
  for (int pass = 0; pass < TM * 2; ++pass) {
    epilogue_stage_rows<TM, TN>(acc, ebuf, pass >> 1, pass & 1, lane);
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int r = rq + 4 * q;
      const f32x4_e v = *reinterpret_cast<const f32x4_e*>(ebuf + r * 256 + ((c4 ^ r) << 4));
      const int m = m_base + pass * 16 + r;
      if (m < M && n_ok) epi.store(epi.row(m), n, v[0], v[1], v[2], v[3]);
    }
  }
}

// FULL: every row and column of the wave tile lies inside the matrix.  That path has no
// branches, which lets the compiler count outstanding memory operations exactly: its stores
// never wait, its addend loads wait for just the loads ahead of them.
template <bool FULL, int TM, int TN, int MODE, typename TOUT>
__device__ inline void wave_epilogue_pair(const f32x16_e (&acc)[TN][TM], char* ebuf, int m_base, int n_base, int M, int N,
                                          const Epilogue<MODE, TOUT>& epi, int lane) {
  using Epi = Epilogue<MODE, TOUT>;
  constexpr int NP = TM * 2;        // passes of 16 rows
  constexpr int ADDEND_AHEAD = 2;   // passes between the fetch of an addend and its use
  constexpr int NBUF = ADDEND_AHEAD + 1;
  const int rps = epi.rows_per_sample();
  const int c4 = lane & 15, rq = lane >> 4;
  const int n = n_base + c4 * 4;
  const bool n_ok = FULL || n < N;
  // the wave's rows lie in sample b0 (first row lo0) and, from row lo1 on, in sample b0 + 1
  int lo0 = 0, lo1 = 0x7fffffff;
  typename Epi::SampleC s0 = {}, s1 = {};
  float4 bb = make_float4(0.f, 0.f, 0.f, 0.f);
  if (n_ok) {
    bb = epi.bias4(n);
    if (rps > 0 && (FULL || m_base < M)) {  // a wave wholly below the matrix has no sample to look up
      const int b0 = m_base / rps;
      lo0 = b0 * rps;
      lo1 = lo0 + rps;
      s0 = epi.sample_consts(b0, n);
      s1 = epi.sample_consts(lo1 < M ? b0 + 1 : b0, n);
    }
  }
  float4 add[NBUF][4];
  auto fetch_addend = [&](int pass, float4* dst) {
    if (!Epi::kHasAddend) return;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int m = m_base + pass * 16 + rq + 4 * q;
      const int tok = m - (m >= lo1 ? lo1 : lo0);
      if (FULL)
        dst[q] = epi.addend(m, tok, n);
      else
        dst[q] = (m < M && n_ok) ? epi.addend(m, tok, n) : make_float4(0.f, 0.f, 0.f, 0.f);
    }
  };
#pragma unroll
  for (int pass = 0; pass < ADDEND_AHEAD && pass < NP; ++pass) fetch_addend(pass, add[pass % NBUF]);
#pragma unroll
  for (int pass = 0; pass < NP; ++pass) {
    if (pass + ADDEND_AHEAD < NP) fetch_addend(pass + ADDEND_AHEAD, add[(pass + ADDEND_AHEAD) % NBUF]);
    epilogue_stage_rows<TM, TN>(acc, ebuf, pass >> 1, pass & 1, lane);
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int r = rq + 4 * q;
      const f32x4_e v = *reinterpret_cast<const f32x4_e*>(ebuf + r * 256 + ((c4 ^ r) << 4));
      const int m = m_base + pass * 16 + r;
      if (FULL || (m < M && n_ok)) {
        const bool second = m >= lo1;
        epi.finish(m, m - (second ? lo1 : lo0), n, v[0], v[1], v[2], v[3], bb, second ? s1 : s0, add[pass % NBUF][q]);
      }
    }
  }
}

// bf16 outputs (bias, bias + GELU) of a wave tile wholly inside the matrix: bias and activation
// are applied in the accumulator layout and the values are rounded to bf16 BEFORE the trip through
// LDS, which halves the LDS traffic and lets a pass cover 32 rows: per pass 8 x ds_write_b64 by
// every lane, 4 x ds_read_b128, 4 stores of 16 bytes per lane (8 rows x 128 bytes each).  A buffer
// row is 128 bytes = eight 16-byte chunks, chunk c of row r sits in slot c ^ ((r >> 1) & 7).
template <int TM, int TN, int MODE>
__device__ inline void wave_epilogue_bf16_full(const f32x16_e (&acc)[TN][TM], char* ebuf, int m_base, int n_base,
                                               const Epilogue<MODE, bf16>& epi, int lane) {
  static_assert(MODE == EPI_BIAS || MODE == EPI_BIAS_GELU, "plain bf16 outputs only");
  typedef __bf16 bf16x4_e __attribute__((ext_vector_type(4)));
  typedef unsigned int u32x4_e __attribute__((ext_vector_type(4)));
  const int l32 = lane & 31, lh = lane >> 5;
  float4 bias[TN][4];
#pragma unroll
  for (int i = 0; i < TN; ++i)
#pragma unroll
    for (int g = 0; g < 4; ++g) bias[i][g] = epi.bias4(n_base + i * 32 + g * 8 + lh * 4);
  const int wswz = (l32 >> 1) & 7;
  char* wrow = ebuf + l32 * 128 + lh * 8;
  const int rrow = lane >> 3, rc = lane & 7;  // this lane reads chunk rc of rows rrow + 8 q
  bf16* const obase = reinterpret_cast<bf16*>(epi.a.out) + (long long)(m_base + rrow) * epi.a.ldo + n_base + rc * 8;
#pragma unroll
  for (int j = 0; j < TM; ++j) {
    epilogue_wave_fence();
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        float v0 = acc[i][j][4 * g] + bias[i][g].x, v1 = acc[i][j][4 * g + 1] + bias[i][g].y,
              v2 = acc[i][j][4 * g + 2] + bias[i][g].z, v3 = acc[i][j][4 * g + 3] + bias[i][g].w;
        if (MODE == EPI_BIAS_GELU) {
          v0 = gelu_tanh_f(v0);
          v1 = gelu_tanh_f(v1);
          v2 = gelu_tanh_f(v2);
          v3 = gelu_tanh_f(v3);
        } else {
          const float cs = epi.colscale(n_base + i * 32 + g * 8 + lh * 4);
          v0 *= cs;
          v1 *= cs;
          v2 *= cs;
          v3 *= cs;
        }
        const bf16x4_e pk = {(bf16)v0, (bf16)v1, (bf16)v2, (bf16)v3};
        *reinterpret_cast<bf16x4_e*>(wrow + (((i * 4 + g) ^ wswz) << 4)) = pk;
      }
    epilogue_wave_fence();
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int r = rrow + 8 * q;
      const u32x4_e v = *reinterpret_cast<const u32x4_e*>(ebuf + r * 128 + ((rc ^ ((r >> 1) & 7)) << 4));
      __builtin_nontemporal_store(v, reinterpret_cast<u32x4_e*>(obase + (long long)(j * 32 + 8 * q) * epi.a.ldo));
    }
  }
}

// Returns a lower bound on the number of store instructions the wave has issued (every lane
// active): 4 per 16-row pass on the branch-free path, unknown (0) on the guarded ones.
template <int TM, int TN, int MODE, typename TOUT>
__device__ inline int wave_epilogue(const f32x16_e (&acc)[TN][TM], char* ebuf, int m_base, int n_base, int M, int N,
                                    const Epilogue<MODE, TOUT>& epi, int lane) {
  static_assert(TN == 2, "waves own 64 output columns");
  const int rps = epi.rows_per_sample();
  if (rps > 0 && rps < TM * 32) {
    wave_epilogue_rows<TM, TN, MODE, TOUT>(acc, ebuf, m_base, n_base, M, N, epi, lane);
  } else if (m_base + TM * 32 <= M && n_base + TN * 32 <= N) {
    if constexpr ((MODE == EPI_BIAS || MODE == EPI_BIAS_GELU) && std::is_same<TOUT, bf16>::value) {
      wave_epilogue_bf16_full<TM, TN, MODE>(acc, ebuf, m_base, n_base, epi, lane);
      return TM * 4;
    } else {
      wave_epilogue_pair<true, TM, TN, MODE, TOUT>(acc, ebuf, m_base, n_base, M, N, epi, lane);
      return TM * 2 * 4;
    }
  } else {
    wave_epilogue_pair<false, TM, TN, MODE, TOUT>(acc, ebuf, m_base, n_base, M, N, epi, lane);
  }
  return 0;
}

}  // namespace br
