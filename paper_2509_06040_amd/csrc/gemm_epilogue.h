// Epilogue of the MFMA GEMM kernels, shared by all tile shapes whose waves own 64 output
// columns.  The 32x32 accumulator layout gives a lane 4 consecutive columns of ONE row, so a
// direct store would touch 32 rows per instruction.  Each wave instead passes its accumulators
// through a private 4 KB LDS buffer, 16 rows at a time (16-byte columns XOR-swizzled by the row:
// conflict-free for the column-wise writes and the row-wise reads), and then handles rows of 64
// consecutive columns with 16 lanes x 16 bytes each.  For the gated-residual epilogue the
// residual values of the next 16 rows are fetched while the current ones are processed.
#pragma once
#include "dit.h"

namespace br {

typedef float f32x16_e __attribute__((ext_vector_type(16)));
typedef float f32x4_e __attribute__((ext_vector_type(4)));

template <int TM, int TN, int MODE, typename TOUT>
__device__ inline void wave_epilogue(const f32x16_e (&acc)[TN][TM], char* ebuf, int m_base, int n_base, int M, int N,
                                     const Epilogue<MODE, TOUT>& epi, int lane) {
  static_assert(TN == 2, "waves own 64 output columns");
  const int l32 = lane & 31, lh = lane >> 5;
  const int c4 = lane & 15, rq = lane >> 4;
  const int n = n_base + c4 * 4;
  const bool n_ok = n < N;
  // sample index of the wave's first row, found once; rows are mapped from it without dividing
  const int rps = epi.rows_per_sample();
  int b0 = 0, lo0 = 0;
  if (rps > 0) {
    b0 = m_base / rps;
    lo0 = b0 * rps;
  }
  auto row_of = [&](int m) {
    int b = b0, lo = lo0;
    while (m - lo >= rps && rps > 0) {
      lo += rps;
      ++b;
    }
    return epi.row_in_sample(m, b, m - lo);
  };
  constexpr int NP = TM * 2;  // passes of 16 rows
  float4 pre[4], pre_next[4];
  auto fetch_pre = [&](int pass, float4* dst) {
    if (MODE != EPI_BIAS_GATE_RES) return;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int m = m_base + pass * 16 + rq + 4 * q;
      dst[q] = (m < M && n_ok) ? epi.residual(m, n) : make_float4(0.f, 0.f, 0.f, 0.f);
    }
  };
  fetch_pre(0, pre);
#pragma unroll
  for (int pass = 0; pass < NP; ++pass) {
    const int j = pass >> 1, p = pass & 1;
    if (pass + 1 < NP) fetch_pre(pass + 1, pre_next);
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
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int r = rq + 4 * q;
      const f32x4_e v = *reinterpret_cast<const f32x4_e*>(ebuf + r * 256 + ((c4 ^ r) << 4));
      const int m = m_base + pass * 16 + r;
      if (m < M && n_ok) {
        const auto row = row_of(m);
        epi.store_pre(row, n, v[0], v[1], v[2], v[3], pre[q]);
      }
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) pre[q] = pre_next[q];
  }
}

}  // namespace br
