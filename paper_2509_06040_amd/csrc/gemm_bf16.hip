// bf16 GEMM on the gfx950 matrix cores: C[m, n] = sum_k A[m, k] W[n, k], fp32
// accumulate, fused epilogue.  Both operands are k-contiguous, so a lane's MFMA
// operand is one 16-byte LDS read.  The weights feed the MFMA row operand and the
// activations the column operand: a lane then owns 4 consecutive output columns
// of one output row, which makes the epilogue's bias / gate / residual accesses
// and the stores 8- or 16-byte vectors.
//
// Tile BM x BN x 64 per workgroup, WGM x WGN wavefronts, v_mfma_f32_32x32x16_bf16.
// LDS rows are 128 bytes (eight 16-byte chunks); chunk c of row r sits in slot
// c ^ (r & 7), which keeps both the staging writes and the operand reads free of
// bank conflicts.  Global loads of tile k+1 are in flight while tile k is
// multiplied; two LDS buffers, one barrier per k-step.
#include "common.h"
#include "dit.h"
#include "prof.h"

namespace br {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

template <int BM, int BN, int WGM, int WGN, int MODE, typename TOUT>
__global__ __launch_bounds__(WGM* WGN * 64) void gemm_bf16_kernel(const bf16* __restrict__ A, int lda,
                                                                  const bf16* __restrict__ W, int ldw, int M, int N,
                                                                  int K, int tiles_m, int tiles_n,
                                                                  Epilogue<MODE, TOUT> epi) {
  constexpr int NT = WGM * WGN * 64;
  constexpr int WTM = BM / WGM, WTN = BN / WGN;
  constexpr int TM = WTM / 32, TN = WTN / 32;
  constexpr int CA = BM * 8 / NT, CW = BN * 8 / NT;  // 16-byte chunks per thread and tile
  static_assert(BM * 8 % NT == 0 && BN * 8 % NT == 0, "tile / thread mismatch");
  extern __shared__ __attribute__((aligned(16))) char smem[];
  uint4* sA = reinterpret_cast<uint4*>(smem);                 // [2][BM * 8] chunks
  uint4* sW = sA + 2 * BM * 8;                                // [2][BN * 8] chunks

  // Workgroup -> tile: consecutive workgroup ids go round-robin to the 8 XCDs, so
  // give each XCD a contiguous range of tiles (n fastest): tiles that share an
  // activation panel then share one L2.
  const int nwg = tiles_m * tiles_n;
  int wg = blockIdx.x;
  {
    const int per = nwg / 8, rem = nwg % 8, x = wg % 8, i = wg / 8;
    // XCD x owns per (+1 if x < rem) tiles starting at x*per + min(x, rem)
    wg = x * per + (x < rem ? x : rem) + i;
  }
  const int tile_m = wg / tiles_n, tile_n = wg % tiles_n;
  const int m0 = tile_m * BM, n0 = tile_n * BN;

  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int wm0 = (wv % WGM) * WTM, wn0 = (wv / WGM) * WTN;
  const int l32 = lane & 31, lh = lane >> 5;

  // staging: chunk id -> (row, k-chunk); rows beyond the matrix are clamped (their
  // products are never stored)
  const bf16* ga[CA];
  const bf16* gw[CW];
  int sa_off[CA], sw_off[CW];
#pragma unroll
  for (int i = 0; i < CA; ++i) {
    const int id = tid + i * NT, row = id >> 3, c = id & 7;
    const int gm = min(m0 + row, M - 1);
    ga[i] = A + (size_t)gm * lda + c * 8;
    sa_off[i] = row * 8 + (c ^ (row & 7));
  }
#pragma unroll
  for (int i = 0; i < CW; ++i) {
    const int id = tid + i * NT, row = id >> 3, c = id & 7;
    const int gn = min(n0 + row, N - 1);
    gw[i] = W + (size_t)gn * ldw + c * 8;
    sw_off[i] = row * 8 + (c ^ (row & 7));
  }

  f32x16 acc[TN][TM];
#pragma unroll
  for (int i = 0; i < TN; ++i)
#pragma unroll
    for (int j = 0; j < TM; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  uint4 ra[CA], rw[CW];
  const int nk = K / 64;
#pragma unroll
  for (int i = 0; i < CA; ++i) ra[i] = *reinterpret_cast<const uint4*>(ga[i]);
#pragma unroll
  for (int i = 0; i < CW; ++i) rw[i] = *reinterpret_cast<const uint4*>(gw[i]);
#pragma unroll
  for (int i = 0; i < CA; ++i) sA[sa_off[i]] = ra[i];
#pragma unroll
  for (int i = 0; i < CW; ++i) sW[sw_off[i]] = rw[i];
  __syncthreads();

  for (int kt = 0; kt < nk; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < nk) {
#pragma unroll
      for (int i = 0; i < CA; ++i) ra[i] = *reinterpret_cast<const uint4*>(ga[i] + (size_t)(kt + 1) * 64);
#pragma unroll
      for (int i = 0; i < CW; ++i) rw[i] = *reinterpret_cast<const uint4*>(gw[i] + (size_t)(kt + 1) * 64);
    }
    const uint4* cA = sA + cur * BM * 8;
    const uint4* cW = sW + cur * BN * 8;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      bf16x8 fa[TM], fw[TN];
      const int c = ks * 2 + lh;
#pragma unroll
      for (int j = 0; j < TM; ++j) {
        const int row = wm0 + j * 32 + l32;
        fa[j] = *reinterpret_cast<const bf16x8*>(&cA[row * 8 + (c ^ (row & 7))]);
      }
#pragma unroll
      for (int i = 0; i < TN; ++i) {
        const int row = wn0 + i * 32 + l32;
        fw[i] = *reinterpret_cast<const bf16x8*>(&cW[row * 8 + (c ^ (row & 7))]);
      }
#pragma unroll
      for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw[i], fa[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < nk) {
      uint4* nA = sA + (cur ^ 1) * BM * 8;
      uint4* nW = sW + (cur ^ 1) * BN * 8;
#pragma unroll
      for (int i = 0; i < CA; ++i) nA[sa_off[i]] = ra[i];
#pragma unroll
      for (int i = 0; i < CW; ++i) nW[sw_off[i]] = rw[i];
    }
    __syncthreads();
  }

  // accumulator layout of the 32x32 MFMA: lane owns output row (= MFMA column)
  // m = l32 and output columns n = 8 g + 4 lh + {0..3}, g = 0..3
#pragma unroll
  for (int j = 0; j < TM; ++j) {
    const int m = m0 + wm0 + j * 32 + l32;
    if (m < M) {
      const auto row = epi.row(m);
#pragma unroll
      for (int i = 0; i < TN; ++i) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int n = n0 + wn0 + i * 32 + g * 8 + lh * 4;
          if (n < N) epi.store(row, n, acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]);
        }
      }
    }
  }
}

template <int BM, int BN, int WGM, int WGN, int MODE, typename TOUT>
static br_status gemm_launch(const bf16* A, int lda, const bf16* W, int ldw, int M, int N, int K, const EpiArgs& ea,
                             hipStream_t st) {
  Epilogue<MODE, TOUT> epi{ea};
  const int tiles_m = cdiv(M, BM), tiles_n = cdiv(N, BN);
  const size_t lds = (size_t)2 * (BM + BN) * 128;
  auto kern = gemm_bf16_kernel<BM, BN, WGM, WGN, MODE, TOUT>;
  if (lds > 65536) {
    static bool attr_done = false;  // per instantiation
    if (!attr_done) {
      BR_HIP(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
      attr_done = true;
    }
  }
  hipLaunchKernelGGL(kern, dim3(tiles_m * tiles_n), dim3(WGM * WGN * 64), lds, st, A, lda, W, ldw, M, N, K, tiles_m,
                     tiles_n, epi);
  BR_LAUNCH_CHECK();
  return BR_OK;
}

// variant: 0 = 128x128 (4 waves), 1 = 256x128 (8 waves), 2 = 256x256 (8 waves), 3 = 128x256 (8 waves);
// -1 = choose by problem size.
template <int MODE, typename TOUT>
static br_status gemm_variant(const bf16* A, int lda, const bf16* W, int ldw, int M, int N, int K, const EpiArgs& ea,
                              int variant, hipStream_t st) {
  if (variant < 0) {
    const long long t256 = (long long)cdiv(M, 256) * cdiv(N, 256);
    const long long t2561 = (long long)cdiv(M, 256) * cdiv(N, 128);
    variant = t256 >= 512 ? 2 : (t2561 >= 512 ? 1 : 0);
  }
  ProfScope ps(st, PROF_GEMM + MODE * 8 + variant, 2.0 * M * N * K);
  switch (variant) {
    case 0: return gemm_launch<128, 128, 2, 2, MODE, TOUT>(A, lda, W, ldw, M, N, K, ea, st);
    case 1: return gemm_launch<256, 128, 4, 2, MODE, TOUT>(A, lda, W, ldw, M, N, K, ea, st);
    case 2: return gemm_launch<256, 256, 2, 4, MODE, TOUT>(A, lda, W, ldw, M, N, K, ea, st);
    case 3: return gemm_launch<128, 256, 2, 4, MODE, TOUT>(A, lda, W, ldw, M, N, K, ea, st);
  }
  return fail(BR_EINVAL, "gemm: unknown variant");
}

br_status launch_gemm_bf16(int mode, const bf16* A, int lda, const bf16* W, int ldw, int M, int N, int K,
                           const EpiArgs& ea, int variant, hipStream_t st) {
  BR_REQUIRE(K % 64 == 0 && K >= 64, BR_ESHAPE, "bf16 gemm: K must be a positive multiple of 64");
  BR_REQUIRE(lda % 8 == 0 && ldw % 8 == 0, BR_ESHAPE, "bf16 gemm: leading dimensions must be multiples of 8");
  switch (mode) {
    case EPI_BIAS: return gemm_variant<EPI_BIAS, bf16>(A, lda, W, ldw, M, N, K, ea, variant, st);
    case EPI_BIAS_GELU: return gemm_variant<EPI_BIAS_GELU, bf16>(A, lda, W, ldw, M, N, K, ea, variant, st);
    case EPI_BIAS_GATE_RES: return gemm_variant<EPI_BIAS_GATE_RES, float>(A, lda, W, ldw, M, N, K, ea, variant, st);
    case EPI_PATCH_EMBED: return gemm_variant<EPI_PATCH_EMBED, float>(A, lda, W, ldw, M, N, K, ea, variant, st);
    case EPI_BIAS_F32: return gemm_variant<EPI_BIAS_F32, float>(A, lda, W, ldw, M, N, K, ea, variant, st);
    case EPI_UNPATCH: return gemm_variant<EPI_UNPATCH, float>(A, lda, W, ldw, M, N, K, ea, variant, st);
  }
  return fail(BR_EINVAL, "gemm: unknown epilogue");
}

}  // namespace br
