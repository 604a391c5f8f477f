// bf16 GEMM on the gfx950 matrix cores: C[m, n] = sum_k A[m, k] W[n, k], fp32
// accumulate, fused epilogue.  Both operands are k-contiguous, so a lane's MFMA
// operand is one 16-byte LDS read.  The weights feed the MFMA row operand and the
// activations the column operand (v_mfma_f32_32x32x16_bf16).
//
// This file holds the one-tile-per-workgroup kernels (BM x BN tile, WGM x WGN
// wavefronts) used for small problems and for K that is not a multiple of 128, and
// the dispatch; the persistent kernel for large problems is in gemm_bf16_stream.hip.
#include <type_traits>

#include <cmath>

#include "common.h"
#include "dit.h"
#include "gemm_epilogue.h"
#include "prof.h"

namespace br {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
// native vector type: arrays of HIP's uint4 struct are not promoted to registers
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// ---------------------------------------------------------------------------
// Deep-pipelined variant: operand tiles go from global memory straight into LDS
// (global_load_lds_dwordx4, no register staging), BK = 32 per stage, four stages,
// three of them in flight while the fourth is multiplied.  One tile's worth of
// registers is freed and, more importantly, about three times as many bytes are in
// flight per compute unit, which is what hides the L2/HBM latency.
//
// An LDS-direct load writes 64 lanes x 16 bytes to consecutive LDS addresses, i.e.
// 16 tile rows of 64 bytes; the swizzle is therefore applied on the global side:
// the lane that fills slot s of row r fetches k-chunk s ^ ((r >> 2) & 3).  Sixteen
// consecutive rows at one k-chunk then cover all 64 LDS banks exactly once.
// Each stage is its own __shared__ array and the k-loop is unrolled by the number
// of stages, so the compiler can tell the buffers apart and does not serialise the
// LDS reads of one stage against the loads in flight for the others.
#define BR_GPTR(p) ((const void __attribute__((address_space(1)))*)(p))
#define BR_LPTR(p) ((void __attribute__((address_space(3)))*)(p))

template <int BYTES, int S>
__shared__ __attribute__((aligned(1024))) char g_stage[BYTES];

template <int BM, int BN, int WGM, int WGN, int MODE, typename TOUT>
__global__ __launch_bounds__(WGM* WGN * 64) void gemm_bf16_dma_kernel(const bf16* __restrict__ A, int lda,
                                                                      const bf16* __restrict__ W, int ldw, int M, int N,
                                                                      int K, int tiles_m, int tiles_n, int group_n,
                                                                      Epilogue<MODE, TOUT> epi) {
  constexpr int NW = WGM * WGN;
  constexpr int WTM = BM / WGM, WTN = BN / WGN;
  constexpr int TM = WTM / 32, TN = WTN / 32;
  constexpr int IA = BM / 16 / NW, IW = BN / 16 / NW;  // LDS-direct loads per wave and stage
  constexpr int LPT = IA + IW;
  constexpr int SA = BM * 64, STAGE = (BM + BN) * 64;   // bytes
  static_assert(BM % (16 * NW) == 0 && BN % (16 * NW) == 0, "tile / wave mismatch");

  const int nwg = tiles_m * tiles_n;
  int wg = blockIdx.x;
  {
    const int per = nwg / 8, rem = nwg % 8, x = wg % 8, i = wg / 8;
    wg = x * per + (x < rem ? x : rem) + i;
  }
  int tile_m, tile_n;
  {
    const int gsz = tiles_m * group_n;
    const int g = wg / gsz, idx = wg - g * gsz;
    const int gn = min(group_n, tiles_n - g * group_n);
    tile_m = idx / gn;
    tile_n = g * group_n + idx - tile_m * gn;
  }
  const int m0 = tile_m * BM, n0 = tile_n * BN;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm0 = (wv % WGM) * WTM, wn0 = (wv / WGM) * WTN;
  const int l32 = lane & 31, lh = lane >> 5;

  // global source of this lane for each of its loads (k advances by 32 per stage)
  const bf16* ga[IA];
  const bf16* gw[IW];
#pragma unroll
  for (int j = 0; j < IA; ++j) {
    const int row = (wv * IA + j) * 16 + (lane >> 2), c = (lane & 3) ^ ((row >> 2) & 3);
    ga[j] = A + (size_t)min(m0 + row, M - 1) * lda + c * 8;
  }
#pragma unroll
  for (int j = 0; j < IW; ++j) {
    const int row = (wv * IW + j) * 16 + (lane >> 2), c = (lane & 3) ^ ((row >> 2) & 3);
    gw[j] = W + (size_t)min(n0 + row, N - 1) * ldw + c * 8;
  }
  // byte offsets of this lane's operand fragments inside a stage, per k16 step
  int fa_off[2][TM], fw_off[2][TN];
#pragma unroll
  for (int ks = 0; ks < 2; ++ks) {
#pragma unroll
    for (int j = 0; j < TM; ++j) {
      const int row = wm0 + j * 32 + l32;
      fa_off[ks][j] = row * 64 + (((ks * 2 + lh) ^ ((row >> 2) & 3)) << 4);
    }
#pragma unroll
    for (int i = 0; i < TN; ++i) {
      const int row = wn0 + i * 32 + l32;
      fw_off[ks][i] = SA + row * 64 + (((ks * 2 + lh) ^ ((row >> 2) & 3)) << 4);
    }
  }

  f32x16 acc[TN][TM];
#pragma unroll
  for (int i = 0; i < TN; ++i)
#pragma unroll
    for (int j = 0; j < TM; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int nk = K / 32;
  // The LDS-direct loads are issued from inline assembly: the compiler then does not
  // see LDS being written and adds no waits of its own; completion is tracked here
  // by hand.  Every step issues exactly LPT loads (past the end of K the last k-tile
  // is fetched again into a stage nobody reads), so "at most 2*LPT loads outstanding"
  // always means that the stage about to be multiplied has landed.
  auto issue = [&](auto S, int kt) {
    char* stage_ptr = g_stage<STAGE, decltype(S)::value>;
    const unsigned base = (unsigned)(uintptr_t)BR_LPTR(stage_ptr);
    const int kk = min(kt, nk - 1);
#pragma unroll
    for (int j = 0; j < IA; ++j) {
      const bf16* src = ga[j] + (size_t)kk * 32;
      const unsigned dst = base + (wv * IA + j) * 1024;
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(dst), "v"(src) : "memory", "m0");
    }
#pragma unroll
    for (int j = 0; j < IW; ++j) {
      const bf16* src = gw[j] + (size_t)kk * 32;
      const unsigned dst = base + SA + (wv * IW + j) * 1024;
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(dst), "v"(src) : "memory", "m0");
    }
  };
  // Operand fragments are prefetched one k16 half-step ahead: while the MFMAs of
  // (kt, first half) run, the fragments of (kt, second half) are read; while those
  // are multiplied, the first-half fragments of stage kt+1 are read.  The barrier
  // sits between the two halves, where every wave still has MFMAs in flight.
  bf16x8 fa0[TM], fw0[TN], fa1[TM], fw1[TN];
  auto read_half = [&](const char* stage, int ks, bf16x8* a, bf16x8* w) {
#pragma unroll
    for (int j = 0; j < TM; ++j) a[j] = *reinterpret_cast<const bf16x8*>(stage + fa_off[ks][j]);
#pragma unroll
    for (int i = 0; i < TN; ++i) w[i] = *reinterpret_cast<const bf16x8*>(stage + fw_off[ks][i]);
  };
  auto mma_half = [&](const bf16x8* a, const bf16x8* w) {
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
      for (int j = 0; j < TM; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w[i], a[j], acc[i][j], 0, 0, 0);
  };
  auto step = [&](auto S, int kt) {
    constexpr int CUR = decltype(S)::value, NXT = (CUR + 1) & 3;
    const char* cur = g_stage<STAGE, CUR>;
    const char* nxt = g_stage<STAGE, NXT>;
    read_half(cur, 1, fa1, fw1);
    __builtin_amdgcn_sched_barrier(0);  // keep the LDS reads ahead of the MFMAs they overlap with
    mma_half(fa0, fw0);
    __builtin_amdgcn_sched_barrier(0);  // ... and the MFMAs ahead of the barrier
    // own loads of stage kt+1 landed (only the two younger stages may be outstanding)
    // and both halves of stage kt are in registers -> barrier -> true for every wave:
    // stage kt+1 may be read and stage kt may be refilled
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(2 * LPT) : "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    issue(std::integral_constant<int, CUR>{}, kt + 4);
    read_half(nxt, 0, fa0, fw0);
    __builtin_amdgcn_sched_barrier(0);
    mma_half(fa1, fw1);
    __builtin_amdgcn_sched_barrier(0);
  };
  using I0 = std::integral_constant<int, 0>;
  using I1 = std::integral_constant<int, 1>;
  using I2 = std::integral_constant<int, 2>;
  using I3 = std::integral_constant<int, 3>;

  issue(I0{}, 0);
  issue(I1{}, 1);
  issue(I2{}, 2);
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * LPT) : "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
  issue(I3{}, 3);
  read_half(g_stage<STAGE, 0>, 0, fa0, fw0);
  for (int kt = 0;; kt += 4) {
    step(I0{}, kt);
    if (kt + 1 >= nk) break;
    step(I1{}, kt + 1);
    if (kt + 2 >= nk) break;
    step(I2{}, kt + 2);
    if (kt + 3 >= nk) break;
    step(I3{}, kt + 3);
    if (kt + 4 >= nk) break;
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the refills past the end of K
  __syncthreads();                                  // every wave is done with the stages
  {
    static_assert(STAGE >= 4 * 4096 && WTN == 64, "epilogue staging needs 4 KB per wave");
    char* ebuf = (wv < 4 ? g_stage<STAGE, 0> : g_stage<STAGE, 1>)+(wv & 3) * 4096;
    wave_epilogue<TM, TN, MODE, TOUT>(acc, ebuf, m0 + wm0, n0 + wn0, M, N, epi, lane);
  }
}

template <int BM, int BN, int WGM, int WGN, int MODE, typename TOUT>
static br_status gemm_dma_launch(const bf16* A, int lda, const bf16* W, int ldw, int M, int N, int K, const EpiArgs& ea,
                                 int group_n, hipStream_t st) {
  Epilogue<MODE, TOUT> epi{ea};
  const int tiles_m = cdiv(M, BM), tiles_n = cdiv(N, BN);
  if (group_n <= 0 || group_n > tiles_n) group_n = tiles_n;
  hipLaunchKernelGGL((gemm_bf16_dma_kernel<BM, BN, WGM, WGN, MODE, TOUT>), dim3(tiles_m * tiles_n), dim3(WGM * WGN * 64),
                     0, st, A, lda, W, ldw, M, N, K, tiles_m, tiles_n, group_n, epi);
  BR_LAUNCH_CHECK();
  return BR_OK;
}

// variant bits 0..3: kernel, 4 / 5 / 6 = 256x256 / 128x128 / 256x128 tiles, one tile per workgroup, LDS-direct loads
// in a four-stage ring; 7 = persistent 256x256 kernel with a continuous operand stream (gemm_bf16_stream.hip);
// bits 4..11: column-group width of the tile walk (0 = all columns).  variant < 0 = choose by problem size.
template <int MODE, typename TOUT>
static br_status gemm_variant(const bf16* A, int lda, const bf16* W, int ldw, int M, int N, int K, const EpiArgs& ea,
                              int variant, hipStream_t st) {
  int tile, group_n = 0, row_block = 0, stagger_slack = 0, stagger_crit = 0;
  if (variant < 0) {
    // Measured on MI355X.  With r = (256x256 tiles) / (compute units):
    // up to half a round of tiles, 256x128 tiles put twice as many units to work; up to one
    // round the persistent 256x256 kernel is best; beyond that it stays best unless the last
    // round would be mostly empty (r = 1.08 costs two rounds), where 128x128 tiles win.
    const int cu = device_cu_count();
    const long long tiles_m = cdiv(M, 256), tiles_n = cdiv(N, 256);
    const long long t256 = tiles_m * tiles_n;
    const double r = (double)t256 / (double)cu;
    const bool stream_ok = gemm_stream_supported(M, N, K, (size_t)M * lda * 2, (size_t)N * ldw * 2);
    // One or two whole rounds and a last one that fills at most half the units: the rows are independent,
    // so the matrix is cut in two launches, as many rows as make whole rounds for the persistent kernel and
    // the rest -- at most half a round -- for the 256x128 tiles, which take half a tile time.  With
    // per-sample epilogue operands the cut falls between two samples.  Measured on 1101-token samples:
    // 3-16 % at 16 samples (1.1 to 4.3 rounds), 2-7 % at 24 and 32.  From three whole rounds on it does not
    // pay: the few units of a sparse last round run faster than a full round's (64 samples, N = 1024,
    // 4.3 rounds: 1-4 % slower when cut).
    if (stream_ok && r > 1.0 && r < 3.0 && (MODE == EPI_BIAS || MODE == EPI_BIAS_GELU || MODE == EPI_BIAS_GATE_RES)) {
      const long long whole = t256 / cu;
      long long head_rows = (whole * cu / tiles_n) * 256;
      const int rps = MODE == EPI_BIAS_GATE_RES ? ea.L : 256;
      head_rows = head_rows / rps * rps;
      const long long tail_rows = M - head_rows;
      if (head_rows > 0 && tail_rows > 0 && cdiv(tail_rows, 256) * tiles_n * 2 <= cu &&
          cdiv(head_rows, 256) * tiles_n <= whole * cu) {
        EpiArgs tail = ea;
        tail.out = (char*)ea.out + (size_t)head_rows * ea.ldo * sizeof(TOUT);
        if (MODE == EPI_BIAS_GATE_RES) tail.condmap = ea.condmap + head_rows / rps;
        const int head_variant = 7 | ((MODE == EPI_BIAS_GATE_RES && K <= 2048) ? (6 << 12) : 0);  // (the start stagger below)
        const br_status head = gemm_variant<MODE, TOUT>(A, lda, W, ldw, (int)head_rows, N, K, ea, head_variant, st);
        if (head != BR_OK) return head;
        return gemm_variant<MODE, TOUT>(A + (size_t)head_rows * lda, lda, W, ldw, (int)tail_rows, N, K, tail, 6, st);
      }
    }
    if (r <= 0.5)
      tile = 6;
    else if (r > 1.0 && std::ceil(r) / r > 1.4)
      tile = 5;
    else
      tile = stream_ok ? 7 : 4;
    // The fp32 gated residual reads and writes 512 KB per tile; with a short k-loop (K <= 2048) these
    // bursts of a die's 32 workgroups, all in step, are a third of the launch.  Workgroups with one tile
    // less than the longest list start up to 7 x 3 us late, in groups of four, which costs the launch
    // nothing and spreads the bursts: measured 6 % (64 samples) to 14 % (32 samples) on the image
    // network's projection GEMM (1101-token samples, N = K = 1024), nothing on deeper k-loops.
    if (MODE == EPI_BIAS_GATE_RES && K <= 2048) stagger_slack = 300;
  } else {
    tile = variant & 15;
    group_n = (variant >> 4) & 255;
    stagger_slack = ((variant >> 12) & 255) * 50;  // half microseconds -> 10 ns ticks
    stagger_crit = ((variant >> 20) & 15) * 50;
    row_block = ((variant >> 24) & 127) * 8;
  }
  ProfScope ps(st, PROF_GEMM + MODE * 8 + tile, 2.0 * M * N * K);
  switch (tile) {
    case 4: return gemm_dma_launch<256, 256, 2, 4, MODE, TOUT>(A, lda, W, ldw, M, N, K, ea, group_n, st);
    case 5: return gemm_dma_launch<128, 128, 2, 2, MODE, TOUT>(A, lda, W, ldw, M, N, K, ea, group_n, st);
    case 6: return gemm_dma_launch<256, 128, 4, 2, MODE, TOUT>(A, lda, W, ldw, M, N, K, ea, group_n, st);
    case 7: return launch_gemm_bf16_stream(MODE, A, lda, W, ldw, M, N, K, ea, group_n, row_block, stagger_slack, stagger_crit, st);
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
