// Persistent bf16 GEMM for gfx950: C[m, n] = sum_k A[m, k] W[n, k], fp32 accumulate,
// fused epilogue.  One workgroup per compute unit walks a list of 256x256 output
// tiles; the operand stream (global memory -> LDS directly) never stops at a tile
// boundary: while the last k-steps of a tile are multiplied the first stage of the
// next tile is already being fetched, and it keeps landing while the finished tile
// goes through its epilogue.
//
// Stages are 64 deep (128-byte row segments: measured 1.6x the L2->LDS throughput of
// 64-byte segments on MI355X) and there are two of them; the refill of a stage is
// issued three quarters of the way through the other one, right after the only
// barrier of the stage.  Measured with the math in the loop, one 64 KB stage in
// flight beats three 32 KB stages in flight.
//
// Operand loads of a tile wholly inside the matrix take a scalar block address and one of two
// constant per-lane offsets, so the k-loop issues no vector arithmetic beside the MFMAs (the
// two do not overlap on this hardware).
//
// Epilogue (gemm_epilogue.h): the MFMA accumulator layout gives a lane 4 consecutive columns
// of ONE row, which would make every store instruction touch 32 different rows.  Each wave
// therefore passes its tile through a private 4 KB LDS buffer and writes whole row segments.
//
// Requirements: K % 128 == 0 (every tile starts on ring slot 0), K >= 128, operands below 4 GiB.
#include <type_traits>

#include "common.h"
#include "dit.h"
#include "gemm_epilogue.h"

namespace br {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

#define BR_LPTR(p) ((void __attribute__((address_space(3)))*)(p))

namespace {
constexpr int BM = 256, BN = 256, WGM = 2, WGN = 4, NW = 8;
constexpr int WTM = 128, WTN = 64, TM = 4, TN = 2;
constexpr int BK = 64;                                              // k-depth of a stage
constexpr int IA = BM / 8 / NW, IW = BN / 8 / NW, LPT = IA + IW;    // LDS-direct loads per wave and stage (8 rows each)
constexpr int SA = BM * 128, STAGE = (BM + BN) * 128;               // bytes
constexpr int EPILOGUE_STORES = TM * 2 * 4;                         // store instructions of a full wave tile
}  // namespace

template <int S>
__shared__ __attribute__((aligned(1024))) char g_ring[STAGE];
__shared__ __attribute__((aligned(1024))) char g_epi[NW * 4096];

__device__ inline const char* uniform_ptr(const char* p) {
  const unsigned long long v = reinterpret_cast<unsigned long long>(p);
  const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)v), hi = __builtin_amdgcn_readfirstlane((unsigned)(v >> 32));
  return reinterpret_cast<const char*>(((unsigned long long)hi << 32) | lo);
}

// Maps the j-th tile of workgroup `wg` to (tile_m, tile_n); false when the list is exhausted.
// Consecutive workgroup ids are spread over the 8 XCDs, so XCD x = wg % 8 gets a contiguous
// range of the tile order, shared by its workgroups in round-robin.  The order: blocks of
// row_block row panels outermost, inside a block column groups of group_n, inside a group rows
// outermost.  The 32 tiles an XCD works on at once then span 8 row panels x 4 column panels (the
// squarest footprint: fewest operand panels per round), and from one round to the next the XCD
// keeps its rows of A and moves on to the next columns of W: A, the operand that does not fit
// in the Infinity Cache at the large shapes, comes from HBM once per row block, while the
// weights, which do fit, are what is fetched again.  row_block >= tiles_m gives column groups
// over all rows.
__device__ inline bool stream_tile(int wg, int nwg, int j, int tiles_m, int tiles_n, int group_n, int row_block, int* tm,
                                   int* tn) {
  const int nt = tiles_m * tiles_n;
  const int x = wg & 7, i = wg >> 3, per_x = (nwg - x + 7) >> 3;  // workgroups on this XCD
  const int per = nt / 8, rem = nt % 8;
  const int start = x * per + (x < rem ? x : rem), cnt = per + (x < rem ? 1 : 0);
  const int local = i + j * per_x;
  if (local >= cnt) return false;
  int t = start + local;
  const int bsz = row_block * tiles_n;       // tiles of a full row block
  const int rb = t / bsz;
  t -= rb * bsz;
  const int rows = min(row_block, tiles_m - rb * row_block);
  const int gsz = rows * group_n;
  const int g = t / gsz, idx = t - g * gsz;
  const int gn = min(group_n, tiles_n - g * group_n);
  *tm = rb * row_block + idx / gn;
  *tn = g * group_n + idx - (idx / gn) * gn;
  return true;
}

template <int MODE, typename TOUT>
__global__ __launch_bounds__(512) void gemm_bf16_stream_kernel(const bf16* __restrict__ A, int lda,
                                                               const bf16* __restrict__ W, int ldw, int M, int N, int K,
                                                               int tiles_m, int tiles_n, int group_n, int row_block, int stagger_slack, int stagger_crit,
                                                               Epilogue<MODE, TOUT> epi) {
  const int tid = threadIdx.x, lane = tid & 63;
  // Workgroups that start together stay in step tile after tile, so the epilogues of the 32
  // workgroups of a compute die hit that die's memory port in one burst per round, with the port
  // idle in between.  Shifting groups of workgroups against each other spreads that traffic.
  // The four workgroups that share a row panel of A (consecutive ids on a die) keep one phase,
  // so they still fetch the panel together.  A workgroup whose tile list is one shorter than
  // the longest on its die starts up to 7 * stagger_slack ticks late (10 ns units) at no cost
  // to the launch; the others start up to 7 * stagger_crit ticks late.
  if (stagger_slack > 0 || stagger_crit > 0) {
    const int nt = tiles_m * tiles_n, x = blockIdx.x & 7, i = blockIdx.x >> 3, per_x = ((int)gridDim.x - x + 7) >> 3;
    const int cnt = nt / 8 + (x < nt % 8 ? 1 : 0);
    const int n_mine = i < cnt ? (cnt - i + per_x - 1) / per_x : 0, n_max = (cnt + per_x - 1) / per_x;
    const unsigned long long wait = (unsigned long long)((i >> 2) & 7) * (unsigned)(n_mine < n_max ? stagger_slack : stagger_crit);
    const unsigned long long t0 = wall_clock64();
    while (wall_clock64() - t0 < wait) __builtin_amdgcn_s_sleep(16);
  }
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm0 = (wv % WGM) * WTM, wn0 = (wv / WGM) * WTN;
  const int l32 = lane & 31, lh = lane >> 5;
  const int nst = K / BK;  // stages per tile (even)

  // A stage row is 128 bytes = eight 16-byte chunks; chunk c of row r sits in slot
  // c ^ ((r >> 1) & 7): sixteen consecutive rows at one chunk index then cover all 64 LDS
  // banks.  An LDS-direct load fills 8 consecutive rows (lane = 8 * row + slot), so the
  // swizzle is applied to the global address the lane fetches from.
  const int ld_row = lane >> 3;                                        // row inside an 8-row block
  // all rows this lane ever loads have (row >> 1) & 7 == (ld_row >> 1) & 3 + 4 * (block & 1)
  auto src_off = [&](int tile_row0, int blk, int limit, int ld) {
    const int row = blk * 8 + ld_row;
    const int c = (lane & 7) ^ ((row >> 1) & 7);
    return (unsigned)(((size_t)min(tile_row0 + row, limit - 1) * ld + c * 8) * 2);
  };
  // fragment byte offsets inside a stage for k16-step 0; step ks is the same offset ^ (ks << 5)
  int fa_off[TM], fw_off[TN];
#pragma unroll
  for (int j = 0; j < TM; ++j) {
    const int row = wm0 + j * 32 + l32;
    fa_off[j] = row * 128 + ((lh ^ ((row >> 1) & 7)) << 4);
  }
#pragma unroll
  for (int i = 0; i < TN; ++i) {
    const int row = wn0 + i * 32 + l32;
    fw_off[i] = SA + row * 128 + ((lh ^ ((row >> 1) & 7)) << 4);
  }

  int tile_j = 0, tm = 0, tn = 0, tmn = 0, tnn = 0;
  stream_tile(blockIdx.x, gridDim.x, 0, tiles_m, tiles_n, group_n, row_block, &tm, &tn);
  bool has_next = stream_tile(blockIdx.x, gridDim.x, 1, tiles_m, tiles_n, group_n, row_block, &tmn, &tnn);

  // Per-lane byte offsets of an LDS-direct load from the first row of its 8-row block, for
  // even and odd blocks (the swizzle of a row depends on the block only through its parity);
  // the block's base address is uniform and is carried in scalar registers, so a load of a
  // tile wholly inside the matrix costs no vector arithmetic at all.  Vector instructions
  // and MFMAs do not overlap on this hardware: every one saved here is matrix time gained.
  static_assert(IA % 2 == 0 && IW % 2 == 0, "block parity must follow the load index");
  unsigned voff_a[2], voff_w[2];
#pragma unroll
  for (int par = 0; par < 2; ++par) {
    const unsigned c = (lane & 7) ^ ((ld_row >> 1) | (4 * par));
    voff_a[par] = (unsigned)ld_row * (unsigned)lda * 2 + c * 16;
    voff_w[par] = (unsigned)ld_row * (unsigned)ldw * 2 + c * 16;
  }

  // Stream element q of the current tile: stage q if q < nst, stage q - nst of the next tile
  // otherwise (the last stage again when there is no next tile: a fetch nobody reads).
  auto issue = [&](auto S, int q) {
    char* ring = g_ring<decltype(S)::value>;
    const unsigned base = (unsigned)(uintptr_t)BR_LPTR(ring);
    const bool wrap = q >= nst && has_next;
    const unsigned kb = (unsigned)(wrap ? q - nst : min(q, nst - 1)) * (BK * 2);
    const int rm = (wrap ? tmn : tm) * BM, rn = (wrap ? tnn : tn) * BN;
    if (rm + BM <= M && rn + BN <= N) {
      // (the addresses are uniform; saying so keeps them in scalar registers in every instantiation)
      const char* a_blk = uniform_ptr(reinterpret_cast<const char*>(A) + ((size_t)(rm + wv * IA * 8) * lda) * 2 + kb);
      const char* w_blk = uniform_ptr(reinterpret_cast<const char*>(W) + ((size_t)(rn + wv * IW * 8) * ldw) * 2 + kb);
#pragma unroll
      for (int j = 0; j < IA; ++j) {
        const unsigned dst = base + (wv * IA + j) * 1024;
        const char* blk = a_blk + (size_t)j * 8 * lda * 2;
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(dst), "v"(voff_a[j & 1]), "s"(blk) : "memory", "m0");
      }
#pragma unroll
      for (int j = 0; j < IW; ++j) {
        const unsigned dst = base + SA + (wv * IW + j) * 1024;
        const char* blk = w_blk + (size_t)j * 8 * ldw * 2;
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(dst), "v"(voff_w[j & 1]), "s"(blk) : "memory", "m0");
      }
    } else {  // ragged tile: rows past the end read the last row
      const bf16* a_base = A;
      const bf16* w_base = W;
#pragma unroll
      for (int j = 0; j < IA; ++j) {
        const unsigned src = src_off(rm, wv * IA + j, M, lda) + kb;
        const unsigned dst = base + (wv * IA + j) * 1024;
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(dst), "v"(src), "s"(a_base) : "memory", "m0");
      }
#pragma unroll
      for (int j = 0; j < IW; ++j) {
        const unsigned src = src_off(rn, wv * IW + j, N, ldw) + kb;
        const unsigned dst = base + SA + (wv * IW + j) * 1024;
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(dst), "v"(src), "s"(w_base) : "memory", "m0");
      }
    }
  };

  f32x16 acc[TN][TM];
  auto zero_acc = [&]() {
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
      for (int j = 0; j < TM; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
  };
  zero_acc();

  // two fragment sets: set (ks & 1) holds k16-step ks
  bf16x8 fa[2][TM], fw[2][TN];
  auto read_frags = [&](const char* stage, int ks, int set) {
#pragma unroll
    for (int j = 0; j < TM; ++j) fa[set][j] = *reinterpret_cast<const bf16x8*>(stage + (fa_off[j] ^ (ks << 5)));
#pragma unroll
    for (int i = 0; i < TN; ++i) fw[set][i] = *reinterpret_cast<const bf16x8*>(stage + (fw_off[i] ^ (ks << 5)));
  };
  auto mma = [&](int set) {
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
      for (int j = 0; j < TM; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw[set][i], fa[set][j], acc[i][j], 0, 0, 0);
  };
  // One stage = four k16-steps; the fragments of step ks+1 are read while step ks is multiplied.
  // After the reads of the last step have been issued and have arrived, the other stage must
  // have landed too (nothing younger is in flight); one barrier then makes both true for every
  // wave, the freed stage is refilled, and the first fragments of the other stage are read.
  // `stores_behind`: the wave has issued at least that many stores since the fetch of the
  // other stage (the epilogue of a tile wholly inside the matrix).  Memory operations retire in
  // issue order, so the other stage has landed once no more than that many are outstanding,
  // and the stores' write acknowledgements need not be waited for yet.
  auto stage_step = [&](auto S, int q, int stores_behind) {
    constexpr int CUR = decltype(S)::value, NXT = CUR ^ 1;
    const char* cur = g_ring<CUR>;
#pragma unroll
    for (int ks = 0; ks < 3; ++ks) {
      read_frags(cur, ks + 1, (ks + 1) & 1);
      __builtin_amdgcn_sched_barrier(0);
      mma(ks & 1);
      __builtin_amdgcn_sched_barrier(0);
    }
    if (stores_behind >= EPILOGUE_STORES)
      asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(EPILOGUE_STORES) : "memory");
    else if (stores_behind >= EPILOGUE_STORES / 2)
      asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(EPILOGUE_STORES / 2) : "memory");
    else
      asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    issue(std::integral_constant<int, CUR>{}, q + 2);
    read_frags(g_ring<NXT>, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    mma(1);
    __builtin_amdgcn_sched_barrier(0);
  };
  using I0 = std::integral_constant<int, 0>;
  using I1 = std::integral_constant<int, 1>;

  issue(I0{}, 0);
  issue(I1{}, 1);
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(LPT) : "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
  read_frags(g_ring<0>, 0, 0);

  char* ebuf = g_epi + wv * 4096;
  int stores_behind = 0;
  for (;;) {
    stage_step(I0{}, 0, stores_behind);
    stage_step(I1{}, 1, 0);
    for (int q = 2; q < nst; q += 2) {
      stage_step(I0{}, q, 0);
      stage_step(I1{}, q + 1, 0);
    }
    // ---- epilogue of tile (tm, tn); the next tile's first stages keep landing meanwhile
    stores_behind = wave_epilogue<TM, TN, MODE, TOUT>(acc, ebuf, tm * BM + wm0, tn * BN + wn0, M, N, epi, lane);
    zero_acc();
    if (!has_next) break;
    // read the next tile's first fragments again rather than keep them alive across the
    // epilogue, which needs the registers for the rows it fetches ahead
    read_frags(g_ring<0>, 0, 0);
    tm = tmn;
    tn = tnn;
    ++tile_j;
    has_next = stream_tile(blockIdx.x, gridDim.x, tile_j + 1, tiles_m, tiles_n, group_n, row_block, &tmn, &tnn);
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the fetches past the end of the stream
}

template <int MODE, typename TOUT>
static br_status stream_launch(const bf16* A, int lda, const bf16* W, int ldw, int M, int N, int K, const EpiArgs& ea,
                               int group_n, int row_block, int stagger_slack, int stagger_crit, hipStream_t st) {
  Epilogue<MODE, TOUT> epi{ea};
  const int tiles_m = cdiv(M, BM), tiles_n = cdiv(N, BN);
  // Default walk: column groups of 4.  The 32 tiles an XCD works on at once then span 8 row
  // panels x 4 column panels, the squarest footprint, i.e. the fewest operand panels to pull
  // into its L2 per round (a third fewer fetched bytes than whole rows of 12 or 16 tiles).
  if (group_n <= 0 || group_n > tiles_n) group_n = tiles_n > 4 ? 4 : tiles_n;
  // An A operand larger than the 256 MB Infinity Cache would come from HBM once per column group
  // when the groups run over all rows (9 to 12 times for the QKV and FC1 shapes of the large
  // networks); in blocks of 8 row panels an XCD finishes all columns of its rows before it moves
  // on, and only the weights are fetched again.  Measured: 3-7 % shorter launches at those shapes,
  // no difference where A fits in the cache.
  if (row_block <= 0) row_block = ((size_t)M * K * 2 >= (256u << 20) && tiles_n > group_n) ? 8 : tiles_m;
  if (row_block > tiles_m) row_block = tiles_m;
  const int n_cu = device_cu_count();
  const int nt = tiles_m * tiles_n;
  const int grid = nt < n_cu ? nt : n_cu;
  hipLaunchKernelGGL((gemm_bf16_stream_kernel<MODE, TOUT>), dim3(grid), dim3(512), 0, st, A, lda, W, ldw, M, N, K,
                     tiles_m, tiles_n, group_n, row_block, stagger_slack, stagger_crit, epi);
  BR_LAUNCH_CHECK();
  return BR_OK;
}

bool gemm_stream_supported(int M, int N, int K, size_t bytes_a, size_t bytes_w) {
  // 32-bit byte offsets from the operand bases
  return K >= 128 && K % 128 == 0 && bytes_a < (1ull << 32) && bytes_w < (1ull << 32);
}

br_status launch_gemm_bf16_stream(int mode, const bf16* A, int lda, const bf16* W, int ldw, int M, int N, int K,
                                  const EpiArgs& ea, int group_n, int row_block, int stagger_slack, int stagger_crit,
                                  hipStream_t st) {
  BR_REQUIRE(stagger_slack >= 0 && stagger_slack <= 20000 && stagger_crit >= 0 && stagger_crit <= 20000, BR_EINVAL,
             "streaming gemm: stagger out of range");
  BR_REQUIRE(gemm_stream_supported(M, N, K, (size_t)M * lda * 2, (size_t)N * ldw * 2), BR_ESHAPE,
             "streaming gemm: needs K % 128 == 0 and operands below 4 GiB");
  switch (mode) {
    case EPI_BIAS: return stream_launch<EPI_BIAS, bf16>(A, lda, W, ldw, M, N, K, ea, group_n, row_block, stagger_slack, stagger_crit, st);
    case EPI_BIAS_GELU: return stream_launch<EPI_BIAS_GELU, bf16>(A, lda, W, ldw, M, N, K, ea, group_n, row_block, stagger_slack, stagger_crit, st);
    case EPI_BIAS_GATE_RES: return stream_launch<EPI_BIAS_GATE_RES, float>(A, lda, W, ldw, M, N, K, ea, group_n, row_block, stagger_slack, stagger_crit, st);
    case EPI_PATCH_EMBED: return stream_launch<EPI_PATCH_EMBED, float>(A, lda, W, ldw, M, N, K, ea, group_n, row_block, stagger_slack, stagger_crit, st);
    case EPI_BIAS_F32: return stream_launch<EPI_BIAS_F32, float>(A, lda, W, ldw, M, N, K, ea, group_n, row_block, stagger_slack, stagger_crit, st);
    case EPI_UNPATCH: return stream_launch<EPI_UNPATCH, float>(A, lda, W, ldw, M, N, K, ea, group_n, row_block, stagger_slack, stagger_crit, st);
  }
  return fail(BR_EINVAL, "gemm: unknown epilogue");
}

}  // namespace br
