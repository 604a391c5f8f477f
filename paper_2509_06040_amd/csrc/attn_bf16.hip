// bf16 flash attention on the gfx950 matrix cores: softmax(Q K^T / sqrt(d)) V over
// all L tokens of a sample, one workgroup per (128 queries, head, sample), four
// wavefronts of 32 queries each, key/value tiles of 64 keys in LDS.
//
// Scores are computed transposed, S^T = K Q^T: in the 32x32 MFMA accumulator a
// lane then holds 16 keys of ONE query (the other 16 sit in lane ^ 32), so the
// reference / sum / rescale of the online softmax are per-lane scalars and the
// exponentiated tile is already laid out as the column operand of O^T = V^T P^T.
// The contraction order of that product is permuted to match the accumulator layout.
//
// Both tiles travel from global memory straight into LDS (no registers, no vector
// instructions on the way), row-major as they lie in the QKV buffer, with their 16-byte
// chunks permuted per row so that fragment reads spread over the banks.  The row operand
// of the second product needs V transposed; the LDS transpose read delivers that: in a
// group of 16 lanes, lane 4 r + q supplies the address of 8 bytes (4 values of row r) and
// lane j receives element j of rows 0..3, so each lane ends up with four consecutive keys
// of its own channel.
#include <type_traits>
#include <utility>

#include "common.h"
#include "dit.h"
#include "prof.h"

namespace br {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

#define BR_LPTR(p) ((void __attribute__((address_space(3)))*)(p))

// f(integral_constant<int, 0>) ... f(integral_constant<int, N - 1>), in order
template <int... I, class F>
__device__ __forceinline__ void static_for_impl(std::integer_sequence<int, I...>, F&& f) { (f(std::integral_constant<int, I>{}), ...); }
template <int N, class F>
__device__ __forceinline__ void static_for(F&& f) { static_for_impl(std::make_integer_sequence<int, N>{}, f); }

constexpr int KV_TILE = 64;

// (a uniform address; saying so keeps it in scalar registers)
static __device__ inline const char* uniform_ptr(const char* p) {
  const unsigned long long v = reinterpret_cast<unsigned long long>(p);
  const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)v), hi = __builtin_amdgcn_readfirstlane((unsigned)(v >> 32));
  return reinterpret_cast<const char*>(((unsigned long long)hi << 32) | lo);
}

// Slot permutations of the K and V tiles: 16-byte chunk c of row r sits in slot c ^ swz(r).
// The LDS has 64 banks of 4 bytes; a 16-byte read is served 16 lanes at a time and an 8-byte
// read 32 lanes at a time, conflict-free when those lanes cover all 256 bytes of a bank row.
//   K (ds_read_b128, lanes 0..15 = 16 consecutive rows at one chunk index): with 256-byte rows
//   the rows must land in 16 different slots, with 128-byte rows (two per bank row) row pairs in 8.
//   V (transposing 8-byte reads, 32 lanes = 4 consecutive rows x 4 consecutive chunks): with
//   256-byte rows the four rows take the four groups of 4 slots, with 128-byte rows the rows
//   r and r + 2, which share a bank row, take different halves.
template <int DH>
__device__ inline int k_swz(int r) { return DH == 128 ? (r & 15) : ((r >> 1) & 7); }
template <int DH>
__device__ inline int v_swz(int r) { return DH == 128 ? ((r & 3) << 2) : (((r >> 1) & 1) << 2); }

// With at most 256 registers a wave (two waves per SIMD) the compiler keeps the MFMA results in
// ordinary vector registers, where the softmax works on them directly (accumulation registers
// would cost a copy per element).  Head dim 64 runs three waves per SIMD (168 registers: the
// tile loop then spills nothing; a fourth wave bought no time).
// PRE: the q third of the buffer already carries the factor log2(e) / sqrt(DH), as the network's
// QKV projection writes it; otherwise the exponent is scaled here, one multiplication per score.
template <int DH, bool PRE>
__global__ __launch_bounds__(256, DH == 64 ? 3 : 2) void attn_bf16_kernel(const bf16* __restrict__ qkv, bf16* __restrict__ out, int L,
                                                           int H, int NH, int n_pairs, int grouped, float scale_log2) {
  constexpr int CH = DH / 8;    // 16-byte chunks per K row
  constexpr int KS = DH / 16;   // MFMA k-steps of the score product
  constexpr int DB = DH / 32;   // 32-row blocks of O^T
  constexpr int RPI = 64 / CH;              // rows covered by one 1 KB load
  constexpr int LPW = KV_TILE / RPI / 4;    // loads per wave, tile and operand
  constexpr int NPAR = RPI == 8 ? 2 : 4;    // distinct slot patterns among a wave's loads (the swizzle period is 16 rows)
  constexpr int ROW_B = CH * 16;            // bytes per row
  constexpr int TILE_B = KV_TILE * ROW_B;
  // Operand fragments are read from LDS RA matrix instructions ahead of the one that consumes them
  // (0: each read directly before its use, left to the compiler's scheduling).  With two waves a
  // SIMD the LDS latency in front of every matrix instruction is otherwise exposed: 2-4 % of the
  // launch at head dim 128, no more beyond two steps; nothing at head dim 64 with its three waves.
  constexpr int RA = DH == 64 ? 0 : 2;
  __shared__ __attribute__((aligned(1024))) char sK[2][TILE_B];
  __shared__ __attribute__((aligned(1024))) char sV[2][TILE_B];

  // Workgroups are dispatched round-robin over the 8 XCDs.  All query tiles of one
  // (sample, head) read the same keys and values, so they are given to one XCD and run
  // back to back there: K/V then come out of that XCD's L2 instead of being fetched 8 times.
  // (With few pairs that would leave XCDs idle: then tiles are simply dealt out in order.)
  const int nq = (L + 127) / 128;
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
  const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, lh = lane >> 5;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const size_t ld = (size_t)3 * H;
  const bf16* base = qkv + (size_t)b * L * ld + (size_t)h * DH;
  const int qi = qt * 128 + wv * 32 + l32;
  const int qc = min(qi, L - 1);
  const bool active = qt * 128 + wv * 32 < L;  // (uniform over the wave)

  bf16x8 qf[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks)
    qf[ks] = *reinterpret_cast<const bf16x8*>(base + (size_t)qc * ld + ks * 16 + lh * 8);

  f32x16 o[DB];
#pragma unroll
  for (int d = 0; d < DB; ++d)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[d][r] = 0.f;
  float m_run = 0.f, l_run = 0.f;  // reference (a bf16 value) and row sum of the probabilities taken against it
  const bf16x2 one2 = {(bf16)1.0f, (bf16)1.0f};
  // the k-step that subtracts the reference: key side 1 in k-slot 0, query side -m_run there
  bf16x8 onef, mf;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    onef[e] = (bf16)((e == 0 && lh == 0) ? 1.f : 0.f);
    mf[e] = (bf16)0.f;
  }

  // Key and value tiles go from global memory straight into LDS, 1 KB (RPI rows) per
  // instruction: lane i fills bytes 16 i .. 16 i + 15 of the instruction's span, so the chunk
  // permutation is applied on the global side.
  const unsigned ldb = (unsigned)(ld * 2);
  const int lrow = lane / CH, slot = lane % CH;
  unsigned koff[NPAR], voff[NPAR];
#pragma unroll
  for (int par = 0; par < NPAR; ++par) {
    const int r16 = ((RPI * par) & 15) + lrow;  // row of the tile, modulo the swizzle period
    koff[par] = lrow * ldb + (H + (slot ^ k_swz<DH>(r16)) * 8) * 2;
    voff[par] = lrow * ldb + (2 * H + (slot ^ v_swz<DH>(r16)) * 8) * 2;
  }
  auto issue = [&](int k0, int buf) {
    const unsigned kdst = (unsigned)(uintptr_t)BR_LPTR(sK[buf]) + wv * LPW * 1024;
    const unsigned vdst = (unsigned)(uintptr_t)BR_LPTR(sV[buf]) + wv * LPW * 1024;
    if (k0 + KV_TILE <= L) {
      const char* blk = uniform_ptr(reinterpret_cast<const char*>(base) + (size_t)(k0 + wv * LPW * RPI) * ldb);
#pragma unroll
      for (int t = 0; t < LPW; ++t) {
        const char* src = blk + (size_t)t * RPI * ldb;
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(kdst + t * 1024), "v"(koff[t % NPAR]), "s"(src) : "memory", "m0");
      }
#pragma unroll
      for (int t = 0; t < LPW; ++t) {
        const char* src = blk + (size_t)t * RPI * ldb;
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(vdst + t * 1024), "v"(voff[t % NPAR]), "s"(src) : "memory", "m0");
      }
    } else {  // ragged last tile: rows past the end read the last key (their scores are masked)
      const char* blk = uniform_ptr(reinterpret_cast<const char*>(base));
#pragma unroll
      for (int t = 0; t < LPW; ++t) {
        const int row = (wv * LPW + t) * RPI + lrow;
        const unsigned off = (unsigned)min(k0 + row, L - 1) * ldb + (H + (slot ^ k_swz<DH>(row)) * 8) * 2;
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(kdst + t * 1024), "v"(off), "s"(blk) : "memory", "m0");
      }
#pragma unroll
      for (int t = 0; t < LPW; ++t) {
        const int row = (wv * LPW + t) * RPI + lrow;
        const unsigned off = (unsigned)min(k0 + row, L - 1) * ldb + (2 * H + (slot ^ v_swz<DH>(row)) * 8) * 2;
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(vdst + t * 1024), "v"(off), "s"(blk) : "memory", "m0");
      }
    }
  };

  // transposed reads of V: in a group of 16 lanes, lane 4 r + q supplies the 8 bytes at
  // (key K0 + r, d0 + 4 q .. 4 q + 3) and lane j receives (keys K0 .. K0 + 3, d0 + j)
  const int jj = lane & 15, g1 = (lane >> 4) & 1;
  const int vrow = 4 * lh + (jj >> 2);  // row within a group of 8 keys
  unsigned vaddr[DB];
#pragma unroll
  for (int d = 0; d < DB; ++d) {
    const int chunk = d * 4 + 2 * g1 + ((jj & 3) >> 1);
    vaddr[d] = vrow * ROW_B + (chunk ^ v_swz<DH>(vrow)) * 16 + 8 * (jj & 1);
  }

  // Two LDS buffers, one barrier per tile: the next tile is fetched while the current one is
  // multiplied.  Every iteration issues the same number of fetches (the last one fetches its
  // own tile again, into the idle buffer), so the wait below is exact.
  const int nkv = (L + KV_TILE - 1) / KV_TILE;
  issue(0, 0);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  // Pin the query fragments in registers here; left alone, the compiler sinks their loads
  // into the loop.
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) asm volatile("" : "+v"(qf[ks]));
  // One key tile.  NKB: 32-key blocks of the tile that hold any key at all (2, or 1 in a short
  // last tile); MASK: the tile runs past the end of the sequence.  Only the last tile of a
  // ragged sequence is compiled with masking, so the loop over full tiles carries none of it.
  // BUF: the LDS buffer of the tile (it & 1) as a constant, so that fragment addresses are a
  // loop-invariant per-lane register plus an immediate.
  auto tile = [&](int it, auto NKBc, auto MASKc, auto BUFc) {
    constexpr int NKB = decltype(NKBc)::value;
    constexpr bool MASK = decltype(MASKc)::value;
    constexpr int buf = decltype(BUFc)::value;
    const int k0 = it * KV_TILE;
    // the other buffer was last read one tile ago, before the previous barrier
    issue(min(it + 1, nkv - 1) * KV_TILE, buf ^ 1);

    // S^T tile minus the reference: s[kb][r] = score of key k0 + 32 kb + 8 (r/4) + 4 lh + r%4 for query
    // l32, less m_run of that query.  The subtraction rides on the matrix pipe: one more k-step whose
    // key side is the constant 1 and whose query side is -m_run (exact in bf16).
    f32x16 s[2];
    auto scores = [&]() __attribute__((always_inline)) {
      if constexpr (RA == 0) {
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb) {
#pragma unroll
          for (int r = 0; r < 16; ++r) s[kb][r] = 0.f;
          s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(onef, mf, s[kb], 0, 0, 0);
          const int row = kb * 32 + l32;
#pragma unroll
          for (int ks = 0; ks < KS; ++ks) {
            const int c = ks * 2 + lh;
            const bf16x8 kf = *reinterpret_cast<const bf16x8*>(&sK[buf][(row * CH + (c ^ k_swz<DH>(row))) * 16]);
            s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], s[kb], 0, 0, 0);
          }
        }
      } else {
        constexpr int N = NKB * KS;
        auto read_k = [&](int i) __attribute__((always_inline)) {
          const int row = (i / KS) * 32 + l32, c = (i % KS) * 2 + lh;
          return *reinterpret_cast<const bf16x8*>(&sK[buf][(row * CH + (c ^ k_swz<DH>(row))) * 16]);
        };
        bf16x8 kf[RA + 1];
#pragma unroll
        for (int i = 0; i < RA && i < N; ++i) kf[i] = read_k(i);
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb) {
#pragma unroll
          for (int r = 0; r < 16; ++r) s[kb][r] = 0.f;
          s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(onef, mf, s[kb], 0, 0, 0);
        }
        static_for<N>([&](auto Ic) __attribute__((always_inline)) {
          constexpr int i = decltype(Ic)::value;
          if (i + RA < N) kf[(i + RA) % (RA + 1)] = read_k(i + RA);
          __builtin_amdgcn_sched_barrier(0);
          s[i / KS] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[i % (RA + 1)], qf[i % KS], s[i / KS], 0, 0, 0);
          __builtin_amdgcn_sched_barrier(0);
        });
      }
      if (MASK) {  // keys past the end
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int key = k0 + kb * 32 + 8 * (r >> 2) + 4 * lh + (r & 3);
            if (key >= L) s[kb][r] = -INFINITY;
          }
      }
    };
    // p = 2^(s) (scores already in units of log2 e / sqrt(d)) or 2^(s scale): rounded to bf16 as the
    // column operand of the second product, step 2 kb + j; l_tile = this lane's sum of the rounded
    // values (what that product sums), two per instruction.
    bf16x8 pf[2 * NKB];
    float l_tile;
    auto probabilities = [&]() __attribute__((always_inline)) {
      l_tile = 0.f;
#pragma unroll
      for (int st = 0; st < 2 * NKB; ++st) {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float x = s[st >> 1][8 * (st & 1) + e];
          pf[st][e] = (bf16)__builtin_amdgcn_exp2f(PRE ? x : x * scale_log2);
        }
#pragma unroll
        for (int e = 0; e < 8; e += 2) {
          const bf16x2 pr = {pf[st][e], pf[st][e + 1]};
          l_tile = __builtin_amdgcn_fdot2_f32_bf16(pr, one2, l_tile, false);
        }
      }
    };
    // Softmax does not care which reference m is subtracted as long as numerator and denominator use
    // the same one; here it is whatever the query's running maximum was when it last had to move.
    // It has to move only when a probability would leave the comfortable range, and since
    // probabilities are positive that shows in the row sum the kernel forms anyway: no maximum is
    // taken on the way.  When some lane's sum of 32 probabilities passes 2^10 (or is not a number:
    // overflow), and on a wave's first tile, the scores are formed once more, the reference follows
    // the maximum (rounded to bf16; the accumulators are rescaled, 1 + DH/2 multiplications per lane)
    // and the probabilities are taken again.  With an exact running maximum nearly every tile of a
    // sequence rescales, and maximum, scale-and-subtract and rescale were half of the kernel's vector
    // instructions -- which on this chip are not hidden behind the matrix instructions.
    scores();
    probabilities();
    if (it == 0 || __builtin_amdgcn_ballot_w64(!(l_tile <= 1024.f)) != 0) {
      scores();
      float mx = -INFINITY;
#pragma unroll
      for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[kb][r]);
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      const float m_new = (float)(bf16)(m_run + (it == 0 ? mx : fmaxf(mx, 0.f)));
      const float delta = m_new - m_run;
      if (it != 0) {
        const float alpha = __builtin_amdgcn_exp2f(PRE ? -delta : -delta * scale_log2);
        l_run *= alpha;
#pragma unroll
        for (int d = 0; d < DB; ++d)
#pragma unroll
          for (int r = 0; r < 16; ++r) o[d][r] *= alpha;
      }
#pragma unroll
      for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) s[kb][r] -= delta;
      m_run = m_new;
      mf[0] = lh == 0 ? (bf16)(-m_new) : (bf16)0.f;
      probabilities();
    }
    l_run += l_tile;

    // O^T += V^T P^T; k-slot (lh, e) of step (kb, j) is key 32 kb + 16 j + 8 (e/4) + 4 lh + e%4
    const char __attribute__((address_space(3)))* vt = (const char __attribute__((address_space(3)))*)BR_LPTR(sV[buf]);
    if constexpr (RA == 0) {
#pragma unroll
      for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
#pragma unroll
          for (int d = 0; d < DB; ++d) {
            const auto* p0 = vt + vaddr[d] + (kb * 32 + j * 16) * ROW_B;
            const s16x4 v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)p0);
            const s16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(p0 + 8 * ROW_B));
            union { s16x4 s[2]; bf16x8 v; } u;
            u.s[0] = v0;
            u.s[1] = v1;
            o[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(u.v, pf[2 * kb + j], o[d], 0, 0, 0);
          }
        }
    } else {
      constexpr int N = 2 * NKB * DB;
      auto read_v = [&](int i) __attribute__((always_inline)) {
        const int st = i / DB, d = i % DB;  // step st = 2 kb + j covers keys 16 st .. 16 st + 15
        const auto* p0 = vt + vaddr[d] + st * 16 * ROW_B;
        union { s16x4 s[2]; bf16x8 v; } u;
        u.s[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)p0);
        u.s[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(p0 + 8 * ROW_B));
        return u.v;
      };
      bf16x8 vf[RA + 1];
#pragma unroll
      for (int i = 0; i < RA && i < N; ++i) vf[i] = read_v(i);
      static_for<N>([&](auto Ic) __attribute__((always_inline)) {
        constexpr int i = decltype(Ic)::value;
        if (i + RA < N) vf[(i + RA) % (RA + 1)] = read_v(i + RA);
        __builtin_amdgcn_sched_barrier(0);
        o[i % DB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[i % (RA + 1)], pf[i / DB], o[i % DB], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
      });
    }
    // the next tile has landed in this wave's share of the other buffer; after the barrier, in all of it
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
  };
  using K1 = std::integral_constant<int, 1>;
  using K2 = std::integral_constant<int, 2>;
  const int nfull = L / KV_TILE;
  using B0 = std::integral_constant<int, 0>;
  using B1 = std::integral_constant<int, 1>;
  if (active) {
    int it = 0;
    for (; it + 2 <= nfull; it += 2) {
      tile(it, K2{}, std::false_type{}, B0{});
      tile(it + 1, K2{}, std::false_type{}, B1{});
    }
    if (it < nfull) tile(it, K2{}, std::false_type{}, B0{});
    if (nfull < nkv) {
      const bool one = L - nfull * KV_TILE <= 32;
      if (nfull & 1) {
        if (one) tile(nfull, K1{}, std::true_type{}, B1{});
        else tile(nfull, K2{}, std::true_type{}, B1{});
      } else {
        if (one) tile(nfull, K1{}, std::true_type{}, B0{});
        else tile(nfull, K2{}, std::true_type{}, B0{});
      }
    }
  } else {
    // a wave whose 32 queries all lie past the end only keeps up its share of the tile traffic
    for (int it = 0; it < nkv; ++it) {
      issue(min(it + 1, nkv - 1) * KV_TILE, (it & 1) ^ 1);
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      __syncthreads();
    }
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


br_status launch_attention_bf16(const bf16* qkv, bf16* out, int B, int L, int NH, int DH, int q_prescaled, hipStream_t st) {
  BR_REQUIRE(L >= 1, BR_EINVAL, "attention: empty sequence");
  // the ragged last tile addresses its rows with 32-bit byte offsets from the sample's first row
  BR_REQUIRE((unsigned long long)L * 3ull * NH * DH * 2ull < (1ull << 32), BR_ESHAPE,
             "attention: one sample's QKV rows exceed 4 GiB");
  const long long n_pairs = (long long)B * NH;
  const int grouped = n_pairs >= 32 ? 1 : 0;
  const long long n_blocks = (grouped ? (n_pairs + 7) / 8 * 8 : n_pairs) * cdiv(L, 128);
  BR_REQUIRE(n_blocks <= 0x7FFFFFFFLL, BR_ESHAPE, "attention: too many workgroups for one launch");
  dim3 g((unsigned)n_blocks), blk(256);
  const float scale_log2 = (float)(1.4426950408889634 / sqrt((double)DH));
  const int H = NH * DH;
  ProfScope ps(st, PROF_ATTN + DH, 4.0 * B * (double)L * L * H);
#define BR_ATTN_GO(DHc, PREc) \
  hipLaunchKernelGGL((attn_bf16_kernel<DHc, PREc>), g, blk, 0, st, qkv, out, L, H, NH, (int)n_pairs, grouped, scale_log2)
  if (DH == 64 && q_prescaled) BR_ATTN_GO(64, true);
  else if (DH == 64) BR_ATTN_GO(64, false);
  else if (DH == 128 && q_prescaled) BR_ATTN_GO(128, true);
  else if (DH == 128) BR_ATTN_GO(128, false);
#undef BR_ATTN_GO
  else return fail(BR_ESHAPE, "bf16 attention: head dim must be 64 or 128");
  BR_LAUNCH_CHECK();
  return BR_OK;
}

}  // namespace br
