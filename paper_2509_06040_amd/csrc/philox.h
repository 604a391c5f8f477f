// Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy as
// 1, 2, 3", SC'11) and the uniform -> normal transform used for the branch noise
// of Eq. 2.  Counter = (element quad, node id, step, stream tag); key = the two
// halves of the 64-bit seed.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace br {

enum : uint32_t { TAG_ETA = 0, TAG_XI0 = 1, TAG_ROOT = 2, TAG_DEPTH = 3 };

struct PhiloxKey {
  uint32_t k0[10], k1[10];  // round keys: seed halves advanced by the Weyl constants
};

__host__ __device__ inline PhiloxKey philox_key(uint64_t seed) {
  PhiloxKey k;
  uint32_t a = (uint32_t)seed, b = (uint32_t)(seed >> 32);
  for (int r = 0; r < 10; ++r) {
    k.k0[r] = a;
    k.k1[r] = b;
    a += 0x9E3779B9u;
    b += 0xBB67AE85u;
  }
  return k;
}

__host__ __device__ inline void philox4x32_10(const PhiloxKey& key, uint32_t c0, uint32_t c1,
                                              uint32_t c2, uint32_t c3, uint32_t out[4]) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
    const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
    const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ key.k0[r];
    const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ key.k1[r];
    c1 = (uint32_t)p1;
    c3 = (uint32_t)p0;
    c0 = n0;
    c2 = n2;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// Top 23 bits centred in their cell: u = (2k+1)/2^24, exact in fp32, in (0, 1).
__device__ inline float philox_uniform(uint32_t x) {
  return (float)(x >> 9) * 1.1920928955078125e-07f + 5.9604644775390625e-08f;
}

// Four standard normals of one quad: Box-Muller on word pairs (0,1), (2,3); the
// first word of a pair gives the radius, the second the angle; cos to the even
// element, sin to the odd.  v_sin/v_cos take their argument in revolutions, so
// the uniform is the argument itself.
__device__ inline void philox_normal4(const PhiloxKey& key, uint32_t quad, uint32_t node, uint32_t step,
                                      uint32_t tag, float n[4]) {
  uint32_t w[4];
  philox4x32_10(key, quad, node, step, tag, w);
#pragma unroll
  for (int p = 0; p < 2; ++p) {
    const float ua = philox_uniform(w[2 * p]), ub = philox_uniform(w[2 * p + 1]);
    // -2 ln u = -2 ln2 * log2 u
    // hardware sqrt (1 ulp) without the denormal fix-up sequence: the argument is in [0, 34]
    const float r = __builtin_amdgcn_sqrtf(-1.3862943611198906f * __builtin_amdgcn_logf(ua));
    n[2 * p] = r * __builtin_amdgcn_cosf(ub);
    n[2 * p + 1] = r * __builtin_amdgcn_sinf(ub);
  }
}

}  // namespace br
