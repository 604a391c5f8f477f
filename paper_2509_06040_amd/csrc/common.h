// Internal declarations shared by the translation units of libbranchrollout.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_bf16.h>
#include <stdint.h>
#include <mutex>
#include <string>
#include <vector>

#include "../../include/branchrollout.h"

namespace br {

void set_error(const std::string& msg);
br_status fail(br_status code, const std::string& msg);

#define BR_REQUIRE(cond, code, msg)                       \
  do {                                                    \
    if (!(cond)) return ::br::fail((code), (msg));        \
  } while (0)

#define BR_HIP(call)                                                                  \
  do {                                                                                \
    hipError_t e_ = (call);                                                           \
    if (e_ != hipSuccess)                                                             \
      return ::br::fail(BR_EDEVICE, std::string(#call) + ": " + hipGetErrorString(e_)); \
  } while (0)

#define BR_LAUNCH_CHECK() BR_HIP(hipGetLastError())

// Compute units of the current device (cached per device; 256 if the query fails).
int device_cu_count();

static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
static inline int cdiv(long long a, long long b) { return (int)((a + b - 1) / b); }

// Maps sample b of a batch to its latent row and its condition: either explicit
// device arrays or the frontier formula row = (b / width) * n_nodes + off + b % width.
struct SampleMap {
  const int* rows;  // dev or nullptr
  const int* cond;  // dev or nullptr
  int n_nodes, off, width;
  const int* group = nullptr;  // dev or nullptr: modulation group of a sample (default: its condition)
};

// Streaming stores of four consecutive elements, for data that the writing kernel does not
// read again: the lines are not kept in the cache of the compute die that wrote them, which
// leaves that cache to the operands still in use.
__device__ inline void store4_stream(float* p, float a, float b, float c, float d) {
  typedef float f32x4 __attribute__((ext_vector_type(4)));
  f32x4 v = {a, b, c, d};
  __builtin_nontemporal_store(v, reinterpret_cast<f32x4*>(p));
}
__device__ inline void store4_stream(__bf16* p, float a, float b, float c, float d) {
  typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
  bf16x4 v = {(__bf16)a, (__bf16)b, (__bf16)c, (__bf16)d};
  __builtin_nontemporal_store(v, reinterpret_cast<bf16x4*>(p));
}

}  // namespace br

namespace br {
// Pinned host staging for small host -> device uploads that must not make the caller wait: upload()
// copies `n` ints into pinned memory owned by this object and enqueues the transfer on `st`.  Before
// the pinned buffer is written again, the host waits for the previous transfer out of it (an event
// recorded behind that transfer), which has long finished unless uploads follow each other
// immediately.  The first use, and every growth, allocates (hipHostMalloc).  Serialised by a mutex.
struct PinnedStage {
  int* host = nullptr;
  size_t cap = 0;
  hipEvent_t ev = nullptr;
  bool pending = false;
  std::mutex mu;
  br_status upload(const int* src, size_t n, int* dst_dev, hipStream_t st);
  ~PinnedStage();
};
}  // namespace br

struct br_tree {
  int T, K, n_tree, n_nodes, n_leaves;
  std::vector<int> splits;         // effective (empty when K == 1)
  std::vector<uint8_t> is_split;   // [T]
  std::vector<int> width, off;     // [T+1], [T+2]
  std::vector<int> parent, depth, branch, leaf_lo, leaf_hi;  // [n_nodes]
  // lazily created device mirror: off[T+2], parent, depth, leaf_lo, leaf_hi, first_child, n_child
  mutable int* d_mem = nullptr;
  mutable int d_device = -1;
  mutable br::PinnedStage plan_stage;  // launch plans of br_logprob
  std::vector<int> first_child, n_child;
};

namespace br {
struct TreeDev {
  const int *off, *parent, *depth, *leaf_lo, *leaf_hi, *first_child, *n_child;
};
br_status tree_device(const br_tree* t, TreeDev* out);

// host Philox word (used by the seeded depth mask)
void philox_host(uint64_t seed, uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t out[4]);
}  // namespace br
