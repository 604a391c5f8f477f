// Rollout-tree topology (Sec. 3.2 "Preliminaries"; Alg. 1, tree-building loop) and
// the depth-pruning masks (Sec. 3.4), host side.
#include <algorithm>
#include <cmath>
#include <new>
#include <mutex>
#include <numeric>

#include "common.h"
#include "philox.h"

namespace br {

static thread_local std::string g_err;
void set_error(const std::string& msg) { g_err = msg; }
br_status fail(br_status code, const std::string& msg) {
  g_err = msg;
  return code;
}

void philox_host(uint64_t seed, uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t out[4]) {
  const PhiloxKey k = philox_key(seed);
  philox4x32_10(k, c0, c1, c2, c3, out);
}

int device_cu_count() {
  static int cached[64] = {0};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
  if (cached[dev] == 0) {
    int n = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
    cached[dev] = n;
  }
  return cached[dev];
}

br_status PinnedStage::upload(const int* src, size_t n, int* dst_dev, hipStream_t st) {
  if (n == 0) return BR_OK;
  std::lock_guard<std::mutex> lock(mu);
  if (pending) {  // the previous transfer reads the buffer: let it finish before overwriting
    BR_HIP(hipEventSynchronize(ev));
    pending = false;
  }
  if (n > cap) {
    if (host) (void)hipHostFree(host);
    host = nullptr;
    cap = 0;
    const size_t want = n + n / 2 + 256;
    if (hipHostMalloc((void**)&host, want * sizeof(int), hipHostMallocDefault) != hipSuccess || !host) {
      host = nullptr;
      return fail(BR_ENOMEM, "pinned staging buffer: host allocation failed");
    }
    cap = want;
  }
  if (!ev) BR_HIP(hipEventCreateWithFlags(&ev, hipEventDisableTiming));
  std::copy(src, src + n, host);
  BR_HIP(hipMemcpyAsync(dst_dev, host, n * sizeof(int), hipMemcpyHostToDevice, st));
  BR_HIP(hipEventRecord(ev, st));
  pending = true;
  return BR_OK;
}

PinnedStage::~PinnedStage() {
  if (pending && ev) (void)hipEventSynchronize(ev);
  if (host) (void)hipHostFree(host);
  if (ev) (void)hipEventDestroy(ev);
}

br_status tree_device(const br_tree* t, TreeDev* out) {
  // one mirror per tree, created by br_tree_upload or by the first call that needs it; the
  // lock makes that first call safe when several threads share one tree
  static std::mutex mu;
  std::lock_guard<std::mutex> lock(mu);
  int dev = 0;
  BR_HIP(hipGetDevice(&dev));
  const size_t nn = (size_t)t->n_nodes, noff = (size_t)t->T + 2;
  if (t->d_mem && t->d_device != dev) {
    (void)hipFree(t->d_mem);
    t->d_mem = nullptr;
  }
  if (!t->d_mem) {
    std::vector<int> h(noff + 6 * nn);
    std::copy(t->off.begin(), t->off.end(), h.begin());
    const std::vector<int>* arrs[6] = {&t->parent, &t->depth, &t->leaf_lo, &t->leaf_hi, &t->first_child, &t->n_child};
    for (int a = 0; a < 6; ++a) std::copy(arrs[a]->begin(), arrs[a]->end(), h.begin() + noff + a * nn);
    int* d = nullptr;
    if (hipMalloc((void**)&d, h.size() * sizeof(int)) != hipSuccess || !d)
      return fail(BR_ENOMEM, "tree: device allocation of the topology arrays failed");
    hipError_t e = hipMemcpy(d, h.data(), h.size() * sizeof(int), hipMemcpyHostToDevice);
    if (e != hipSuccess) {
      (void)hipFree(d);
      return fail(BR_EDEVICE, std::string("hipMemcpy(tree): ") + hipGetErrorString(e));
    }
    t->d_mem = d;
    t->d_device = dev;
  }
  const int* d = t->d_mem;
  out->off = d;
  out->parent = d + noff;
  out->depth = d + noff + nn;
  out->leaf_lo = d + noff + 2 * nn;
  out->leaf_hi = d + noff + 3 * nn;
  out->first_child = d + noff + 4 * nn;
  out->n_child = d + noff + 5 * nn;
  return BR_OK;
}

}  // namespace br

using namespace br;

extern "C" const char* br_last_error(void) { return g_err.c_str(); }

extern "C" br_status br_tree_build(int32_t T, const int32_t* split_steps, int32_t n_splits, int32_t K,
                                   int32_t n_tree, br_tree** out) {
  BR_REQUIRE(out != nullptr, BR_EINVAL, "br_tree_build: out is NULL");
  BR_REQUIRE(T >= 1 && T <= 1024, BR_EINVAL, "br_tree_build: T must be in [1, 1024]");
  BR_REQUIRE(K >= 1, BR_EINVAL, "br_tree_build: K must be >= 1");
  BR_REQUIRE(n_tree >= 1, BR_EINVAL, "br_tree_build: n_tree must be >= 1");
  BR_REQUIRE(n_splits >= 0 && (n_splits == 0 || split_steps != nullptr), BR_EINVAL,
             "br_tree_build: split_steps is NULL or n_splits < 0");
  for (int i = 0; i < n_splits; ++i) {
    BR_REQUIRE(split_steps[i] >= 0 && split_steps[i] < T, BR_EINVAL, "br_tree_build: split step outside [0, T)");
    BR_REQUIRE(i == 0 || split_steps[i] > split_steps[i - 1], BR_EINVAL,
               "br_tree_build: split steps must be strictly ascending");
  }
  br_tree* t = new (std::nothrow) br_tree();
  BR_REQUIRE(t != nullptr, BR_ENOMEM, "br_tree_build: out of host memory");
  t->T = T;
  t->K = K;
  t->n_tree = n_tree;
  t->is_split.assign(T, 0);
  if (K > 1)
    for (int i = 0; i < n_splits; ++i) {
      t->splits.push_back(split_steps[i]);
      t->is_split[split_steps[i]] = 1;
    }
  // widths and level offsets, guarding the int32 range of global node ids
  t->width.assign(T + 1, 1);
  t->off.assign(T + 2, 0);
  long long total = 0;
  for (int d = 0; d <= T; ++d) {
    long long w = d == 0 ? 1 : (long long)t->width[d - 1] * (t->is_split[d - 1] ? K : 1);
    total += w;
    if (w > INT32_MAX || total * n_tree > INT32_MAX) {
      delete t;
      return fail(BR_EINVAL, "br_tree_build: n_tree * n_nodes does not fit in int32");
    }
    t->width[d] = (int)w;
    t->off[d + 1] = (int)total;
  }
  const int nn = (int)total;
  t->n_nodes = nn;
  t->n_leaves = t->width[T];
  t->parent.assign(nn, -1);
  t->depth.assign(nn, 0);
  t->branch.assign(nn, 0);
  t->leaf_lo.assign(nn, 0);
  t->leaf_hi.assign(nn, 0);
  t->first_child.assign(nn, -1);
  t->n_child.assign(nn, 0);
  for (int d = 0; d <= T; ++d) {
    const int span = t->n_leaves / t->width[d];  // leaves under each node of this depth
    for (int j = 0; j < t->width[d]; ++j) {
      const int n = t->off[d] + j;
      t->depth[n] = d;
      t->leaf_lo[n] = j * span;
      t->leaf_hi[n] = (j + 1) * span;
      if (d > 0) {
        const bool sp = t->is_split[d - 1];
        t->parent[n] = t->off[d - 1] + (sp ? j / K : j);
        t->branch[n] = sp ? j % K : 0;
      }
      if (d < T) {
        const bool sp = t->is_split[d];
        t->first_child[n] = t->off[d + 1] + (sp ? j * K : j);
        t->n_child[n] = sp ? K : 1;
      }
    }
  }
  *out = t;
  return BR_OK;
}

extern "C" br_status br_tree_info(const br_tree* t, int32_t* n_nodes, int32_t* n_edges, int32_t* n_leaves,
                                  int32_t* n_tree, const int32_t** width, const int32_t** off,
                                  const int32_t** parent, const int32_t** depth, const int32_t** branch,
                                  const int32_t** leaf_lo, const int32_t** leaf_hi) {
  BR_REQUIRE(t != nullptr, BR_EINVAL, "br_tree_info: tree is NULL");
  if (n_nodes) *n_nodes = t->n_nodes;
  if (n_edges) *n_edges = t->n_nodes - 1;
  if (n_leaves) *n_leaves = t->n_leaves;
  if (n_tree) *n_tree = t->n_tree;
  if (width) *width = t->width.data();
  if (off) *off = t->off.data();
  if (parent) *parent = t->parent.data();
  if (depth) *depth = t->depth.data();
  if (branch) *branch = t->branch.data();
  if (leaf_lo) *leaf_lo = t->leaf_lo.data();
  if (leaf_hi) *leaf_hi = t->leaf_hi.data();
  return BR_OK;
}

extern "C" br_status br_tree_upload(const br_tree* t) {
  BR_REQUIRE(t != nullptr, BR_EINVAL, "br_tree_upload: tree is NULL");
  TreeDev td;
  return tree_device(t, &td);
}

extern "C" void br_tree_free(br_tree* t) {
  if (!t) return;
  if (t->d_mem) (void)hipFree(t->d_mem);
  delete t;
}

extern "C" br_status br_depth_mask_window(int32_t T, int32_t last_split, int32_t window, int32_t iter,
                                          int32_t every, int32_t stop, uint8_t* mask_out) {
  BR_REQUIRE(mask_out != nullptr, BR_EINVAL, "br_depth_mask_window: mask_out is NULL");
  BR_REQUIRE(T >= 1 && window >= 0 && iter >= 0 && every >= 1 && last_split >= 0 && stop >= 0, BR_EINVAL,
             "br_depth_mask_window: arguments out of range");
  int start = std::min(last_split + iter / every, stop - window);
  start = std::max(start, 0);
  for (int i = 0; i < T; ++i) mask_out[i] = (i >= start && i < start + window) ? 1 : 0;
  return BR_OK;
}

extern "C" br_status br_mix_schedule(int32_t T, const int32_t* split_steps, int32_t n_splits,
                                     const uint8_t* window_mask, float eta, float* sigma_out, uint8_t* ode_mask_out) {
  BR_REQUIRE(sigma_out != nullptr && ode_mask_out != nullptr && window_mask != nullptr, BR_EINVAL,
             "br_mix_schedule: NULL argument");
  BR_REQUIRE(T >= 1 && n_splits >= 0 && (n_splits == 0 || split_steps != nullptr), BR_EINVAL,
             "br_mix_schedule: arguments out of range");
  BR_REQUIRE(std::isfinite(eta) && eta > 0.f, BR_EINVAL, "br_mix_schedule: eta must be positive");
  for (int i = 0; i < n_splits; ++i)
    BR_REQUIRE(split_steps[i] >= 0 && split_steps[i] < T, BR_EINVAL, "br_mix_schedule: split step outside [0, T)");
  for (int i = 0; i < T; ++i) {
    bool sde = window_mask[i] != 0;
    for (int k = 0; k < n_splits; ++k) sde = sde || split_steps[k] == i;
    sigma_out[i] = sde ? eta : 0.f;
    ode_mask_out[i] = sde ? 0 : 1;
  }
  return BR_OK;
}

extern "C" br_status br_depth_mask_seeded(int32_t T, int32_t n_drop, uint64_t seed, uint8_t* mask_out) {
  BR_REQUIRE(mask_out != nullptr, BR_EINVAL, "br_depth_mask_seeded: mask_out is NULL");
  BR_REQUIRE(T >= 1 && n_drop >= 0 && n_drop <= T, BR_EINVAL, "br_depth_mask_seeded: need 0 <= n_drop <= T");
  std::vector<std::pair<uint32_t, int>> key(T);
  for (int i = 0; i < T; ++i) {
    uint32_t w[4];
    philox_host(seed, 0u, 0u, (uint32_t)i, TAG_DEPTH, w);
    key[i] = {w[0], i};
  }
  std::sort(key.begin(), key.end());
  for (int i = 0; i < T; ++i) mask_out[i] = 0;
  for (int i = 0; i < n_drop; ++i) mask_out[key[i].second] = 1;
  return BR_OK;
}
