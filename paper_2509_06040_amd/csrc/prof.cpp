// Per-launch timing: an event pair around each instrumented launch, summed per
// kernel id when read.  Not thread-safe; meant for a single benchmarking thread.
#include <map>
#include <vector>

#include "../../include/branchrollout_ops.h"
#include "common.h"
#include "prof.h"

namespace br {
namespace {
struct Rec {
  int id;
  double work;
  hipEvent_t a, b;
  bool shared_a;  // `a` is the previous record's `b`
};
bool g_on = false;
bool g_chain = false;
hipEvent_t g_chain_prev = nullptr;  // closing event of the last launch of the running chain
hipStream_t g_chain_stream = nullptr;
std::vector<Rec> g_recs;
std::vector<hipEvent_t> g_pool;
hipEvent_t get_event() {
  if (!g_pool.empty()) {
    hipEvent_t e = g_pool.back();
    g_pool.pop_back();
    return e;
  }
  hipEvent_t e = nullptr;
  (void)hipEventCreate(&e);
  return e;
}
}  // namespace

bool prof_on() { return g_on; }
void prof_chain(bool on) {
  g_chain = on;
  g_chain_prev = nullptr;
}
void prof_begin(hipStream_t st, int id, double work) {
  const bool share = g_chain && g_chain_prev != nullptr && g_chain_stream == st;
  Rec r{id, work, share ? g_chain_prev : get_event(), get_event(), share};
  if (!share) (void)hipEventRecord(r.a, st);
  g_recs.push_back(r);
}
void prof_end(hipStream_t st) {
  (void)hipEventRecord(g_recs.back().b, st);
  if (g_chain) {
    g_chain_prev = g_recs.back().b;
    g_chain_stream = st;
  }
}
}  // namespace br

using namespace br;

extern "C" br_status br_profile_enable(int32_t on) {
  g_on = on != 0;
  return BR_OK;
}

extern "C" br_status br_profile_read(int32_t max_ids, int32_t* ids, double* work, double* ms, int64_t* launches,
                                     int32_t* n_ids) {
  BR_REQUIRE(ids && work && ms && launches && n_ids && max_ids >= 0, BR_EINVAL, "br_profile_read: NULL argument");
  std::map<int, std::pair<std::pair<double, double>, long long>> agg;
  for (Rec& r : g_recs) {
    BR_HIP(hipEventSynchronize(r.b));
    float t = 0.f;
    BR_HIP(hipEventElapsedTime(&t, r.a, r.b));
    auto& a = agg[r.id];
    a.first.first += r.work;
    a.first.second += t;
    a.second += 1;
    if (!r.shared_a) g_pool.push_back(r.a);
    g_pool.push_back(r.b);
  }
  g_recs.clear();
  int n = 0;
  for (auto& kv : agg) {
    if (n >= max_ids) break;
    ids[n] = kv.first;
    work[n] = kv.second.first.first;
    ms[n] = kv.second.first.second;
    launches[n] = kv.second.second;
    ++n;
  }
  *n_ids = n;
  return BR_OK;
}
