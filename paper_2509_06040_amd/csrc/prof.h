// Optional per-launch timing with HIP events on the launch stream (off by default).
#pragma once
#include <hip/hip_runtime.h>

namespace br {
enum ProfId {
  PROF_GEMM = 0,        // + epilogue * 8 + variant
  PROF_ATTN = 100,      // + head dim
  PROF_SDE_STEP = 200,
  PROF_LOGP_EVAL = 201,
  PROF_LN_MOD = 300,
  PROF_ADALN = 301,     // the adaLN modulation GEMV (weight streaming)
};
bool prof_on();
void prof_begin(hipStream_t st, int id, double work);  // work: flops or bytes of this launch
void prof_end(hipStream_t st);
// Inside a chain every launch on the stream is an instrumented one, back to back: the event
// that closes one launch also opens the next, which halves the events put between kernels.
void prof_chain(bool on);
struct ProfChain {
  bool on;
  explicit ProfChain(bool enable) : on(enable && prof_on()) {
    if (on) prof_chain(true);
  }
  ~ProfChain() {
    if (on) prof_chain(false);
  }
};
struct ProfScope {
  hipStream_t st;
  bool on;
  ProfScope(hipStream_t s, int id, double work) : st(s), on(prof_on()) {
    if (on) prof_begin(st, id, work);
  }
  ~ProfScope() {
    if (on) prof_end(st);
  }
};
}  // namespace br
