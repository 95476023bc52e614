// Optional HIP-event timing of one chosen kernel (benchmark aid; off by default).
#pragma once
#include <hip/hip_runtime.h>

namespace roco {

enum ProfKernel : int {
  kProfDecodeSelect = 0, kProfDecodeAttend = 1, kProfDecodeFinish = 2,
  kProfPrefillRows = 3, kProfPrefillColumns = 4, kProfPrefillSelect = 5, kProfPrefillGather = 6, kProfReadProbe = 7,
  kProfBlockPrepare = 8, kProfBlockAttend = 9, kProfBlockFinish = 10,
  kProfMfmaProbe = 11,
  kProfKernels = 12
};

extern int g_prof_which;  // -1 = off
extern int g_prof_every;  // bracket every n-th launch of the profiled kernel (event records cost a few microseconds)
extern int g_prof_count;
void prof_record(hipStream_t s, bool begin);

// Brackets one kernel launch with events when that kernel is the profiled one.
struct ProfScope {
  hipStream_t s;
  bool on;
  ProfScope(int which, hipStream_t stream) : s(stream), on(which == g_prof_which) {
    if (on) on = (g_prof_count++ % g_prof_every) == 0;
    if (on) prof_record(s, true);
  }
  ~ProfScope() {
    if (on) prof_record(s, false);
  }
};

}  // namespace roco
