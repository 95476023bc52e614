#include "profile.hpp"

#include <vector>

#include "../../include/roco.h"

namespace roco {

int g_prof_which = -1;
int g_prof_every = 1;
int g_prof_count = 0;

namespace {
std::vector<hipEvent_t> g_events;  // pairs: [2i] start, [2i+1] stop
size_t g_used = 0;                 // events handed out since the last read
}  // namespace

void prof_record(hipStream_t s, bool begin) {
  if (begin && (g_used & 1u)) return;    // unbalanced; ignore
  if (!begin && !(g_used & 1u)) return;
  if (g_used == g_events.size()) {
    hipEvent_t e;
    if (hipEventCreate(&e) != hipSuccess) { g_prof_which = -1; return; }
    g_events.push_back(e);
  }
  (void)hipEventRecord(g_events[g_used++], s);
}

}  // namespace roco

extern "C" {

int roco_profile_kernel(int which) {
  if (which < -1 || which >= ROCO_PROF_KERNELS) return ROCO_EINVAL;
  roco::g_prof_which = which;
  roco::g_prof_count = 0;
  return ROCO_OK;
}

int roco_profile_sampling(int every) {
  if (every < 1) return ROCO_EINVAL;
  roco::g_prof_every = every;
  roco::g_prof_count = 0;
  return ROCO_OK;
}

int roco_profile_read(double* total_ms, int64_t* launches) {
  using namespace roco;
  double sum = 0.0;
  int64_t n = 0;
  for (size_t i = 0; i + 1 < g_used; i += 2) {
    float ms = 0.0f;
    if (hipEventSynchronize(g_events[i + 1]) != hipSuccess) return ROCO_EHIP;
    if (hipEventElapsedTime(&ms, g_events[i], g_events[i + 1]) != hipSuccess) return ROCO_EHIP;
    sum += ms;
    ++n;
  }
  g_used = 0;
  if (total_ms) *total_ms = sum;
  if (launches) *launches = n;
  return ROCO_OK;
}

}  // extern "C"
