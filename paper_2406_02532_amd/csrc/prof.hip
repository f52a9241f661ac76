// Optional per-kernel timing with HIP events, recorded on the caller's stream around individual
// launches.  Off by default (the hooks are a branch on a flag); a benchmark switches it on to get
// the duration of each kernel class inside its own timed region.
#include <vector>

#include "kernels.h"

namespace {
struct Prof {
  bool on = false, skip = false;
  int cap = 0, n = 0, only = 0;  // only != 0: time launches of that kernel class alone
  std::vector<hipEvent_t> beg, end;
  std::vector<int> tag;
} g_prof;
}  // namespace

void sx_prof_begin(int tag, hipStream_t st) {
  g_prof.skip = g_prof.only != 0 && tag != g_prof.only;
  if (!g_prof.on || g_prof.skip || g_prof.n >= g_prof.cap) return;
  g_prof.tag[g_prof.n] = tag;
  (void)hipEventRecord(g_prof.beg[g_prof.n], st);
}
void sx_prof_end(hipStream_t st) {
  if (!g_prof.on || g_prof.skip || g_prof.n >= g_prof.cap) return;
  (void)hipEventRecord(g_prof.end[g_prof.n], st);
  ++g_prof.n;
}

extern "C" int sx_profile_enable(int32_t max_records) {
  if (max_records < 1 || max_records > (1 << 20)) return SX_ERR_SHAPE;
  while (g_prof.cap < max_records) {
    hipEvent_t a, b;
    SX_HIP_TRY(hipEventCreate(&a));
    SX_HIP_TRY(hipEventCreate(&b));
    g_prof.beg.push_back(a);
    g_prof.end.push_back(b);
    g_prof.tag.push_back(0);
    ++g_prof.cap;
  }
  g_prof.n = 0;
  g_prof.on = true;
  return SX_OK;
}

extern "C" int sx_profile_select(int32_t kernel_class) {
  if (kernel_class < 0) return SX_ERR_SHAPE;
  g_prof.only = kernel_class;
  return SX_OK;
}

extern "C" int sx_profile_disable(void) {
  g_prof.on = false;
  return SX_OK;
}

extern "C" int sx_profile_read(int32_t* tags, float* ms, int32_t cap, int32_t* n_out) {
  if (!tags || !ms || !n_out) return SX_ERR_NULL;
  const int n = g_prof.n < cap ? g_prof.n : cap;
  for (int i = 0; i < n; ++i) {
    SX_HIP_TRY(hipEventSynchronize(g_prof.end[i]));
    float t = 0.f;
    SX_HIP_TRY(hipEventElapsedTime(&t, g_prof.beg[i], g_prof.end[i]));
    tags[i] = g_prof.tag[i];
    ms[i] = t;
  }
  *n_out = n;
  g_prof.n = 0;
  return SX_OK;
}
