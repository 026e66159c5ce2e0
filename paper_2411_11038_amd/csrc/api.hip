// Library-level entry points that are not tied to one kernel family.
#include "common.hpp"

extern "C" int efqat_version(void) { return EFQAT_VERSION; }

extern "C" const char* efqat_strerror(int code) {
  switch (code) {
    case EFQAT_OK: return "ok";
    case EFQAT_ERR_NULL_PTR: return "a required pointer is NULL";
    case EFQAT_ERR_BAD_SHAPE: return "a dimension is non-positive or too large";
    case EFQAT_ERR_BAD_BITS: return "bit width outside 2..8";
    case EFQAT_ERR_BAD_K: return "k outside 0..C_out";
    case EFQAT_ERR_BAD_LAYOUT: return "unknown layout / mode flag";
    case EFQAT_ERR_WORKSPACE: return "workspace too small";
    case EFQAT_ERR_HIP: return "a HIP call or kernel launch failed";
    case EFQAT_ERR_BAD_DTYPE: return "unknown element type";
    case EFQAT_ERR_ALIGNMENT: return "a pointer is not aligned as required";
    default: return "unknown error code";
  }
}

// ---- optional event timing of kernel classes (benchmarks only; off by default, not thread-safe)
namespace efqat {

static const int kMaxProf = 4096;
static bool g_prof_on = false;
static hipEvent_t g_prof_ev[PROF_CLASSES][kMaxProf][2];
static int g_prof_made[PROF_CLASSES];
static int g_prof_used[PROF_CLASSES];

bool prof_begin(int which, hipStream_t st, int* slot) {
  if (!g_prof_on || g_prof_used[which] >= kMaxProf) return false;
  const int i = g_prof_used[which];
  if (i >= g_prof_made[which]) {
    if (hipEventCreate(&g_prof_ev[which][i][0]) != hipSuccess) return false;
    if (hipEventCreate(&g_prof_ev[which][i][1]) != hipSuccess) return false;
    g_prof_made[which] = i + 1;
  }
  if (hipEventRecord(g_prof_ev[which][i][0], st) != hipSuccess) return false;
  *slot = i;
  return true;
}

void prof_end(int which, hipStream_t st, int slot) {
  if (hipEventRecord(g_prof_ev[which][slot][1], st) == hipSuccess) g_prof_used[which] = slot + 1;
}

}  // namespace efqat

extern "C" int efqat_profile_enable(int on) {
  efqat::g_prof_on = on != 0;
  for (int c = 0; c < efqat::PROF_CLASSES; ++c) efqat::g_prof_used[c] = 0;
  return EFQAT_OK;
}

extern "C" int efqat_profile_read(int which, double* total_ms, int64_t* launches) {
  if (which < 0 || which >= efqat::PROF_CLASSES) return EFQAT_ERR_BAD_LAYOUT;
  if (!total_ms || !launches) return EFQAT_ERR_NULL_PTR;
  double sum = 0.0;
  const int n = efqat::g_prof_used[which];
  for (int i = 0; i < n; ++i) {
    float ms = 0.0f;
    if (hipEventSynchronize(efqat::g_prof_ev[which][i][1]) != hipSuccess) return EFQAT_ERR_HIP;
    if (hipEventElapsedTime(&ms, efqat::g_prof_ev[which][i][0], efqat::g_prof_ev[which][i][1]) != hipSuccess)
      return EFQAT_ERR_HIP;
    sum += (double)ms;
  }
  *total_ms = sum;
  *launches = n;
  return EFQAT_OK;
}
