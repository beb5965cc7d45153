// Status strings and the per-thread record of the last HIP error.
#include "common.h"
#include <vector>

namespace gptaq {
static thread_local int g_last_hip_error = 0;
void set_last_hip_error(hipError_t e) { g_last_hip_error = (int)e; }
}  // namespace gptaq

namespace gptaq {
namespace {
struct ProfState {
  unsigned mask = 0;
  std::vector<hipEvent_t> ev[kProfTags];     // begin/end pairs, in launch order
  size_t used[kProfTags] = {0};
} g_prof;
}  // namespace
bool prof_enabled(int tag) { return (g_prof.mask >> tag) & 1u; }
void prof_mark(int tag, hipStream_t s, bool begin) {
  std::vector<hipEvent_t>& v = g_prof.ev[tag];
  size_t& u = g_prof.used[tag];
  if (begin && (u & 1)) return;                 // unbalanced: ignore
  if (u == v.size()) {
    hipEvent_t e;
    if (hipEventCreate(&e) != hipSuccess) return;
    v.push_back(e);
  }
  if (hipEventRecord(v[u], s) == hipSuccess) ++u;
}
}  // namespace gptaq

namespace gptaq {
namespace {
std::mutex g_side_mutex;
SideStream g_side[64];
}  // namespace
std::mutex& side_stream_mutex() { return g_side_mutex; }
SideStream* side_stream(int nevents) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return nullptr;
  SideStream& ss = g_side[dev];
  if (!ss.stream && hipStreamCreateWithFlags(&ss.stream, hipStreamNonBlocking) != hipSuccess) return nullptr;
  while ((int)ss.events.size() < nevents) {
    hipEvent_t e;
    if (hipEventCreateWithFlags(&e, hipEventDisableTiming) != hipSuccess) return nullptr;
    ss.events.push_back(e);
  }
  return &ss;
}
}  // namespace gptaq

extern "C" int gptaq_profile_enable(int mask) {
  using namespace gptaq;
  g_prof.mask = (unsigned)mask;
  for (int t = 0; t < kProfTags; ++t) g_prof.used[t] = 0;
  return GPTAQ_OK;
}

extern "C" int gptaq_profile_read(int tag, int64_t* launches, double* total_ms) {
  using namespace gptaq;
  if (tag < 0 || tag >= kProfTags || !launches || !total_ms) return GPTAQ_EDIM;
  double ms = 0.0;
  const size_t pairs = g_prof.used[tag] / 2;
  for (size_t i = 0; i < pairs; ++i) {
    if (hipEventSynchronize(g_prof.ev[tag][2 * i + 1]) != hipSuccess) return GPTAQ_ELAUNCH;
    float t = 0.f;
    if (hipEventElapsedTime(&t, g_prof.ev[tag][2 * i], g_prof.ev[tag][2 * i + 1]) != hipSuccess) return GPTAQ_ELAUNCH;
    ms += (double)t;
  }
  *launches = (int64_t)pairs;
  *total_ms = ms;
  return GPTAQ_OK;
}

extern "C" const char* gptaq_status_string(int status) {
  switch (status) {
    case GPTAQ_OK: return "ok";
    case GPTAQ_ENULL: return "a required pointer is NULL";
    case GPTAQ_EDIM: return "dimension, leading dimension or alignment out of range";
    case GPTAQ_EUNSUPPORTED: return "unsupported bits/group/blocksize combination";
    case GPTAQ_EWORKSPACE: return "workspace too small or not 256-byte aligned";
    case GPTAQ_ELAUNCH: return "HIP launch failed";
    case GPTAQ_ETOOLARGE: return "problem larger than the library's built-in scratch buffer allows";
    default: return "unknown status";
  }
}

extern "C" int gptaq_last_hip_error(void) { return gptaq::g_last_hip_error; }
