// Status strings and the per-thread record of the last HIP error.
#include "common.h"

namespace gptaq {
static thread_local int g_last_hip_error = 0;
void set_last_hip_error(hipError_t e) { g_last_hip_error = (int)e; }
}  // namespace gptaq

extern "C" const char* gptaq_status_string(int status) {
  switch (status) {
    case GPTAQ_OK: return "ok";
    case GPTAQ_ENULL: return "a required pointer is NULL";
    case GPTAQ_EDIM: return "dimension, leading dimension or alignment out of range";
    case GPTAQ_EUNSUPPORTED: return "unsupported bits/group/blocksize combination";
    case GPTAQ_EWORKSPACE: return "workspace too small or not 256-byte aligned";
    case GPTAQ_ELAUNCH: return "HIP launch failed";
    default: return "unknown status";
  }
}

extern "C" int gptaq_last_hip_error(void) { return gptaq::g_last_hip_error; }
