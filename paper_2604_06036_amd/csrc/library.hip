// Library identification and per-thread HIP error bookkeeping.
#include "common.h"

namespace {
thread_local int g_last_hip_error = 0;
}

namespace cs {
int note_hip(hipError_t e) {
  if (e == hipSuccess) return CS_OK;
  g_last_hip_error = static_cast<int>(e);
  return CS_EHIP;
}
}  // namespace cs

extern "C" const char* cs_version(void) { return "codecsight-mi355x 0.1 (gfx950)"; }

extern "C" int cs_last_hip_error(void) { return g_last_hip_error; }
