// Library-wide entry points: version and error bookkeeping.
#include "common.h"

namespace graft {
static thread_local int32_t g_last_hip_error = 0;
void set_last_hip_error(int32_t e) { g_last_hip_error = e; }
}  // namespace graft

extern "C" int32_t graft_last_hip_error(void) { return graft::g_last_hip_error; }
extern "C" int32_t graft_version(void) { return 100; }
