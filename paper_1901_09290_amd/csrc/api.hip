// Library-level entry points: version and the last HIP error seen by any call.
#include <atomic>

#include "common.h"

namespace pt {
static std::atomic<int32_t> g_last_hip_error{0};
void set_hip_error(hipError_t e) { g_last_hip_error.store((int32_t)e); }
}  // namespace pt

extern "C" int32_t pt_version(void) { return 100; }
extern "C" int32_t pt_last_hip_error(void) { return pt::g_last_hip_error.load(); }
