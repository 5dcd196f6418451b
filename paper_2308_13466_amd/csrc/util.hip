// Status strings, last-error slot and version of libsat.
#include "sat_internal.h"

namespace sat {
static thread_local int32_t g_last_hip_error = 0;
void set_last_hip_error(hipError_t e) { g_last_hip_error = static_cast<int32_t>(e); }
}  // namespace sat

extern "C" const char* sat_status_string(sat_status s) {
  switch (s) {
    case SAT_OK: return "SAT_OK";
    case SAT_EINVAL: return "SAT_EINVAL: null pointer, negative size, ld < d or inconsistent sizes";
    case SAT_EUNSUPPORTED: return "SAT_EUNSUPPORTED: element type or dimension not compiled in";
    case SAT_EALIGN: return "SAT_EALIGN: pointer or leading dimension breaks an alignment requirement";
    case SAT_EWORKSPACE: return "SAT_EWORKSPACE: workspace missing or too small";
    case SAT_EHIP: return "SAT_EHIP: a HIP call failed (see sat_last_hip_error)";
    default: return "unknown sat_status";
  }
}

extern "C" int32_t sat_last_hip_error(void) { return sat::g_last_hip_error; }

extern "C" int32_t sat_version(void) { return 0 * 10000 + 1 * 100 + 0; }
