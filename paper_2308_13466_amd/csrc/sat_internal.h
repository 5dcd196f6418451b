// Internal helpers shared by the library's translation units (not installed).
#ifndef SAT_INTERNAL_H_
#define SAT_INTERNAL_H_

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/sat.h"

namespace sat {

// Records the hipError_t behind the calling thread's last SAT_EHIP.
void set_last_hip_error(hipError_t e);

inline sat_status check_launch() {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) {
    set_last_hip_error(e);
    return SAT_EHIP;
  }
  return SAT_OK;
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline bool aligned256(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 255u) == 0; }

constexpr int kWave = 64;

}  // namespace sat

#endif  // SAT_INTERNAL_H_
