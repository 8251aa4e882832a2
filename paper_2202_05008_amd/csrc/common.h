// Internal helpers of the gfx950 library: error reporting and launch checks.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <stdarg.h>

#include "../../include/evo.h"

namespace evo {

// Thread-local message behind evo_last_error().
void set_error(const char* fmt, ...);

inline int fail(int code, const char* what) {
  set_error("%s", what);
  return code;
}

#define EVO_REQUIRE(cond, code, ...)        \
  do {                                      \
    if (!(cond)) {                          \
      evo::set_error(__VA_ARGS__);          \
      return (code);                        \
    }                                       \
  } while (0)

// After a kernel launch: report launch-configuration errors without synchronising.
inline int check_launch(const char* name) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) {
    set_error("launch of %s failed: %s", name, hipGetErrorString(e));
    return EVO_ERR_HIP;
  }
  return EVO_OK;
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

inline hipStream_t as_stream(void* s) { return reinterpret_cast<hipStream_t>(s); }

constexpr int kWave = 64;

}  // namespace evo
