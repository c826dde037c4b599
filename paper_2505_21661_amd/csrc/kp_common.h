// Shared host-side helpers of libkperf (error reporting, HIP call checking).
#pragma once
#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdio>

#include "kperf.h"

namespace kp {

char* last_error_buf();
uint32_t rec_cost();  // the value of kp_set_rec_cost: goes into the header of every trace recorded from now on
constexpr int kLastErrorLen = 512;

inline kp_status fail(kp_status code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(last_error_buf(), kLastErrorLen, fmt, ap);
  va_end(ap);
  return code;
}

inline void clear_error() { last_error_buf()[0] = '\0'; }

#define KP_HIP_TRY(expr)                                                                   \
  do {                                                                                     \
    hipError_t kp_e_ = (expr);                                                             \
    if (kp_e_ != hipSuccess)                                                               \
      return ::kp::fail(KP_ERR_HIP, "%s failed: %s", #expr, hipGetErrorString(kp_e_));     \
  } while (0)

inline bool is_pow2(unsigned long long x) { return x && !(x & (x - 1)); }

}  // namespace kp
