// Shared host-side helpers of the library: status codes, error text, launch checks.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>

#include "../../include/evict.h"

namespace evict {

void set_error(const char* fmt, ...);

#define EVICT_HIP_CHECK(expr)                                                          \
  do {                                                                                 \
    hipError_t e_ = (expr);                                                            \
    if (e_ != hipSuccess) {                                                            \
      evict::set_error("%s failed: %s (%s:%d)", #expr, hipGetErrorString(e_), __FILE__, __LINE__); \
      return EVICT_E_HIP;                                                              \
    }                                                                                  \
  } while (0)

#define EVICT_REQUIRE(cond, code, ...)   \
  do {                                   \
    if (!(cond)) {                       \
      evict::set_error(__VA_ARGS__);     \
      return (code);                     \
    }                                    \
  } while (0)

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

inline int launch_status(const char* what) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) {
    set_error("launch of %s failed: %s", what, hipGetErrorString(e));
    return EVICT_E_HIP;
  }
  return EVICT_OK;
}

// status bits written by kernels into the context's device status word
enum : int { ST_BAD_PARENT = 1, ST_BAD_EXPERT = 2, ST_BAD_CTXLEN = 4, ST_BAD_TREE_SIZE = 8, ST_BAD_PAGE = 16,
              ST_PATH_TRUNCATED = 32, ST_BAD_PROB = 64, ST_BAD_COST = 128 };

}  // namespace evict
