// Internal helpers shared by the q8conv translation units (host side only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "q8conv.h"

#define Q8_REQUIRE(cond, code) \
  do {                         \
    if (!(cond)) return (code); \
  } while (0)

static inline int q8_launch_status() {
  return hipGetLastError() == hipSuccess ? Q8_OK : Q8_EHIP;
}

static inline bool q8_finite_pos(float q) { return q > 0.0f && q <= 3.402823466e38f; }

static inline bool q8_aligned(const void* p, size_t a) {
  return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0;
}
