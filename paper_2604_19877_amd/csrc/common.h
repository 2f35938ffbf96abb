// Internal helpers shared by the translation units of libsamixers (host side only).
#pragma once
#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdint>
#include <cstdio>

#include "samixers.h"

namespace sa {

// Records a formatted message for sa_last_error() and returns `code`.
sa_status fail(sa_status code, const char* fmt, ...);

inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

// Event bracketing of one kernel launch when profiling is enabled (see sa_prof_enable).
struct ProfScope {
  int kernel;
  hipStream_t stream;
  hipEvent_t start = nullptr, stop = nullptr;
  ProfScope(int kernel_id, hipStream_t s);
  ~ProfScope();
};

// Turns the sticky launch error (if any) into a status.
sa_status check_launch(const char* what);

}  // namespace sa

#define SA_REQUIRE(cond, code, ...)                   \
  do {                                                \
    if (!(cond)) return sa::fail((code), __VA_ARGS__); \
  } while (0)
