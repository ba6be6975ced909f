// Shared host-side helpers of the library: error reporting and argument checks.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include "feplb.h"

namespace feplb {

void set_error(const char* fmt, ...);

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// backward-pass launchers (ffn_backward.hip), used by feplb_grouped_ffn_backward
hipError_t launch_wgrad(const void* P, int ldp, int M, const void* Q, int ldq, int N, const int* offsets,
                        const int* order, int g_begin, int n_groups, int R_cap, void* const* c0, void* const* c1,
                        int n_split, int ldc, bool accumulate, hipStream_t s);
hipError_t launch_wgrad_order(const int* offsets, int g_begin, int n_groups, int R_cap, int* order, hipStream_t s);
hipError_t launch_transpose(const void* const* src, int g_begin, int n_groups, int rows, int cols, void* dst,
                            size_t group_stride, hipStream_t s);

}  // namespace feplb

#define FEPLB_FAIL(code, ...)        \
  do {                               \
    feplb::set_error(__VA_ARGS__);   \
    return (code);                   \
  } while (0)

#define FEPLB_REQUIRE(cond, code, ...) \
  do {                                 \
    if (!(cond)) FEPLB_FAIL(code, __VA_ARGS__); \
  } while (0)

#define FEPLB_HIP(expr)                                                         \
  do {                                                                          \
    hipError_t e__ = (expr);                                                    \
    if (e__ != hipSuccess)                                                      \
      FEPLB_FAIL(FEPLB_EHIP, "%s: %s", #expr, hipGetErrorString(e__));          \
  } while (0)

#define FEPLB_LAUNCH_CHECK(name)                                                \
  do {                                                                          \
    hipError_t e__ = hipGetLastError();                                         \
    if (e__ != hipSuccess)                                                      \
      FEPLB_FAIL(FEPLB_EHIP, "launch of %s: %s", name, hipGetErrorString(e__)); \
  } while (0)
