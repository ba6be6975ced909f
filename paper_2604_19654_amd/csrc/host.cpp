// Error text, version, and the staging copy of dynamic experts' weights
// (paper Section 2.2 Phase 2 / Section 2.3: weights move on a copy engine, on a
// stream of their own, while the static experts compute).
#include <stdarg.h>
#include <string.h>
#include "common.h"

namespace feplb {
static thread_local char g_err[512] = "";
void set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
}
}  // namespace feplb

extern "C" const char* feplb_version(void) { return "feplb-mi355x 0.1 (gfx950)"; }
extern "C" const char* feplb_last_error(void) { return feplb::g_err; }

extern "C" size_t feplb_expert_bytes(int32_t d, int32_t f, int32_t elem_bytes) {
  if (d < 0 || f < 0 || elem_bytes < 0) return 0;
  return (size_t)3 * (size_t)d * (size_t)f * (size_t)elem_bytes;
}

extern "C" int32_t feplb_stage_weights(void* slot, const void* src, size_t bytes,
                                       void* side_stream, void* done_event) {
  FEPLB_REQUIRE(slot && src, FEPLB_EINVAL, "stage_weights: null buffer");
  if (bytes)
    FEPLB_HIP(hipMemcpyAsync(slot, src, bytes, hipMemcpyDefault, (hipStream_t)side_stream));
  if (done_event)
    FEPLB_HIP(hipEventRecord((hipEvent_t)done_event, (hipStream_t)side_stream));
  return FEPLB_OK;
}

extern "C" int32_t feplb_stream_wait(void* stream, void* event) {
  FEPLB_REQUIRE(event, FEPLB_EINVAL, "stream_wait: null event");
  FEPLB_HIP(hipStreamWaitEvent((hipStream_t)stream, (hipEvent_t)event, 0));
  return FEPLB_OK;
}
